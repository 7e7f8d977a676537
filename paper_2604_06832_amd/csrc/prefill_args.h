// Argument blocks of the large-M prefill kernels (prefill.h) and of the host call that runs one chunk through them.
#pragma once
#include "common.h"

namespace bd {

constexpr int kPfTokens = 128;        // tokens per workgroup tile (8 token tiles of 16)
constexpr int kPfThreads = 256;       // four wavefronts, 2 (rows) x 2 (tokens)
constexpr int kPfSplit = 4;           // K splits of the down projection over workgroups

struct PfGemmArgs {
  const bf16x8* w;        // fragments of this layer's phase, tile-major
  int NT, KS;             // 16-row tiles and k-steps of the phase
  const bf16x8* xin;      // packed activations of the chunk
  int MTc;                // token tiles of the chunk (any number: a workgroup's eight may reach past the end)
  int Mvalid;             // rows of the chunk; the rows that pad its last tile write no Q, K or V
  int RG, TG;             // workgroup grid: row groups x token groups
  const float* rs;        // [Mc] 1/rms of the rows of the residual stream (QKV, gate/up)
  const float* wscale;    // e4m3 weights: one scale per phase row, applied to the accumulators; else nullptr
  const float2* rope;     // [Mc][D/2] (QKV)
  float* x;               // [Mc][H] residual stream, updated in place (O, down)
  int SK;                 // K split over workgroups (direct kernel; 1 = none)
  float* part;            // SK > 1: [SK][Mc][H] partial products of the splits, added to x by the next norm kernel
  u16* q;                 // [Mc][n_q][D] (QKV)
  u16* Kc; u16* Vc;       // this layer's packed cache (QKV)
  int max_kb, n0;         // key blocks per kv head; position of the chunk's first row
  u16* act;               // packed SwiGLU output (gate/up)
  int H, QD, KVD, D, n_q;
  const int* pages;       // page of every 32-key block of the cache (null: contiguous)
  const DevState* st; int skippable;   // nothing to do once the block is complete (DevState::skip)
};

struct PfAttnArgs {
  const u16* q;           // [Mc][n_q][D], rotated, dims in rotary-pair order
  const u16* Kc; const u16* Vc;
  int max_kb, n0, Mc, n_q, n_kv;
  float scale_log2e;
  u16* out;               // packed attention output (K = n_q*D)
  int MTc;
  int mode;               // visibility among the chunk's own rows: BD_MODE_* (bits 8.. = B of a quadratic forward)
  int Mvalid;             // rows of the chunk: keys n0 + Mvalid .. do not exist
  const int* pages;       // page of every 32-key block of the cache (null: contiguous)
  int n_chunks;           // pf_attn_split_kernel: the key blocks of an item are dealt to this many workgroups (block kb to
                          // chunk kb mod n_chunks), each leaving an unnormalised partial in `part`; pf_attn_merge_kernel finishes
  float* part;            // [items][n_chunks] x (D/16 x 64 x 4 partial output + 64 maxima + 64 sums), fp32
  const DevState* st; int skippable;   // nothing to do once the block is complete (DevState::skip)
};
#ifndef BD_PF_ATTN_CHUNKS
#define BD_PF_ATTN_CHUNKS 4
#endif
#ifndef BD_PF_ATTN_TILES
#define BD_PF_ATTN_TILES 1
#endif
constexpr int kPfAttnChunks = BD_PF_ATTN_CHUNKS;   // key chunks per attention item in forwards of at most 64 rows
constexpr int kPfAttnTiles = BD_PF_ATTN_TILES;     // query tiles of a head that share a workgroup (and its key/value loads) there

// One chunk of rows through all layers (k_prefill.hip): plain pointers and sizes of the context.  The rows are prompt
// rows (embeds / ids from row `off`), or, with `block` set, the tokens of a decode block (ids[0..rows), masked rows
// taking the mask token, position 0 seeded from the carry like the prologue of the decode kernels does).
struct PfChunk {
  int rows, off;                  // rows of the chunk; prompt row of its first row
  int n0;                         // cache position of its first row
  const float* embeds; int n_embed; const int32_t* ids;
  bool block;                     // rows are a decode block
  int32_t* seed_tokens; uint8_t* seed_mask; const uint8_t* mask;
  int mode;                       // BD_MODE_* among the chunk's rows (prompt chunks: causal)
  int quad_W;                     // > 0: rows are groups of quad_W tokens, row r at position n + r / W + r % W (Alg. 2)
  int skippable;
  const u16* table; int vocab, mask_id;
  int L, H, QD, KVD, NQKV, F, D, n_q, n_kv, max_kb;
  float rms_eps, rope_theta;
  DevState* st;                   // (a block forward writes its seed flag)
  bool fp8, staged;
  const float* gains; const float* wscale; int wscale_layer; int wscale_off[4];
  const u16* w; size_t layer_elems; size_t w_off[4];
  u16* Kc; u16* Vc; size_t kv_layer_elems; const int* pages;
  float* x; u16* xb; float* rs; float2* rope; u16* q; u16* ap; u16* act; float* part;
  float* apart;                   // attention partials of forwards of at most 64 rows
};

}  // namespace bd
