// Shared device-side types and helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned short u16;

constexpr int kWave = 64;
constexpr int kWGThreads = 256;          // every kernel here runs 4 wavefronts per workgroup
constexpr int kWavesPerWG = 4;

// ---- operand layouts -----------------------------------------------------------------------------
// All matrix operands live in HBM in the order the 16x16x32 bf16 MFMA consumes them, so that one
// wavefront's operand load is one contiguous, 16-byte-per-lane, 1 KiB read.
//
//  A/B fragment of a [16 rows] x [32 k] tile: lane l holds row (l & 15), k = 8*(l >> 4) .. +7.
//  C/D fragment of a [16 x 16] tile (4 fp32 per lane): lane l holds column (l & 15),
//  rows 4*(l >> 4) .. +3.
//
//  Packed weight  W[N][K] (N % 16 == 0):  tile (nt, ks) at ((nt*KS + ks)*64 + lane)*8 + e
//       = W[nt*16 + (lane & 15)][ks*32 + 8*(lane >> 4) + e],   KS = ceil(K/32), zero beyond K.
//  Packed activation X[M][K] (MT = ceil(M/16)): tile (ks, mt) at ((ks*MT + mt)*64 + lane)*8 + e
//       = X[mt*16 + (lane & 15)][ks*32 + 8*(lane >> 4) + e].
__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

__device__ inline u16 f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);     // round to nearest even (inputs here are finite)
  return (u16)(u >> 16);
}
__device__ inline float bf16_bits_to_f32(u16 b) { return __uint_as_float(((uint32_t)b) << 16); }

// Index of element (m, k) inside a packed activation with MT row tiles.
__device__ inline size_t xp_index(int m, int k, int MT) {
  int ks = k >> 5, kq = (k >> 3) & 3, e = k & 7;
  int mt = m >> 4, lane = kq * 16 + (m & 15);
  return (((size_t)ks * MT + mt) * 64 + lane) * 8 + e;
}

// ---- packed cache layouts (per layer, per kv head; key blocks of 32 keys) --------------------------
// K: block kb, half t (0/1), d-step ds (32 dims):  lane l holds key kb*32 + 8*(i/4) + 4*t + (i%4) with
//    i = l & 15, dims ds*32 + 8*(l>>4) .. +7.            index ((kb*2 + t)*DS + ds)*64 + l   (bf16x8)
// V: block kb, d-tile dt (16 dims): lane l holds dim dt*16 + (l & 15), keys kb*32 + 8*(l>>4) .. +7.
//                                                        index (kb*DT + dt)*64 + l           (bf16x8)
// The K cache stores the 32 keys of a block in the row order that makes the two S^T accumulator tiles of a lane
// (S^T[key, col] = K[key, :] . Q[col, :]) line up with the k-order of the P fragment of O^T = V^T . P^T.
__device__ inline size_t kp_index(int key, int d, int DS) {   // element index of K[key][d]
  const int kb = key >> 5, kk = key & 31;
  const int g = kk >> 3, e = kk & 7, t = e >> 2, r = e & 3, i = 4 * g + r;
  const int ds = d >> 5, kq = (d >> 3) & 3;
  return ((((size_t)kb * 2 + t) * DS + ds) * 64 + kq * 16 + i) * 8 + (d & 7);
}
__device__ inline size_t vp_index(int key, int d, int DT) {   // element index of V[key][d]
  const int kb = key >> 5, kk = key & 31;
  const int g = kk >> 3, e = kk & 7;
  return ((((size_t)kb * DT + (d >> 4)) * 64) + g * 16 + (d & 15)) * 8 + e;
}

// Paged cache: the 32-key blocks of a kv head are pages; `pages` maps the block a position falls in (position / 32) to the
// page that holds it (the same page for every layer and kv head).  A null table is the identity.
__device__ inline int page_of_block(const int* pages, int kb) { return pages != nullptr ? pages[kb] : kb; }
__device__ inline int paged_key(const int* pages, int key) { return (page_of_block(pages, key >> 5) << 5) | (key & 31); }

constexpr float kNegBig = -1.0e30f;

// Merge two (max, argmax, sum of exp(. - max)) triples; equal maxima keep the lower index.
// A triple with s == 0 is the empty set (its max is -inf) and merges as the identity.
__device__ inline void stat_merge(float& m, int& i, float& s, float m2, int i2, float s2) {
  if (s2 == 0.f) return;
  if (s == 0.f || m2 > m || (m2 == m && i2 < i)) {
    s = s * __expf(m - m2) + s2;
    m = m2;
    i = i2;
  } else {
    s = s + s2 * __expf(m2 - m);
  }
}

// Chunk geometry of the key-split attention: n_kb key blocks are cut into chunks of chunk_len blocks.
__device__ inline void attn_chunks(int n_keys, int max_chunks, int& n_kb, int& chunk_len, int& n_chunks) {
  n_kb = (n_keys + 31) >> 5;
  chunk_len = (n_kb + max_chunks - 1) / max_chunks;
  if (chunk_len < kWavesPerWG) chunk_len = kWavesPerWG;
  n_chunks = (n_kb + chunk_len - 1) / chunk_len;
}

// In-block visibility of the block's key jb (0-based index inside the block) for the block's query row `row`
// (Sec. 3.3 mask rules; Alg. 1 draft / verify masks; Alg. 2 quadratic mask).  mode 0: all visible; 1: causal;
// 2 + (B << 8): B groups of B+1 rows, a group's first row sees the first rows of the groups up to its own, every other
// row sees the rows of its own group.  (Keys of the committed prefix are visible to every row.)
// QUAD is a compile-time switch: the kernels of ordinary forwards are built without the quadratic rule (its index
// arithmetic costs registers in every phase of the persistent kernels), the quadratic step runs its own instantiations.
template <bool QUAD>
__device__ inline bool block_key_visible(int mode, int row, int jb) {
  if constexpr (!QUAD) {
    return mode == 0 || jb <= row;
  } else {
    const int W = (mode >> 8) + 1;
    const int gi = row / W, gj = row - gi * W, ki = jb / W, kj = jb - ki * W;
    return gj == 0 ? (kj == 0 && ki <= gi) : ki == gi;
  }
}

// State that lives on the device so that replayed launch sequences need no new kernel arguments.
struct DevState {
  int n;             // committed context length
  int seeded;        // 1 if the current denoise call revealed position 0 from the carry
  int carry_cand;    // prediction for position n
  float carry_conf;
  int error;         // sticky device-side error flag (bounded waits)
  int skip;          // bd_decode_block: the current block has no masked position left; its remaining steps do nothing
  int steps;         // bd_decode_block: denoising forwards that really ran for the current block
};

}  // namespace bd
