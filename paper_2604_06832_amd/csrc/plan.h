// Work partition of the persistent forward kernels and the argument block they share (host and device).
//
// Every workgroup owns a fixed (row range, K range) slice of every weight matrix; the functions here say which, and
// where each 1-KiB fragment of it sits in that wavefront's weight stream.  The host uses them to size and pack the
// stream, the kernels to walk it.
#pragma once
#include "common.h"

namespace bd {

constexpr int kMaxKW = 16;   // k-steps (of 32) one wavefront covers in a GEMM phase
constexpr int kT = 2;        // 16-row tiles a wavefront accumulates side by side (one chunk of its stream)
constexpr int kBarGroup = 16;
constexpr int kSpinLimit = 1 << 19;

enum { PH_QKV = 0, PH_O = 1, PH_GU = 2, PH_DOWN = 3, PH_LM = 4, PH_COUNT = 5, PH_END = 6 };

struct PhasePlan {
  int N;        // output rows of the phase (after fusing / interleaving); a multiple of 16
  int KS;       // k-steps
  int ksplit;   // workgroups that share an output row range and split K
  int RW;       // rows of the largest row range (a multiple of 16)
  int kgran;    // k-steps per unit of the K split: 1 (bf16 weights) or 2 (fp8 weights: a 1-KiB fragment of 16 rows
                // x 64 k holds two k-steps, so wavefront ranges start and end on even k-steps)
  int wbytes;   // bytes per streamed weight element: 2 (bf16) or 1 (e4m3)
};
// Row ranges are whole 16-row tiles, spread over the nwg/ksplit row groups as evenly as whole tiles allow
// (group g holds tiles [T*g/G, T*(g+1)/G)).  So every weight fragment of the stream is a full 1 KiB.
__host__ __device__ inline int tile0_of_group(int T, int G, int g) { return (int)((long long)T * g / G); }
__host__ __device__ inline int group_of_tile(int T, int G, int tile) { return (int)((((long long)tile + 1) * G - 1) / T); }

struct MegaPlan {
  int nwg, L, H, QD, KVD, F, V, D, n_q, n_kv;
  PhasePlan ph[PH_COUNT];
  long long wave_stride;   // 16-byte units reserved per wavefront in the weight stream
  int xcd_gu;              // > 0: number of XCDs; the row groups of the gate/up phase are dealt out so that the
                           // workgroups of XCD x (workgroup id mod xcd_gu) produce exactly the features that K slice x of
                           // the down projection (also held by the workgroups of XCD x) consumes
  int gu_cut;              // 1: K slices of unequal size (e4m3 contexts), see phase_tile0_t
  int single;              // bit p set: phase p (QKV, O) has at most one tile per workgroup and no K split; tile j then
                           // belongs to workgroup j (QKV) or nwg-1-j (O).  With consecutive workgroups on consecutive
                           // XCDs this spreads each phase's tiles evenly over the XCDs and stacks both on as few
                           // workgroups as possible; the even spread of T < nwg tiles over nwg groups would put the
                           // tiles of both phases on the same (odd) workgroups, i.e. on half of the XCDs
};
__host__ __device__ inline bool phase_single(const MegaPlan& P, int p) { return ((P.single >> p) & 1) != 0; }
// Tiles of a phase's row groups.  With xcd_gu the gate/up tiles belong to the XCD whose K slice of the down
// projection they feed.  For slices of equal size (bf16 weights: required for xcd_gu) that is the plain even
// spread; with e4m3 weights the slices are whole units of two k-steps and differ by one unit, so the gate/up tiles
// are first cut where the slices are cut (a K unit of kgran k-steps = 4*kgran tiles) and each XCD's share is spread
// over its workgroups (gu_cut).  CUT is a compile-time switch so that the bf16 kernels carry none of this.
__host__ __device__ inline int gu_slice_tile0(const MegaPlan& P, int x) {
  const PhasePlan& d = P.ph[PH_DOWN];
  const int KU = (d.KS + d.kgran - 1) / d.kgran;
  return min((int)((long long)KU * x / P.xcd_gu) * 4 * d.kgran, P.ph[PH_GU].N >> 4);
}
template <bool CUT>
__host__ __device__ inline int phase_tile0_t(const MegaPlan& P, int p, int ng) {
  const PhasePlan& ph = P.ph[p];
  const int T = ph.N >> 4, G = P.nwg / ph.ksplit;
  if constexpr (CUT) {
    if (p == PH_GU && P.gu_cut) {
      if (ng >= G) return T;
      const int per = G / P.xcd_gu, x = ng / per;
      const int b0 = gu_slice_tile0(P, x), b1 = gu_slice_tile0(P, x + 1);
      return b0 + tile0_of_group(b1 - b0, per, ng % per);
    }
  }
  if (phase_single(P, p)) return min(ng, T);
  return tile0_of_group(T, G, ng);
}
__host__ __device__ inline int phase_tile0(const MegaPlan& P, int p, int ng) {
  return P.gu_cut ? phase_tile0_t<true>(P, p, ng) : phase_tile0_t<false>(P, p, ng);
}
__host__ __device__ inline int phase_group_of_tile(const MegaPlan& P, int p, int tile) {
  const PhasePlan& ph = P.ph[p];
  const int T = ph.N >> 4, G = P.nwg / ph.ksplit;
  if (p == PH_GU && P.gu_cut) {
    const int per = G / P.xcd_gu;
    int x = 0;
    while (x + 1 < P.xcd_gu && gu_slice_tile0(P, x + 1) <= tile) ++x;
    const int b0 = gu_slice_tile0(P, x), b1 = gu_slice_tile0(P, x + 1);
    return x * per + group_of_tile(b1 - b0, per, tile - b0);
  }
  if (phase_single(P, p)) return tile;
  return group_of_tile(T, G, tile);
}
// Row group of workgroup `wg` in phase p, and the inverse.
__host__ __device__ inline int row_group_of_wg(const MegaPlan& P, int p, int wg) {
  if (p == PH_GU && P.xcd_gu > 0) return (wg % P.xcd_gu) * (P.nwg / P.xcd_gu) + wg / P.xcd_gu;
  if (phase_single(P, p)) return p == PH_O ? P.nwg - 1 - wg : wg;
  return wg / P.ph[p].ksplit;
}
__host__ __device__ inline int wg_of_row_group(const MegaPlan& P, int p, int ng, int kg) {
  if (p == PH_GU && P.xcd_gu > 0) return (ng % (P.nwg / P.xcd_gu)) * P.xcd_gu + ng / (P.nwg / P.xcd_gu);
  if (phase_single(P, p)) return p == PH_O ? P.nwg - 1 - ng : ng;
  return ng * P.ph[p].ksplit + kg;
}

struct WavePhase { int rows, row0, ng, kg, w0, KW; };

// 16-row tiles per row range of a phase, and (row range, tile) pairs of the whole phase
__host__ __device__ inline int phase_tpg(const PhasePlan& ph) { return (ph.RW + 15) >> 4; }
__host__ __device__ inline int phase_tile_slots(const MegaPlan& P, int p) {
  return (P.nwg / P.ph[p].ksplit) * phase_tpg(P.ph[p]);
}

template <bool CUT>
__host__ __device__ inline WavePhase wave_phase_t(const MegaPlan& P, int p, int wg, int w) {
  const PhasePlan& ph = P.ph[p];
  WavePhase r;
  const int ng = row_group_of_wg(P, p, wg);
  r.ng = ng;
  r.kg = wg % ph.ksplit;
  {
    const int t0 = phase_tile0_t<CUT>(P, p, ng), t1 = phase_tile0_t<CUT>(P, p, ng + 1);
    r.row0 = t0 << 4;
    r.rows = (t1 - t0) << 4;
  }
  // the K split works on units of kgran k-steps (the last unit may reach past KS: zero weights, zero activations)
  const int KU = (ph.KS + ph.kgran - 1) / ph.kgran;
  const int k0 = (int)((long long)KU * r.kg / ph.ksplit), k1 = (int)((long long)KU * (r.kg + 1) / ph.ksplit);
  const int len = k1 - k0;
  const int u0 = k0 + len * w / kWavesPerWG, u1 = k0 + len * (w + 1) / kWavesPerWG;
  r.w0 = u0 * ph.kgran;
  r.KW = (u1 - u0) * ph.kgran;
  return r;
}
__host__ __device__ inline WavePhase wave_phase(const MegaPlan& P, int p, int wg, int w) {
  return P.gu_cut ? wave_phase_t<true>(P, p, wg, w) : wave_phase_t<false>(P, p, wg, w);
}
// 16-byte units one wavefront streams in a phase: per row and k-step 32 weights of wbytes each
__host__ __device__ inline long long wave_phase_units(const PhasePlan& ph, const WavePhase& wp) {
  return (long long)wp.rows * 2 * ph.wbytes * wp.KW;
}
template <bool CUT>
__host__ __device__ inline long long wave_layer_units_t(const MegaPlan& P, int wg, int w) {
  long long s = 0;
  for (int p = 0; p < PH_LM; ++p) s += wave_phase_units(P.ph[p], wave_phase_t<CUT>(P, p, wg, w));
  return s;
}
__host__ __device__ inline long long wave_layer_units(const MegaPlan& P, int wg, int w) {
  return P.gu_cut ? wave_layer_units_t<true>(P, wg, w) : wave_layer_units_t<false>(P, wg, w);
}
// Position (16-byte units from the wavefront's phase start) of row `lr` (local to the row range),
// k-step `ksl` (local to the wavefront), k-quarter kq: tiles of 16 rows go in chunks of two.
__host__ __device__ inline long long stream_pos(int rows, int KW, int lr, int ksl, int kq) {
  const int tile = lr >> 4, i = lr & 15, c = tile >> 1, t = tile & 1;
  const int n_tiles = (rows + 15) >> 4;
  const int R0 = min(16, rows - 32 * c);
  const int R1 = (2 * c + 1 < n_tiles) ? min(16, rows - 32 * c - 16) : 0;
  const int R = t ? R1 : R0;
  return (long long)c * 32 * 4 * KW + (long long)ksl * (R0 + R1) * 4 + (t ? R0 * 4 : 0) + kq * R + i;
}

struct MegaArgs {
  MegaPlan P;
  const bf16x8* wstream;
  DevState* st;
  unsigned* bar;              // barrier words (see grid_barrier)
  unsigned bar_epoch;         // epoch of the last barrier of the previous forward
  int M, MT, mode, want_lm;
  // activations (all write-once per forward)
  float* xv;                  // [2L+1][Mp][H] residual stream versions (fp32: the accumulation chain)
  u16* xb;                    // [2L+1] the same versions rounded to bf16 in packed activation order (K = H): what
                              // the norm-on-load GEMM phases read
  size_t xb_elems;
  float* ssq;                 // [2L+1][parts][Mp] partial sums of squares of each version
  int ssq_parts;              // stride (parts) per version; version 0 has one part, odd versions one per
                              // tile slot of the O phase, even versions one per tile slot of the DOWN phase
  int Mp;
  const float* gains;         // [2L+1][H]: attn_norm l, ffn_norm l, ..., final_norm
  int skippable;              // this launch belongs to a step that does nothing once the block is complete (DevState::skip)
  int local_gu;               // the gate/up -> down hand-over stays inside each XCD (stream_fwd.h): plain stores, XCD barrier
  const int* kv_pages;        // page of every 32-key block of the cache (null: contiguous)
  int no_weights;             // measurement only: the producers request nothing (the consumers multiply what the ring held)
  int attn_local;             // the attention phase stays inside each XCD (stream_fwd.h): partials in the XCD's L2, XCD barrier
  int n_xcd;                  // XCDs (8) when workgroup b runs on XCD b mod n_xcd, else 0
  unsigned* xbar;             // [xcd][32 words] arrival counters of the XCD barriers
  unsigned xbar_epoch;        // XCD barriers run before this launch
  int fp8;                    // the decoder linears are e4m3 codes with one scale per output row: the scale multiplies
                              // the accumulators, and the norm gains (which cannot be folded into the codes) multiply
                              // the bf16 copies of the residual versions that feed them
  const float* wscale;        // [L][wscale_layer] scales in phase-row order: QKV | O | gate/up | down
  int wscale_layer;
  int wscale_off[4];
  float rms_eps;
  const float2* rope;         // [Mp][D/2]
  u16* Q;                     // [L][Mp][n_q][D]  (dims in rotary-pair order)
  u16* Kc; u16* Vc;           // packed caches, [L][n_kv][max_kb] blocks
  size_t kv_layer_elems;
  int max_kb;
  u16* ap;                    // [L] packed attention output (K = QD)
  size_t ap_elems;
  u16* act;                   // [L] packed SwiGLU output (K = F)
  size_t act_elems;
  float* wsD;                 // [L][ksplit][tiles][MT][64] f32x4 partials of the down projection
  size_t wsD_layer_floats;
  unsigned* cntD;             // [L][H/16] arrival counters (zeroed by the prologue kernel)
  // attention
  float* pO; float* pm; float* pl;   // per layer partials
  size_t pO_layer_floats, pml_layer_floats;
  unsigned* cntA;             // [L][groups]
  int attn_max_chunks;
  float scale_log2e;
  // LM head
  float* lm_max; int* lm_idx; float* lm_sum;   // [nwg][Mp]
  float* logits;
  int* row_cand; float* row_conf;
  unsigned long long* trace;  // optional [nwg][10L+4] timestamps of phase boundaries (nullptr = off)
  unsigned long long* trace2; // optional [nwg][64] timestamps inside the GEMM phases of layer 1
};

}  // namespace bd
