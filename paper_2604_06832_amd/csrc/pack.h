// Kernels that run outside the forward proper: block assembly (the prologue of every forward) and the packing of
// weight matrices into the per-wavefront streams.  Compiled into the host translation unit only.
#pragma once
#include "common.h"
#include "plan.h"
#include "prefill_args.h"

namespace bd {

// ---- prologue: block assembly (seed, embedding gather), first sum of squares, rotary table, counters ------------
struct PrologueArgs {
  float* x0; float* ssq0; int H, Mp;
  u16* xb0; int MT;
  const float* embeds; int n_embed; const int* ids; int off;
  int* seed_tokens; uint8_t* seed_mask;       // denoise only: position 0 takes the carry if still masked
  const uint8_t* mask; int mask_id; const u16* table; int vocab;
  DevState* st;
  float2* rope; int half; float theta;
  unsigned* counters; int n_counters;
  int skippable;                              // nothing to do once the block is complete (DevState::skip)
  int quad_W;                                 // > 0: rows are groups of quad_W tokens, row r sits at position n + r / W + r % W (Alg. 2)
  const float* gain0;                         // fp8 weights: gain of the first norm, applied to the bf16 copy (else nullptr)
};

__global__ __launch_bounds__(kWGThreads) void prologue_kernel(PrologueArgs a) {
  __shared__ float wsum[kWavesPerWG];
  __shared__ int s_id;
  const int r = blockIdx.x;
  if (a.skippable && a.st->skip) return;
  for (int i = blockIdx.x * kWGThreads + threadIdx.x; i < a.n_counters; i += gridDim.x * kWGThreads) a.counters[i] = 0u;
  {
    const double pos = (double)(a.st->n + (a.quad_W > 0 ? r / a.quad_W + r % a.quad_W : r));
    for (int i = threadIdx.x; i < a.half; i += kWGThreads) {
      const double inv = exp2(-log2((double)a.theta) * (double)i / (double)a.half);
      const double ang = pos * inv;
      a.rope[(size_t)r * a.half + i] = make_float2((float)cos(ang), (float)sin(ang));
    }
  }
  const int p = a.off + r;
  if (threadIdx.x == 0) {
    int id = -1;
    if (p >= a.n_embed) {
      const int j = p - a.n_embed;
      if (r == 0 && a.seed_mask != nullptr) {
        a.st->seeded = 0;
        if (a.seed_mask[0]) {
          a.seed_tokens[0] = a.st->carry_cand;
          a.seed_mask[0] = 0;
          a.st->seeded = 1;
        }
      }
      id = a.ids[j];
      if (a.mask != nullptr && a.mask[j]) id = a.mask_id;
      id = min(max(id, 0), a.vocab - 1);
    }
    s_id = id;
  }
  __syncthreads();
  const int id = s_id;
  float ss = 0.f;
  for (int c = threadIdx.x; c < a.H; c += kWGThreads) {
    const float v = id < 0 ? a.embeds[(size_t)p * a.H + c] : bf16_bits_to_f32(a.table[(size_t)id * a.H + c]);
    a.x0[(size_t)r * a.H + c] = v;
    a.xb0[xp_index(r, c, a.MT)] = f32_to_bf16_bits(a.gain0 != nullptr ? v * a.gain0[c] : v);
    ss += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) a.ssq0[r] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// ---- weight stream packing ----------------------------------------------------------------------------------
// One source matrix (row-major [n_rows][K], fp32 or bf16 bits) goes into the stream of phase `ph` of
// layer `layer`; `row_map` says where source row r sits among the phase's output rows:
//   0: row_base + r                       (plain)
//   1: rotary pairing inside heads of D   (Q and K: dim i -> 2i, dim i + D/2 -> 2i + 1)
//   2: row_base + 2*r                     (gate: even rows, up: odd rows with row_base = 1)
template <typename SrcT>
__global__ void pack_stream_kernel(const SrcT* __restrict__ src, int n_rows, int K, MegaPlan P, int ph, int layer,
                                   int row_base, int row_map, int D, const float* __restrict__ col_gain,
                                   u16* __restrict__ stream) {
  const int KS = P.ph[ph].KS;
  const size_t total = (size_t)n_rows * KS * 4;             // one thread per (row, k-step, k-quarter)
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int kq = idx & 3;
    const int ks = (int)((idx >> 2) % KS);
    const int rs = (int)(idx / ((size_t)KS * 4));
    int r;
    if (row_map == 1) {
      const int h = rs / D, d = rs % D, half = D >> 1;
      r = row_base + h * D + (d < half ? 2 * d : 2 * (d - half) + 1);
    } else if (row_map == 2) {
      r = row_base + 2 * rs;
    } else {
      r = row_base + rs;
    }
    const PhasePlan& pp = P.ph[ph];
    const int ng = phase_group_of_tile(P, ph, r >> 4);
    const int lr = r - (phase_tile0(P, ph, ng) << 4);
    // which K group / wavefront holds k-step ks
    int kg = 0;
    while ((int)((long long)pp.KS * (kg + 1) / pp.ksplit) <= ks) ++kg;
    const int wg = wg_of_row_group(P, ph, ng, kg);
    int w = 0;
    WavePhase wp = wave_phase(P, ph, wg, 0);
    while (ks >= wp.w0 + wp.KW) { ++w; wp = wave_phase(P, ph, wg, w); }
    long long pos = (long long)(wg * kWavesPerWG + w) * P.wave_stride;
    pos += (ph == PH_LM) ? (long long)P.L * wave_layer_units(P, wg, w) : (long long)layer * wave_layer_units(P, wg, w);
    for (int q = 0; q < ph && ph != PH_LM; ++q) pos += wave_phase_units(P.ph[q], wave_phase(P, q, wg, w));
    pos += stream_pos(wp.rows, wp.KW, lr, ks - wp.w0, kq);
    u16* dst = stream + (size_t)pos * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = ks * 32 + kq * 8 + e;
      u16 o = 0;
      if (k < K) {
        float f;
        if constexpr (sizeof(SrcT) == 4) f = ((const float*)src)[(size_t)rs * K + k];
        else f = bf16_bits_to_f32(((const u16*)src)[(size_t)rs * K + k]);
        if (col_gain != nullptr) f *= col_gain[k];        // gain of the RMSNorm that feeds this matrix
        o = f32_to_bf16_bits(f);
      }
      dst[e] = o;
    }
  }
}

// e4m3 codes of one matrix into the stream: a fragment is 16 rows x 64 k (two k-steps); lane (row i, k-quarter kq)
// holds 8 codes of the even k-step (k = 64j + 8kq ..) followed by 8 codes of the odd one (k = 64j + 32 + 8kq ..).
__global__ void pack_stream_fp8_kernel(const uint8_t* __restrict__ src, int n_rows, int K, MegaPlan P, int ph, int layer,
                                       int row_base, int row_map, int D, uint8_t* __restrict__ stream) {
  const PhasePlan& pp = P.ph[ph];
  const int KP = (pp.KS + 1) / 2;                            // k-step pairs
  const size_t total = (size_t)n_rows * KP * 4;              // one thread per (row, pair, k-quarter)
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int kq = idx & 3;
    const int kp = (int)((idx >> 2) % KP);
    const int rs = (int)(idx / ((size_t)KP * 4));
    int r;
    if (row_map == 1) {
      const int h = rs / D, d = rs % D, half = D >> 1;
      r = row_base + h * D + (d < half ? 2 * d : 2 * (d - half) + 1);
    } else if (row_map == 2) {
      r = row_base + 2 * rs;
    } else {
      r = row_base + rs;
    }
    const int ng = phase_group_of_tile(P, ph, r >> 4);
    const int lr = r - (phase_tile0(P, ph, ng) << 4);
    const int ks = 2 * kp;
    int kg = 0;
    while ((int)((long long)KP * (kg + 1) / pp.ksplit) <= kp) ++kg;
    const int wg = wg_of_row_group(P, ph, ng, kg);
    int w = 0;
    WavePhase wp = wave_phase(P, ph, wg, 0);
    while (ks >= wp.w0 + wp.KW) { ++w; wp = wave_phase(P, ph, wg, w); }
    long long pos = (long long)(wg * kWavesPerWG + w) * P.wave_stride + (long long)layer * wave_layer_units(P, wg, w);
    for (int q = 0; q < ph; ++q) pos += wave_phase_units(P.ph[q], wave_phase(P, q, wg, w));
    // fragment index inside the phase: chunks of two tiles, pairs in order, tiles side by side
    const int tile = lr >> 4, c = tile >> 1, t = tile & 1;
    const int n_tiles = wp.rows >> 4;
    const int nt = (2 * c + 1 < n_tiles) ? 2 : 1;
    const int KWP = wp.KW >> 1;
    const long long frag = (long long)c * 2 * KWP + (long long)((ks - wp.w0) >> 1) * nt + t;
    uint8_t* dst = stream + ((size_t)pos + (size_t)frag * 64 + kq * 16 + (lr & 15)) * 16;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int k = ks * 32 + (e >> 3) * 32 + kq * 8 + (e & 7);
      dst[e] = k < K ? src[(size_t)rs * K + k] : (uint8_t)0;
    }
  }
}

// Per-output-row scales of one fp8 matrix into phase-row order.
__global__ void scatter_scales_kernel(const float* __restrict__ src, int n_rows, int row_base, int row_map, int D,
                                      float* __restrict__ dst) {
  for (int rs = blockIdx.x * blockDim.x + threadIdx.x; rs < n_rows; rs += gridDim.x * blockDim.x) {
    int r;
    if (row_map == 1) {
      const int h = rs / D, d = rs % D, half = D >> 1;
      r = row_base + h * D + (d < half ? 2 * d : 2 * (d - half) + 1);
    } else if (row_map == 2) {
      r = row_base + 2 * rs;
    } else {
      r = row_base + rs;
    }
    dst[r] = src[rs];
  }
}

// Hand-over of rows of the large-M kernels' residual stream to the final norm + LM head of the decode path: the bf16
// copies of rows [0, M) of `xrows` become the last residual version (packed order of MT 16-row tiles, the rows that pad
// the last tile zero) and their sums of squares part 0 of that version's partial sums (the other parts zero; padding
// rows get a harmless 1).  One workgroup per row of the MT tiles.
__global__ __launch_bounds__(kPfThreads) void pf_rows_to_lm_kernel(const float* __restrict__ xrows, int H, int M, int MT,
                                                                   u16* __restrict__ xb, float* __restrict__ ssq, int parts,
                                                                   int Mp, const DevState* st) {
  __shared__ float part[kPfThreads / 64];
  if (st != nullptr && st->skip) return;
  const int m = blockIdx.x;
  float ss = 0.f;
  for (int c = threadIdx.x; c < H; c += kPfThreads) {
    const float v = m < M ? xrows[(size_t)m * H + c] : 0.f;
    ss += v * v;
    xb[xp_index(m, c, MT)] = f32_to_bf16_bits(v);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < kPfThreads / 64; ++w) t += part[w];
  for (int p = threadIdx.x; p < parts; p += kPfThreads) ssq[(size_t)p * Mp + m] = p == 0 ? (m < M ? t : 1.f) : 0.f;
}

// The decode kernels rely on the slots of the partial sums that no tile owns staying zero: clear what the hand-over
// wrote once the LM head has read it.
__global__ void pf_clear_ssq_kernel(float* __restrict__ ssq, int parts, int Mp, int rows, const DevState* st) {
  if (st != nullptr && st->skip) return;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < parts * rows; i += gridDim.x * blockDim.x)
    ssq[(size_t)(i / rows) * Mp + i % rows] = 0.f;
}

// One matrix into the tile-major fragment order of the prefill GEMMs (same row maps and column gains as the
// weight stream of the decode kernels).  One-byte sources are e4m3 codes: every code is a bf16 value, so the copy is
// exact; its row scales and the norm gains stay outside (accumulator epilogue, activation copy).
template <typename SrcT>
__global__ void pack_tiles_kernel(const SrcT* __restrict__ src, int n_rows, int K, int KS, int row_base, int row_map, int D,
                                  const float* __restrict__ col_gain, u16* __restrict__ dst) {
  const size_t total = (size_t)n_rows * KS * 4;             // one thread per (row, k-step, k-quarter)
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int kq = idx & 3;
    const int ks = (int)((idx >> 2) % KS);
    const int rs = (int)(idx / ((size_t)KS * 4));
    int r;
    if (row_map == 1) {
      const int h = rs / D, d = rs % D, half = D >> 1;
      r = row_base + h * D + (d < half ? 2 * d : 2 * (d - half) + 1);
    } else if (row_map == 2) {
      r = row_base + 2 * rs;
    } else {
      r = row_base + rs;
    }
    u16* o = dst + ((((size_t)(r >> 4) * KS + ks) * 64) + kq * 16 + (r & 15)) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = ks * 32 + kq * 8 + e;
      u16 v = 0;
      if (k < K) {
        float f;
        if constexpr (sizeof(SrcT) == 4) f = ((const float*)src)[(size_t)rs * K + k];
        else if constexpr (sizeof(SrcT) == 1) f = __builtin_amdgcn_cvt_f32_fp8((int)((const uint8_t*)src)[(size_t)rs * K + k], 0);
        else f = bf16_bits_to_f32(((const u16*)src)[(size_t)rs * K + k]);
        if (col_gain != nullptr) f *= col_gain[k];
        v = f32_to_bf16_bits(f);
      }
      o[e] = v;
    }
  }
}

}  // namespace bd
