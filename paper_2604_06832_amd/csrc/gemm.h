// Skinny-M weight-streaming GEMM  Y[M<=64, N] = X[M, K] * W[N, K]^T  on the 16x16x32 bf16 MFMA.
//
// The weights are >95% of the bytes a decode forward moves, each read exactly once, so the kernel is
// a streaming reader: every wavefront pulls 1 KiB packed weight tiles straight from HBM into
// registers (16 B per lane, non-temporal), multiplies them against activation fragments that come
// from L2, and the four wavefronts of a workgroup split the K range and reduce through LDS.
#pragma once
#include "common.h"

namespace bd {

enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_LMHEAD = 2 };

struct GemmArgs {
  const bf16x8* Wp;     // packed weights, n_tiles x KS tiles
  const bf16x8* Xp;     // packed activations, KS x MT tiles
  int n_tiles;          // N / 16
  int KS;               // ceil(K / 32)
  int ksplit;           // K split across workgroups (EPI_PARTIAL only; 1 otherwise)
  int M;                // valid rows
  int N;
  float* partial;       // EPI_PARTIAL: [ksplit][MT*16][N] fp32
  u16* act_out;         // EPI_SWIGLU : packed bf16 activation [M][N/2] with MT row tiles
  float* lm_max;        // EPI_LMHEAD : per-workgroup row statistics [gridDim.x][MT*16]
  int* lm_idx;
  float* lm_sum;
  float* logits;        // EPI_LMHEAD : optional fp32 [M][N] dump (nullptr = off)
};

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

template <int MT, int NT, int U>
__device__ inline void gemm_accumulate(const bf16x8* __restrict__ Wp, const bf16x8* __restrict__ Xp, int KS,
                                       int tile0, int ks0, int ks1, int lane, f32x4 (&acc)[NT][MT]) {
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int ks = ks0; ks < ks1; ks += U) {
    bf16x8 wf[NT][U], xf[U][MT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = ks + u < ks1;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        wf[nt][u] = ok ? __builtin_nontemporal_load(Wp + ((size_t)(tile0 + nt) * KS + ks + u) * 64 + lane) : zero;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        xf[u][mt] = ok ? Xp[((size_t)(ks + u) * MT + mt) * 64 + lane] : zero;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nt][u], xf[u][mt], acc[nt][mt], 0, 0, 0);
  }
}

template <int MT, int NT, int EPI>
__global__ __launch_bounds__(kWGThreads) void gemm_kernel(GemmArgs a) {
  constexpr int U = (NT >= 4) ? 4 : 8;
  __shared__ f32x4 red[kWavesPerWG][NT * MT][kWave];
  // the row statistics re-use the reduction buffer once the item loop is over
  float (*s_m)[MT * 16] = reinterpret_cast<float (*)[MT * 16]>(&red[0][0][0]);
  int (*s_i)[MT * 16] = reinterpret_cast<int (*)[MT * 16]>(&red[1][0][0]);
  float (*s_s)[MT * 16] = reinterpret_cast<float (*)[MT * 16]>(&red[2][0][0]);

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const int n_groups = a.n_tiles / NT;
  const int n_items = n_groups * a.ksplit;

  // EPI_LMHEAD: running statistics of this lane's token column over the channels it has seen.
  float rmax[MT];
  int ridx[MT];
  float rsum[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) { rmax[mt] = -INFINITY; ridx[mt] = 0x7FFFFFFF; rsum[mt] = 0.f; }

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int ng = item / a.ksplit, sp = item - ng * a.ksplit;
    const int k0 = (int)((long)a.KS * sp / a.ksplit), k1 = (int)((long)a.KS * (sp + 1) / a.ksplit);
    const int len = k1 - k0;
    const int w0 = k0 + len * wave / kWavesPerWG, w1 = k0 + len * (wave + 1) / kWavesPerWG;

    f32x4 acc[NT][MT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    gemm_accumulate<MT, NT, U>(a.Wp, a.Xp, a.KS, ng * NT, w0, w1, lane, acc);

#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) red[wave][nt * MT + mt][lane] = acc[nt][mt];
    __syncthreads();

    if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
      for (int idx = 0; idx < NT * MT; ++idx) {
        if ((idx & 3) != wave) continue;
        const int nt = idx / MT, mt = idx % MT;
        f32x4 v = red[0][idx][lane];
        v += red[1][idx][lane];
        v += red[2][idx][lane];
        v += red[3][idx][lane];
        const int m = mt * 16 + col;
        const int c = (ng * NT + nt) * 16 + 4 * g;
        if (m < a.M)
          *reinterpret_cast<f32x4*>(a.partial + ((size_t)sp * (MT * 16) + m) * a.N + c) = v;
      }
    } else if constexpr (EPI == EPI_SWIGLU) {
      // tiles come in (gate, up) pairs of the same 16 channels
#pragma unroll
      for (int p = 0; p < (NT / 2) * MT; ++p) {
        if ((p & 3) != wave) continue;
        const int pr = p / MT, mt = p % MT;
        const int ig = (2 * pr) * MT + mt, iu = (2 * pr + 1) * MT + mt;
        f32x4 gt = red[0][ig][lane], up = red[0][iu][lane];
        gt += red[1][ig][lane]; up += red[1][iu][lane];
        gt += red[2][ig][lane]; up += red[2][iu][lane];
        gt += red[3][ig][lane]; up += red[3][iu][lane];
        const int m = mt * 16 + col;
        const int f = ((ng * NT) / 2 + pr) * 16 + 4 * g;      // channel in [0, N/2)
        if (m < a.M) {
          u16 o[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float s = gt[r] / (1.f + __expf(-gt[r]));
            o[r] = f32_to_bf16_bits(s * up[r]);
          }
          uint2 pk;
          pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
          pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
          *reinterpret_cast<uint2*>(a.act_out + xp_index(m, f, MT)) = pk;
        }
      }
    } else {  // EPI_LMHEAD
#pragma unroll
      for (int idx = 0; idx < NT * MT; ++idx) {
        if ((idx & 3) != wave) continue;
        const int nt = idx / MT, mt = idx % MT;
        f32x4 v = red[0][idx][lane];
        v += red[1][idx][lane];
        v += red[2][idx][lane];
        v += red[3][idx][lane];
        const int m = mt * 16 + col;
        const int c = (ng * NT + nt) * 16 + 4 * g;
        if (a.logits != nullptr && m < a.M)
          *reinterpret_cast<f32x4*>(a.logits + (size_t)m * a.N + c) = v;
#pragma unroll
        for (int r = 0; r < 4; ++r) stat_merge(rmax[mt], ridx[mt], rsum[mt], v[r], c + r, 1.f);
      }
    }
    __syncthreads();
  }

  if constexpr (EPI == EPI_LMHEAD) {
    // fold the four lane groups that share a token column, then the four wavefronts
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int off = 16; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(rmax[mt], off);
        const int i2 = __shfl_xor(ridx[mt], off);
        const float s2 = __shfl_xor(rsum[mt], off);
        stat_merge(rmax[mt], ridx[mt], rsum[mt], m2, i2, s2);
      }
      if (g == 0) {
        s_m[wave][mt * 16 + col] = rmax[mt];
        s_i[wave][mt * 16 + col] = ridx[mt];
        s_s[wave][mt * 16 + col] = rsum[mt];
      }
    }
    __syncthreads();
    if (threadIdx.x < MT * 16) {
      const int t = threadIdx.x;
      float m = s_m[0][t];
      int i = s_i[0][t];
      float s = s_s[0][t];
      for (int w = 1; w < kWavesPerWG; ++w) stat_merge(m, i, s, s_m[w][t], s_i[w][t], s_s[w][t]);
      a.lm_max[(size_t)blockIdx.x * (MT * 16) + t] = m;
      a.lm_idx[(size_t)blockIdx.x * (MT * 16) + t] = i;
      a.lm_sum[(size_t)blockIdx.x * (MT * 16) + t] = s;
    }
  }
}

}  // namespace bd
