// Block-causal grouped-query attention over the packed KV cache (split over keys, combined after).
//
// Visibility (training mask rules of Sec. 3.3; draft / verify masks of Alg. 1): every cached prefix
// key is visible to every block row; an in-block key j is visible to block row i always
// (BD_MODE_BIDIR) or iff j <= i (BD_MODE_CAUSAL).  The block's own K/V sit in the cache at
// positions n .. n+M-1 (written by the QKV epilogue), so one key loop covers prefix and block.
//
// Work decomposition: a workgroup item is (kv head, group of JT query-column tiles, key chunk);
// a query column is a (query head of that kv head, block row) pair, 16 columns per tile.  The four
// wavefronts of the workgroup take the chunk's 32-key blocks round-robin, each keeps an online
// softmax (running max, running sum, unnormalised output) per column in registers, and the four are
// merged through LDS into one partial per item.  A second kernel merges the chunks.
//
// MFMA formulation (16x16x32 bf16, transposed so that the softmax statistics of a column stay in
// the lanes that own that column):
//   S^T[key, col] = K[key, :] . Q[col, :]        A = K fragment, B = Q fragment
//   O^T[d,   col] = V^T[d, key] . P^T[key, col]   A = V fragment, B = P fragment (bf16 of exp2(..))
// The K cache stores the 32 keys of a block in the row order that makes the two S^T accumulator
// tiles of a lane line up with the k-order of the P fragment (see kp_index).
#pragma once
#include "common.h"

namespace bd {

struct AttnArgs {
  const u16* Q;            // [MT*16][n_q][D] bf16, rotary applied
  const bf16x8* Kc;        // this layer's packed K cache: [n_kv][max_kb] blocks
  const bf16x8* Vc;
  const DevState* st;
  int M, MT, n_q, n_kv, mode, max_kb;
  int max_chunks;          // upper bound on chunks per (kv head, column group)
  float scale_log2e;       // log2(e) / sqrt(head_dim)
  float* pO;               // partial outputs  [item][DT*JT][64] f32x4
  float* pm;               // partial maxima   [item][JT*16]   (log2 domain)
  float* pl;               // partial sums     [item][JT*16]
  u16* out;                // combine: packed bf16 activation [M][n_q*D] with MT row tiles
};

template <int D, int JT>
__global__ __launch_bounds__(kWGThreads) void attn_partial_kernel(AttnArgs a) {
  constexpr int DS = D / 32, DT = D / 16;
  __shared__ f32x4 sO[DT * JT][kWave];
  __shared__ float sm[kWavesPerWG][JT * 16];
  __shared__ float sl[kWavesPerWG][JT * 16];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const int n = a.st->n;
  const int G = a.n_q / a.n_kv;
  const int Mp = a.MT * 16;
  const int n_jg = (G * a.MT) / JT;
  int n_kb, chunk_len, n_chunks;
  attn_chunks(n + a.M, a.max_chunks, n_kb, chunk_len, n_chunks);
  const int n_items = a.n_kv * n_jg * n_chunks;
  const size_t kv_block = (size_t)32 * D / 8;           // bf16x8 units per key block

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int chunk = item % n_chunks;
    const int jg = (item / n_chunks) % n_jg;
    const int kvh = item / (n_chunks * n_jg);
    const bf16x8* Kh = a.Kc + (size_t)kvh * a.max_kb * kv_block;
    const bf16x8* Vh = a.Vc + (size_t)kvh * a.max_kb * kv_block;

    // query fragments of this lane's columns
    bf16x8 qf[JT][DS];
    int row[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      const int c = (jg * JT + jt) * 16 + col;
      const int hq = c / Mp, m = c - hq * Mp;
      row[jt] = m;
      const u16* qp = a.Q + ((size_t)m * a.n_q + kvh * G + hq) * D + 8 * g;
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) qf[jt][ds] = *reinterpret_cast<const bf16x8*>(qp + ds * 32);
    }

    f32x4 O[DT][JT];
    float mrun[JT], lrun[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      mrun[jt] = kNegBig;
      lrun[jt] = 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) O[dt][jt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int kb_end = min(n_kb, (chunk + 1) * chunk_len);
    for (int kb = chunk * chunk_len + wave; kb < kb_end; kb += kWavesPerWG) {
      bf16x8 kf[2][DS], vf[DT];
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) kf[t][ds] = Kh[(((size_t)kb * 2 + t) * DS + ds) * 64 + lane];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) vf[dt] = Vh[((size_t)kb * DT + dt) * 64 + lane];

      const bool need_mask = (kb * 32 + 31) >= n;       // block touches in-block keys or the tail
      bf16x8 pf[JT];
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
        f32x4 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ds = 0; ds < DS; ++ds)
            s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][ds], qf[jt][ds], s[t], 0, 0, 0);
        }
        // this lane now holds keys kb*32 + 8*g + e, e = 4*t + r, of column (jt, col)
        float v[8];
        bool vis[8];
        float cmax = kNegBig;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          v[e] = s[e >> 2][e & 3] * a.scale_log2e;
          vis[e] = true;
          if (need_mask) {
            const int key = kb * 32 + 8 * g + e;
            const int jb = key - n;                     // index inside the block, if >= 0
            vis[e] = (jb < 0) || (jb < a.M && block_key_visible<false>(a.mode, row[jt], jb));
          }
          if (vis[e]) cmax = fmaxf(cmax, v[e]);
        }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
        const float mnew = fmaxf(mrun[jt], cmax);
        const float alpha = exp2f(mrun[jt] - mnew);
        float psum = 0.f;
        u16 pb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p = vis[e] ? exp2f(v[e] - mnew) : 0.f;
          psum += p;
          pb[e] = f32_to_bf16_bits(p);
        }
        psum += __shfl_xor(psum, 16);
        psum += __shfl_xor(psum, 32);
        lrun[jt] = lrun[jt] * alpha + psum;
        mrun[jt] = mnew;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt][jt] *= alpha;
        union { bf16x8 v8; u16 h[8]; } cv;
#pragma unroll
        for (int e = 0; e < 8; ++e) cv.h[e] = pb[e];
        pf[jt] = cv.v8;
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
          O[dt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf[jt], O[dt][jt], 0, 0, 0);
    }

    // ---- merge the four wavefronts ---------------------------------------------------------------
    if (g == 0) {
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
        sm[wave][jt * 16 + col] = mrun[jt];
        sl[wave][jt * 16 + col] = lrun[jt];
      }
    }
    __syncthreads();
    float mall[JT], lall[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      float mm = sm[0][jt * 16 + col];
#pragma unroll
      for (int w = 1; w < kWavesPerWG; ++w) mm = fmaxf(mm, sm[w][jt * 16 + col]);
      float ll = 0.f;
#pragma unroll
      for (int w = 0; w < kWavesPerWG; ++w) ll += sl[w][jt * 16 + col] * exp2f(sm[w][jt * 16 + col] - mm);
      mall[jt] = mm;
      lall[jt] = ll;
      const float f = exp2f(mrun[jt] - mm);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) O[dt][jt] *= f;
    }
    for (int w = 0; w < kWavesPerWG; ++w) {           // fixed order: wave 0, 1, 2, 3
      if (wave == w) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int jt = 0; jt < JT; ++jt) {
            if (w == 0) sO[dt * JT + jt][lane] = O[dt][jt];
            else sO[dt * JT + jt][lane] += O[dt][jt];
          }
      }
      __syncthreads();
    }
    f32x4* po = reinterpret_cast<f32x4*>(a.pO) + (size_t)item * (DT * JT) * 64;
    for (int idx = wave; idx < DT * JT; idx += kWavesPerWG) po[idx * 64 + lane] = sO[idx][lane];
    if (wave == 0 && g == 0) {
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
        a.pm[(size_t)item * (JT * 16) + jt * 16 + col] = mall[jt];
        a.pl[(size_t)item * (JT * 16) + jt * 16 + col] = lall[jt];
      }
    }
    __syncthreads();
  }
}

// Merge the chunk partials of one (kv head, column group), normalise, store bf16 in the packed
// activation layout the O-projection reads.  One workgroup per (kv head, column group).
template <int D, int JT>
__global__ __launch_bounds__(kWGThreads) void attn_combine_kernel(AttnArgs a) {
  constexpr int DT = D / 16;
  constexpr int kMaxChunks = 128;
  __shared__ float wgt[kMaxChunks][JT * 16];

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const int n = a.st->n;
  const int G = a.n_q / a.n_kv;
  const int Mp = a.MT * 16;
  const int n_jg = (G * a.MT) / JT;
  int n_kb, chunk_len, n_chunks;
  attn_chunks(n + a.M, a.max_chunks, n_kb, chunk_len, n_chunks);

  for (int grp = blockIdx.x; grp < a.n_kv * n_jg; grp += gridDim.x) {
    const int jg = grp % n_jg, kvh = grp / n_jg;
    const size_t item0 = (size_t)grp * n_chunks;
    if (threadIdx.x < JT * 16) {
      const int c = threadIdx.x;
      float mm = kNegBig;
      for (int ch = 0; ch < n_chunks; ++ch) mm = fmaxf(mm, a.pm[(item0 + ch) * (JT * 16) + c]);
      float ll = 0.f;
      for (int ch = 0; ch < n_chunks; ++ch) {
        const float w = exp2f(a.pm[(item0 + ch) * (JT * 16) + c] - mm);
        ll += a.pl[(item0 + ch) * (JT * 16) + c] * w;
        wgt[ch][c] = w;
      }
      const float inv = 1.f / ll;
      for (int ch = 0; ch < n_chunks; ++ch) wgt[ch][c] *= inv;
    }
    __syncthreads();
    const f32x4* po = reinterpret_cast<const f32x4*>(a.pO) + item0 * (DT * JT) * 64;
    for (int idx = wave; idx < DT * JT; idx += kWavesPerWG) {
      const int dt = idx / JT, jt = idx % JT;
      f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int ch = 0; ch < n_chunks; ++ch)
        acc += po[((size_t)ch * (DT * JT) + idx) * 64 + lane] * wgt[ch][jt * 16 + col];
      const int c = (jg * JT + jt) * 16 + col;
      const int hq = c / Mp, m = c - hq * Mp;
      if (m < a.M) {
        const int f = (kvh * G + hq) * D + dt * 16 + 4 * g;
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
        pk.y = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
        *reinterpret_cast<uint2*>(a.out + xp_index(m, f, a.MT)) = pk;
      }
    }
    __syncthreads();
  }
}

// ---- operand conversion of the stand-alone entry point ----
__global__ void unpack_x_kernel(const u16* __restrict__ xp, int M, int K, float* __restrict__ x, int MT) {
  const size_t total = (size_t)M * K;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int m = (int)(idx / K), k = (int)(idx % K);
    x[idx] = bf16_bits_to_f32(xp[xp_index(m, k, MT)]);
  }
}

// fp32 [T][n_kv][D] keys and values -> packed bf16 caches of one layer
__global__ void pack_kv_kernel(const float* __restrict__ k, const float* __restrict__ v, int T, int n_kv, int D,
                               int max_kb, u16* __restrict__ Kc, u16* __restrict__ Vc) {
  const size_t total = (size_t)T * n_kv * D;
  const size_t kv_head_elems = (size_t)max_kb * 32 * D;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int d = idx % D, h = (idx / D) % n_kv, p = (int)(idx / ((size_t)D * n_kv));
    Kc[h * kv_head_elems + kp_index(p, d, D / 32)] = f32_to_bf16_bits(k[idx]);
    Vc[h * kv_head_elems + vp_index(p, d, D / 16)] = f32_to_bf16_bits(v[idx]);
  }
}

}  // namespace bd
