// Small kernels around the GEMMs: operand packing, embedding gather, rotary table, split-K
// reductions with their fused epilogues, and the per-step decision kernels (seed, unmask, commit,
// verify-accept).
#pragma once
#include "attention.h"
#include "common.h"
#include "gemm.h"

namespace bd {

// ---- weight packing ---------------------------------------------------------------------------------
// src is a row-major [n_rows][K] matrix (fp32, bf16 bits, or e4m3 bytes with a per-row scale);
// source row tile i lands in packed tile (tile_off + i*tile_stride), which lets the loader fuse
// Q|K|V and interleave gate/up tiles.
__device__ inline float e4m3_to_f32(uint8_t c) {
  const int e = (c >> 3) & 0xF, m = c & 7;
  float v = (e == 0) ? (float)m * 0.001953125f                       // m/8 * 2^-6
                     : __uint_as_float((uint32_t)(e + 120) << 23) * (1.f + (float)m * 0.125f);
  return (c & 0x80) ? -v : v;
}

template <typename SrcT>
__global__ void pack_weight_kernel(const SrcT* __restrict__ src, const float* __restrict__ row_scale, int n_rows,
                                   int K, int KS, u16* __restrict__ dst, int tile_off, int tile_stride) {
  const size_t total = (size_t)(n_rows / 16) * KS * 512;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int e = idx & 7, lane = (idx >> 3) & 63;
    const size_t tile = idx >> 9;
    const int ks = (int)(tile % KS), nt = (int)(tile / KS);
    const int r = nt * 16 + (lane & 15), k = ks * 32 + 8 * (lane >> 4) + e;
    u16 out = 0;
    if (k < K) {
      if constexpr (sizeof(SrcT) == 4) out = f32_to_bf16_bits(((const float*)src)[(size_t)r * K + k]);
      else if constexpr (sizeof(SrcT) == 2) out = ((const u16*)src)[(size_t)r * K + k];
      else out = f32_to_bf16_bits(e4m3_to_f32(((const uint8_t*)src)[(size_t)r * K + k]) * row_scale[r]);
    }
    dst[(((size_t)(tile_off + nt * tile_stride) * KS + ks) * 64 + lane) * 8 + e] = out;
  }
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, u16* __restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = f32_to_bf16_bits(src[i]);
}

// ---- block assembly: embedding gather into the fp32 residual stream ---------------------------------
// Row r takes embeds[off + r] while off + r < n_embed, else table[id] with id = ids[off + r - n_embed];
// with a mask array, masked rows take the mask token's embedding instead.
__global__ void embed_kernel(float* __restrict__ x, int H, const float* __restrict__ embeds, int n_embed,
                             const int* __restrict__ ids, int off, const uint8_t* __restrict__ mask,
                             int mask_id, const u16* __restrict__ table, int vocab) {
  const int r = blockIdx.x;
  const int p = off + r;
  if (p < n_embed) {
    for (int c = threadIdx.x; c < H; c += blockDim.x) x[(size_t)r * H + c] = embeds[(size_t)p * H + c];
    return;
  }
  int id = ids[p - n_embed];
  if (mask != nullptr && mask[p - n_embed]) id = mask_id;
  id = min(max(id, 0), vocab - 1);
  for (int c = threadIdx.x; c < H; c += blockDim.x) x[(size_t)r * H + c] = bf16_bits_to_f32(table[(size_t)id * H + c]);
}

// ---- rotary table for positions n .. n+M-1: (cos, sin) of pos * theta^(-2i/d), i < d/2 ------------------
__global__ void rope_table_kernel(float2* __restrict__ tab, const DevState* st, int half, float theta) {
  const int m = blockIdx.x;
  const double pos = (double)(st->n + m);
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double inv = exp2(-log2((double)theta) * (double)i / (double)half);
    const double ang = pos * inv;
    tab[(size_t)m * half + i] = make_float2((float)cos(ang), (float)sin(ang));
  }
}

// ---- residual add of split-K partials + RMSNorm -> packed bf16 operand ---------------------------------
// x[m][:] += sum_s partial[s][m][:]   (fixed order s = 0..S-1; S may be 0)
// xp = bf16( x * rsqrt(mean(x^2) + eps) * gain )  in packed activation order.   One workgroup per row.
__global__ __launch_bounds__(kWGThreads) void resid_norm_kernel(float* __restrict__ x, const float* __restrict__ partial,
                                                               int S, int Mp, int H, const float* __restrict__ gain,
                                                               float eps, u16* __restrict__ xp, int MT) {
  __shared__ float wsum[kWavesPerWG];
  const int m = blockIdx.x;
  float* xr = x + (size_t)m * H;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < H; c += kWGThreads * 4) {
    f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);
    for (int s = 0; s < S; ++s) v += *reinterpret_cast<const f32x4*>(partial + ((size_t)s * Mp + m) * H + c);
    *reinterpret_cast<f32x4*>(xr + c) = v;
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  const float rs = rsqrtf(tot / (float)H + eps);
  for (int c = threadIdx.x * 4; c < H; c += kWGThreads * 4) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(xr + c);
    const f32x4 gn = *reinterpret_cast<const f32x4*>(gain + c);
    uint2 pk;
    pk.x = (uint32_t)f32_to_bf16_bits(v[0] * rs * gn[0]) | ((uint32_t)f32_to_bf16_bits(v[1] * rs * gn[1]) << 16);
    pk.y = (uint32_t)f32_to_bf16_bits(v[2] * rs * gn[2]) | ((uint32_t)f32_to_bf16_bits(v[3] * rs * gn[3]) << 16);
    *reinterpret_cast<uint2*>(xp + xp_index(m, c, MT)) = pk;
  }
}

// ---- QKV split-K reduction + rotary + Q store + KV-cache write -------------------------------------------
// partial: [S][Mp][Nqkv] with columns [Q | K | V].  One workgroup per block row m (position n + m).
// Work units of 8 consecutive dims: Q and K units are rotary pairs (dims i..i+7 and i+half..i+half+7).
struct QkvPostArgs {
  const float* partial;
  int S, Mp, n_q, n_kv, D, max_kb;
  const float2* rope;       // [M][D/2]
  const DevState* st;
  u16* Q;                   // [Mp][n_q][D]
  u16* Kc;                  // this layer's packed caches
  u16* Vc;
};

__global__ __launch_bounds__(kWGThreads) void qkv_post_kernel(QkvPostArgs a) {
  const int m = blockIdx.x;
  const int D = a.D, half = D / 2;
  const int N = (a.n_q + 2 * a.n_kv) * D;
  const int key = a.st->n + m;
  const int upr = half / 8;                             // rotary units per head
  const int uq = a.n_q * upr, uk = a.n_kv * upr, uv = a.n_kv * (D / 8);
  const size_t kv_head_elems = (size_t)a.max_kb * 32 * D;
  for (int u = threadIdx.x; u < uq + uk + uv; u += kWGThreads) {
    if (u < uq + uk) {
      const bool isq = u < uq;
      const int uu = isq ? u : u - uq;
      const int h = uu / upr, i0 = (uu % upr) * 8;
      const int cbase = (isq ? 0 : a.n_q * D) + h * D;
      float lo[8], hi[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) { lo[e] = 0.f; hi[e] = 0.f; }
      for (int s = 0; s < a.S; ++s) {
        const float* p = a.partial + ((size_t)s * a.Mp + m) * N + cbase;
#pragma unroll
        for (int e = 0; e < 8; ++e) { lo[e] += p[i0 + e]; hi[e] += p[i0 + half + e]; }
      }
      u16 olo[8], ohi[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float2 cs = a.rope[(size_t)m * half + i0 + e];
        olo[e] = f32_to_bf16_bits(lo[e] * cs.x - hi[e] * cs.y);
        ohi[e] = f32_to_bf16_bits(hi[e] * cs.x + lo[e] * cs.y);
      }
      uint4 plo, phi;
      plo.x = olo[0] | ((uint32_t)olo[1] << 16); plo.y = olo[2] | ((uint32_t)olo[3] << 16);
      plo.z = olo[4] | ((uint32_t)olo[5] << 16); plo.w = olo[6] | ((uint32_t)olo[7] << 16);
      phi.x = ohi[0] | ((uint32_t)ohi[1] << 16); phi.y = ohi[2] | ((uint32_t)ohi[3] << 16);
      phi.z = ohi[4] | ((uint32_t)ohi[5] << 16); phi.w = ohi[6] | ((uint32_t)ohi[7] << 16);
      if (isq) {
        u16* q = a.Q + ((size_t)m * a.n_q + h) * D;
        *reinterpret_cast<uint4*>(q + i0) = plo;
        *reinterpret_cast<uint4*>(q + i0 + half) = phi;
      } else {
        u16* kc = a.Kc + (size_t)h * kv_head_elems;
        *reinterpret_cast<uint4*>(kc + kp_index(key, i0, D / 32)) = plo;
        *reinterpret_cast<uint4*>(kc + kp_index(key, i0 + half, D / 32)) = phi;
      }
    } else {
      const int uu = u - uq - uk;
      const int h = uu / (D / 8), d0 = (uu % (D / 8)) * 8;
      const int cbase = (a.n_q + a.n_kv) * D + h * D + d0;
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = 0.f;
      for (int s = 0; s < a.S; ++s) {
        const float* p = a.partial + ((size_t)s * a.Mp + m) * N + cbase;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += p[e];
      }
      u16* vc = a.Vc + (size_t)h * kv_head_elems;
#pragma unroll
      for (int e = 0; e < 8; ++e) vc[vp_index(key, d0 + e, D / 16)] = f32_to_bf16_bits(v[e]);
    }
  }
}

// Unpack cache positions [pos0, pos0+count) of one layer to fp32 [count][n_kv][D].
// rot_pairs: the K cache holds each head's dims in rotary-pair order (dim i at 2i, dim i + D/2 at 2i + 1).
__global__ void read_kv_kernel(const u16* __restrict__ Kc, const u16* __restrict__ Vc, int n_kv, int D, int max_kb,
                               int pos0, int count, float* __restrict__ k_out, float* __restrict__ v_out,
                               int rot_pairs) {
  const size_t total = (size_t)count * n_kv * D;
  const size_t kv_head_elems = (size_t)max_kb * 32 * D;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int d = idx % D, h = (idx / D) % n_kv, p = (int)(idx / ((size_t)D * n_kv));
    const int dk = rot_pairs ? (d < D / 2 ? 2 * d : 2 * (d - D / 2) + 1) : d;
    if (k_out) k_out[idx] = bf16_bits_to_f32(Kc[h * kv_head_elems + kp_index(pos0 + p, dk, D / 32)]);
    if (v_out) v_out[idx] = bf16_bits_to_f32(Vc[h * kv_head_elems + vp_index(pos0 + p, d, D / 16)]);
  }
}


// ---- helpers of the kernel-level entry points ---------------------------------------------------------------
__global__ void pack_x_kernel(const float* __restrict__ x, int M, int K, u16* __restrict__ xp, int MT) {
  const size_t total = (size_t)M * K;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int m = (int)(idx / K), k = (int)(idx % K);
    xp[xp_index(m, k, MT)] = f32_to_bf16_bits(x[idx]);
  }
}

__global__ void unpack_x_kernel(const u16* __restrict__ xp, int M, int K, float* __restrict__ x, int MT) {
  const size_t total = (size_t)M * K;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int m = (int)(idx / K), k = (int)(idx % K);
    x[idx] = bf16_bits_to_f32(xp[xp_index(m, k, MT)]);
  }
}

__global__ void reduce_partial_kernel(const float* __restrict__ partial, int S, int Mp, int N, int M,
                                      float* __restrict__ y) {
  const size_t total = (size_t)M * N;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int m = (int)(idx / N), c = (int)(idx % N);
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += partial[((size_t)s * Mp + m) * N + c];
    y[idx] = v;
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

// ---- per-step decisions -------------------------------------------------------------------------------------

// Seed (Sec. 3.4, causal context decoding): a block whose position 0 is still masked takes the
// carry's argmax there before the forward.
__global__ void seed_kernel(int* tokens, uint8_t* mask, DevState* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->seeded = 0;
    if (mask[0]) {
      tokens[0] = st->carry_cand;
      mask[0] = 0;
      st->seeded = 1;
    }
  }
}

struct FinishArgs {
  int B;
  DevState* st;
  const int* row_cand;      // [B] argmax id of every row of the forward (row i predicts position i+1)
  const float* row_conf;    // [B] its softmax probability
  // denoise
  int* tokens;
  uint8_t* mask;
  float threshold;
  int fixed_k;
  int* n_unmasked;
  float* conf_out;
  // commit / verify
  const int* draft;
  int commit;
  int* ar_pred;
  int* n_accept;
  int skippable;            // bd_decode_block: do nothing once the block is complete, else count the step and set the flag
};

// Confidence-threshold parallel unmask (Sec. 3.4; "Decoding threshold").  Row i-1 predicts block
// position i.  Launched with one wavefront.
__global__ __launch_bounds__(64) void finish_denoise_kernel(FinishArgs a) {
  __shared__ int s_cand[64];
  __shared__ float s_conf[64];
  __shared__ uint8_t s_mask[64];
  if (a.skippable && a.st->skip) return;
  if ((int)threadIdx.x < a.B) {
    s_cand[threadIdx.x] = a.row_cand[threadIdx.x];
    s_conf[threadIdx.x] = a.row_conf[threadIdx.x];
    s_mask[threadIdx.x] = a.mask[threadIdx.x];
    if (a.conf_out) a.conf_out[threadIdx.x] = threadIdx.x == 0 ? a.st->carry_conf : a.row_conf[threadIdx.x - 1];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int revealed = a.st->seeded;
    int remaining = 0;
    for (int i = 1; i < a.B; ++i) remaining += s_mask[i] ? 1 : 0;
    if (remaining > 0) {
      if (a.fixed_k > 0) {
        const int k = min(a.fixed_k, remaining);
        for (int t = 0; t < k; ++t) {                    // k passes of "most confident still masked"
          int best = -1;
          float bc = -1.f;
          for (int i = 1; i < a.B; ++i)
            if (s_mask[i] && s_conf[i - 1] > bc) { bc = s_conf[i - 1]; best = i; }
          a.tokens[best] = s_cand[best - 1];
          a.mask[best] = 0;
          s_mask[best] = 0;
          ++revealed;
        }
      } else {
        int best = -1, cnt = 0;
        float bc = -1.f;
        for (int i = 1; i < a.B; ++i) {
          if (!s_mask[i]) continue;
          const float c = s_conf[i - 1];
          if (c > bc) { bc = c; best = i; }
          if (c > a.threshold) {
            a.tokens[i] = s_cand[i - 1];
            a.mask[i] = 0;
            s_mask[i] = 0;
            ++cnt;
          }
        }
        if (cnt == 0) {
          a.tokens[best] = s_cand[best - 1];
          a.mask[best] = 0;
          s_mask[best] = 0;
          cnt = 1;
        }
        revealed += cnt;
      }
    }
    if (a.n_unmasked) *a.n_unmasked = revealed;
    if (a.skippable) {
      int left = 0;
      for (int i = 1; i < a.B; ++i) left += s_mask[i] ? 1 : 0;
      a.st->steps += 1;
      a.st->skip = left == 0;
    }
  }
}

// B == 1 (or nothing to denoise): only report the seed.
__global__ void finish_seed_only_kernel(DevState* st, int* n_unmasked, float* conf_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (n_unmasked) *n_unmasked = st->seeded;
    if (conf_out) conf_out[0] = st->carry_conf;
  }
}

// Causal pass: row j's argmax is the autoregressive prediction a_j (Alg. 1 verify step).  Accept
// length = longest prefix of the draft with draft[0] == carry's argmax and draft[j+1] == a_j.
// With commit, the carry moves to the last row and the context length grows by B.
__global__ __launch_bounds__(64) void finish_causal_kernel(FinishArgs a) {
  __shared__ int s_cand[64];
  __shared__ float s_conf[64];
  if ((int)threadIdx.x < a.B) {
    s_cand[threadIdx.x] = a.row_cand[threadIdx.x];
    s_conf[threadIdx.x] = a.row_conf[threadIdx.x];
    if (a.ar_pred) a.ar_pred[threadIdx.x] = a.row_cand[threadIdx.x];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (a.n_accept && a.commit != 2) {
      int k = 0;
      while (k < a.B && a.draft[k] == (k == 0 ? a.st->carry_cand : s_cand[k - 1])) ++k;
      *a.n_accept = k;
    }
    if (a.commit == 1) {
      a.st->carry_cand = s_cand[a.B - 1];
      a.st->carry_conf = s_conf[a.B - 1];
      a.st->n += a.B;
    } else if (a.commit == 2) {
      // Alg. 1 accept + crop in place: draft[0] is the already accepted first token; k = 1 + the number of leading
      // drafts draft[1..] that equal the predictions a_0..; the emitted tokens are a_0..a_{k-1}; the cache keeps the
      // positions of draft[0..k-1] (the rows beyond were written but the length does not cover them), and a_{k-1}
      // becomes the prediction for the new position n.
      int k = 1;
      while (k < a.B && s_cand[k - 1] == a.draft[k]) ++k;
      *a.n_accept = k;
      a.st->carry_cand = s_cand[k - 1];
      a.st->carry_conf = s_conf[k - 1];
      a.st->n += k;
    }
  }
}

// ---- Alg. 2 (quadratic speculative decoding) ------------------------------------------------------------------
// Rows of the quadratic forward: group i = [draft[i], MASK x B].
__global__ void quad_assemble_kernel(const int* draft, int B, int mask_id, int* ids) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  const int W = B + 1;
  if (r < B * W) ids[r] = (r % W == 0) ? draft[r / W] : mask_id;
}
// Draft 0 of Alg. 2's first block is the carry's prediction (the hidden state of the last context row).
__global__ void quad_first_kernel(int* draft, const DevState* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) draft[0] = st->carry_cand;
}
// Accept: P[i][j] = argmax of group i, entry j (predicts position n+i+j+1).  k = 1 + leading drafts d_1.. that equal
// P[0][0], P[1][0], ..; the next draft block is P[k-1][0..B-1]; the prediction of group k-1's first row becomes the
// carry and the context grows by k (the keys and values of the accepted first rows are moved into place afterwards).
__global__ __launch_bounds__(64) void finish_quad_kernel(FinishArgs a, int* next_draft) {
  const int W = a.B + 1;
  if (threadIdx.x == 0) {
    int k = 1;
    while (k < a.B && a.row_cand[(k - 1) * W] == a.draft[k]) ++k;
    *a.n_accept = k;
    for (int j = 0; j < a.B; ++j) next_draft[j] = a.row_cand[(k - 1) * W + j];
    a.st->carry_cand = a.row_cand[(k - 1) * W];
    a.st->carry_conf = a.row_conf[(k - 1) * W];
    a.st->n += k;
  }
}
// The quadratic forward left the keys and values of row r at cache position n0 + r; the accepted tokens are the
// first rows of groups 0..k-1, i.e. rows i*(B+1), and belong at positions n0 + i.  (Destinations 1..k-1 < B+1 never
// coincide with a source, so all moves are independent.)  One workgroup per (layer, kv head).
__global__ void quad_compact_kv_kernel(u16* Kc, u16* Vc, size_t kv_layer_elems, int n_kv, int D, int max_kb, const DevState* st,
                                       const int* k_ptr, int B) {
  const int layer = blockIdx.x / n_kv, h = blockIdx.x % n_kv;
  const int k = *k_ptr;
  const int n0 = st->n - k;                       // the accept kernel has already advanced the length
  u16* kc = Kc + (size_t)layer * kv_layer_elems + (size_t)h * max_kb * 32 * D;
  u16* vc = Vc + (size_t)layer * kv_layer_elems + (size_t)h * max_kb * 32 * D;
  for (int t = threadIdx.x; t < (k - 1) * D; t += blockDim.x) {
    const int i = 1 + t / D, d = t % D;
    kc[kp_index(n0 + i, d, D / 32)] = kc[kp_index(n0 + i * (B + 1), d, D / 32)];
    vc[vp_index(n0 + i, d, D / 16)] = vc[vp_index(n0 + i * (B + 1), d, D / 16)];
  }
}

// All positions of a block masked (the state before the draft pass of Alg. 1).
__global__ void fill_masked_kernel(int* tokens, uint8_t* mask, int B, int mask_id, DevState* st, int first_revealed = 0) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) { tokens[i] = mask_id; mask[i] = (i == 0 && first_revealed) ? 0 : 1; }
  if (i == 0) { st->skip = 0; st->steps = 0; }
}
__global__ void read_steps_kernel(const DevState* st, int* out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *out = st->steps;
}

// Commit without an LM-head pass (prompt chunks before the last one).
__global__ void advance_kernel(DevState* st, int B) {
  if (threadIdx.x == 0 && blockIdx.x == 0) st->n += B;
}

__global__ void set_state_kernel(DevState* st, int n, int clear_carry) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->n = n;
    st->seeded = 0;
    if (clear_carry) { st->carry_cand = -1; st->carry_conf = 0.f; }
  }
}

}  // namespace bd
