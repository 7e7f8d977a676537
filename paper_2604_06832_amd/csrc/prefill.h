// Large-M prefill (Alg. 1 "prefill": one causal forward over the prompt that fills the KV cache).
//
// The decode kernels stream every weight once per forward of at most 64 rows, so a prompt of n tokens pushed
// through them re-reads the model n/64 times.  For the bulk of the prompt this file provides the compute-bound
// form: chunks of up to 1024 rows, each layer as a sequence of tiled MFMA GEMMs with the same fused epilogues as the
// decode path (RMS factor, rotary + Q store + K/V store; residual add; SwiGLU) and a causal attention kernel that
// walks the packed cache with the decode path's per-block routine.  Only the LM head, needed for the last row alone,
// is the decode path's.
//
// Operand layout: both GEMM operands are kept as 1-KiB MFMA fragments (16 rows x 32 k, lane (row i, k-quarter kq)
// holds 8 consecutive k at lane*16 bytes).  Weights: fragment (row tile T, k-step ks) of a layer's phase at
// ((T*KS + ks)*64 + lane) 16-byte units, rows in the decode path's phase-row order (rotary pairs of q/k adjacent,
// (gate f, up f) adjacent, norm gains folded into the columns).  Activations: the packed order of xp_index().
#pragma once
#include "prefill_args.h"
#include "prefill_attn.h"
#include "stream_fwd.h"

namespace bd {

// Epilogue of both GEMM kernels: lane (token column col, row quad g) of a 16 x 16 accumulator tile holds rows
// r .. r+3 of one token.
template <int PH, int WN, int TW>
__device__ inline void pf_epilogue(const PfGemmArgs& a, const f32x4 (&acc)[WN][TW], int T0, int mt0, int wn, int wm, int lane,
                                   int kz = 0) {
  const int col = lane & 15, g = lane >> 4;
#pragma unroll
  for (int i = 0; i < WN; ++i) {
    const int T = T0 + wn * WN + i;
    if (T >= a.NT) continue;
    const int r = T * 16 + 4 * g;
#pragma unroll
    for (int j = 0; j < TW; ++j) {
      if (mt0 + wm * TW + j >= a.MTc) continue;
      const int token = (mt0 + wm * TW + j) * 16 + col;
      f32x4 v = acc[i][j];
      if (a.wscale != nullptr) v *= *reinterpret_cast<const f32x4*>(a.wscale + r);
      if constexpr (PH == PH_QKV) {
        if (token >= a.Mvalid) continue;
        const int D = a.D, half = D >> 1;
        v *= a.rs[token];
        const int key = paged_key(a.pages, a.n0 + token);
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          const int rp = r + 2 * pr;
          if (rp < a.QD + a.KVD) {
            // rotary pair: phase rows (2i, 2i+1) of a head hold dims (i, i + D/2)
            const int dp = rp % D;
            const float2 cs = a.rope[(size_t)token * half + (dp >> 1)];
            const float lo = v[2 * pr] * cs.x - v[2 * pr + 1] * cs.y;
            const float hi = v[2 * pr + 1] * cs.x + v[2 * pr] * cs.y;
            const uint32_t pk = (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
            u16* dst;
            if (rp < a.QD) {
              dst = a.q + ((size_t)token * a.n_q + rp / D) * D + dp;
            } else {
              const int rk = rp - a.QD;
              dst = a.Kc + (size_t)(rk / D) * a.max_kb * 32 * D + kp_index(key, dp, D / 32);
            }
            *reinterpret_cast<uint32_t*>(dst) = pk;
          } else {
            const int rv = rp - a.QD - a.KVD;
            u16* vc = a.Vc + (size_t)(rv / D) * a.max_kb * 32 * D;
            vc[vp_index(key, rv % D, D / 16)] = f32_to_bf16_bits(v[2 * pr]);
            vc[vp_index(key, (rv + 1) % D, D / 16)] = f32_to_bf16_bits(v[2 * pr + 1]);
          }
        }
      } else if constexpr (PH == PH_O || PH == PH_DOWN) {
        if (a.part != nullptr) {
          *reinterpret_cast<f32x4*>(a.part + ((size_t)kz * a.MTc * 16 + token) * a.H + r) = v;
        } else {
          f32x4* xp = reinterpret_cast<f32x4*>(a.x + (size_t)token * a.H + r);
          *xp = *xp + v;
        }
      } else {
        v *= a.rs[token];
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          const float gt = v[2 * pr], up = v[2 * pr + 1];
          a.act[xp_index(token, (r >> 1) + pr, a.MTc)] = f32_to_bf16_bits(gt / (1.f + __expf(-gt)) * up);
        }
      }
    }
  }
}

// C[rows of the phase][tokens] = W * X^T, fp32 accumulation, epilogue per phase.  A workgroup computes
// (2*WN*16) rows x (2*TW*16) tokens; each wavefront WN x TW tiles of 16 x 16.  K advances by BKS k-steps per iteration
// through two LDS stages; the operands of a stage travel global memory -> registers -> LDS, the loads of stage i+1
// being issued before the MFMAs of stage i.  (A second register set, two stages ahead, costs more in registers than
// it hides in latency: measured slower for every shape here.)
template <int PH, int WN, int BKS, int TW>
__global__ __launch_bounds__(kPfThreads, (2 * (2 * WN * BKS * 64 + 2 * TW * BKS * 64) * 16 <= 80 * 1024) ? 2 : 1) void pf_gemm_kernel(PfGemmArgs a) {
  constexpr int AT = 2 * WN;                                        // row tiles per workgroup
  constexpr int BT = 2 * TW;                                        // token tiles per workgroup
  constexpr int A_UNITS = AT * BKS * 64, B_UNITS = BT * BKS * 64;   // 16-byte units per stage
  constexpr int STAGE = A_UNITS + B_UNITS;
  constexpr int A_PER = A_UNITS / kPfThreads, B_PER = B_UNITS / kPfThreads;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  bf16x8* sm = reinterpret_cast<bf16x8*>(lds);
  if (a.skippable && a.st->skip) return;
  // Row group rg runs on XCD rg mod 8 for all of its token groups, so that a weight tile is fetched into one L2.
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int rg = (slot / a.TG) * 8 + xcd, tg = slot % a.TG;
  if (rg >= a.RG) return;
  const int T0 = rg * AT, mt0 = tg * BT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wn = wave >> 1, wm = wave & 1;
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};

  // Operands come through raw buffer loads (an offset past the end returns zeros and moves nothing).  Unit u = thread
  // + 256 i of a stage: for the weights tile u / (BKS*64), unit u mod (BKS*64) of its BKS KiB; for the activations
  // k-step u / 512, unit u mod 512 of the eight token tiles.
  const rsrc_t wr = make_rsrc(a.w, (unsigned)((size_t)a.NT * a.KS * 1024));
  const rsrc_t xr = make_rsrc(a.xin, (unsigned)((size_t)a.KS * a.MTc * 1024));
  struct Regs { bf16x8 a[A_PER], b[B_PER]; };
  constexpr int TU = BKS * 64;                                      // units per weight tile and stage
  const int a_tile = threadIdx.x / TU, a_within = threadIdx.x % TU; // (256 / TU tiles per round of 256 units)
  const int a_base = ((T0 + a_tile) * a.KS) * 1024 + a_within * 16;
  const int a_ksl = a_within >> 6;
  constexpr int UB = BT * 64;                                       // activation units per k-step
  const int b_base = mt0 * 1024 + threadIdx.x * 16;
  const int b_tile = threadIdx.x >> 6;
  auto gload = [&](Regs& R, int it) {
    const int ks0 = it * BKS;
    const bool a_ok = ks0 + a_ksl < a.KS;
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      const int off = a_base + (i * (kPfThreads / TU) * a.KS + ks0) * 1024;
      R.a[i] = buf_load_b(wr, (a_ok && T0 + a_tile + i * (kPfThreads / TU) < a.NT) ? off : kOob);
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      const int ksl = (i * kPfThreads) / UB, part = (i * kPfThreads) % UB;      // units part .. part+255 of that k-step
      const int off = b_base + ((ks0 + ksl) * a.MTc) * 1024 + part * 16;
      R.b[i] = buf_load_b(xr, (ks0 + ksl < a.KS && mt0 + b_tile + part / 64 < a.MTc) ? off : kOob);
    }
  };
  auto lstore = [&](const Regs& R, int stage) {
    bf16x8* A = sm + stage * STAGE;
#pragma unroll
    for (int i = 0; i < A_PER; ++i) A[threadIdx.x + i * kPfThreads] = R.a[i];
#pragma unroll
    for (int i = 0; i < B_PER; ++i) A[A_UNITS + threadIdx.x + i * kPfThreads] = R.b[i];
  };

  f32x4 acc[WN][TW];
#pragma unroll
  for (int i = 0; i < WN; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int stage) {
    const bf16x8* A = sm + stage * STAGE;
    const bf16x8* Bm = A + A_UNITS;
#pragma unroll
    for (int ksl = 0; ksl < BKS; ++ksl) {
      bf16x8 af[WN], bfr[TW];
#pragma unroll
      for (int i = 0; i < WN; ++i) af[i] = A[((wn * WN + i) * BKS + ksl) * 64 + lane];
#pragma unroll
      for (int j = 0; j < TW; ++j) bfr[j] = Bm[(ksl * BT + wm * TW + j) * 64 + lane];
#pragma unroll
      for (int i = 0; i < WN; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  };

  const int n_it = (a.KS + BKS - 1) / BKS;
  Regs R0;
  gload(R0, 0);
  lstore(R0, 0);
  __syncthreads();
  for (int it = 0; it < n_it; ++it) {
    if (it + 1 < n_it) gload(R0, it + 1);
    compute(it & 1);
    if (it + 1 < n_it) lstore(R0, (it + 1) & 1);
    __syncthreads();
  }

  pf_epilogue<PH, WN, TW>(a, acc, T0, mt0, wn, wm, lane);
}

// The same product with the operands loaded straight into LDS (no registers in between) through NST stages: the loads
// of iteration i + NST - 1 are issued, one 1-KiB fragment per instruction and wavefront, before the MFMAs of
// iteration i, and one barrier per iteration both publishes the stage that has landed and frees the one just read.
// (Measured on the gate/up shape: two stages with two workgroups per CU beat deeper pipelines with one.)  Needs KS to
// be a multiple of BKS (no K tail); tiles past the end of the rows or tokens re-read the last valid tile and are
// dropped by the epilogue.  With SK > 1 the workgroups of an output tile split K among them and each leaves its
// product in its own slice of `part` (O and down phases: a 128 x 128 tile then fetches half the operand bytes per
// MFMA of the 64 x 64 tile that the same number of workgroups would otherwise need).
template <int PH, int WN, int BKS, int TW, int NST, int OCC>
__global__ __launch_bounds__(kPfThreads, OCC) void pf_gemm_direct_kernel(PfGemmArgs a) {
  constexpr int AT = 2 * WN, BT = 2 * TW;
  constexpr int AF = AT * BKS, BF = BT * BKS;                       // fragments per stage
  constexpr int PER = (AF + BF) / 4;                                // loads per wavefront and stage
  static_assert(AF % 4 == 0 && BF % 4 == 0, "fragments are dealt to four wavefronts");
  static_assert((NST - 2) * PER <= 63, "outstanding loads must fit the counter");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  if (a.skippable && a.st->skip) return;
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int per = a.TG * a.SK;                                      // workgroups of a row group: token groups x K splits
  const int rg = (slot / per) * 8 + xcd, tg = (slot % per) / a.SK, kz = slot % a.SK;
  if (rg >= a.RG) return;
  const int T0 = rg * AT, mt0 = tg * BT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wn = wave >> 1, wm = wave & 1;
  const rsrc_t wr = make_rsrc(a.w, (unsigned)((size_t)a.NT * a.KS * 1024));
  const rsrc_t xr = make_rsrc(a.xin, (unsigned)((size_t)a.KS * a.MTc * 1024));

  const int n_it = a.KS / BKS / a.SK, it0 = kz * n_it;             // this workgroup's share of K
  // Every row group walks its K range from another starting point (fixed by its number: same sums on every run), so that
  // the workgroups running at the same time do not all ask the same L2 channels for the same activation fragment.
  const int rot = (rg * 5) % n_it;
  auto issue = [&](int it) {
    char* base = lds + (it % NST) * ((AF + BF) * 1024);
    int itr = it + rot;
    if (itr >= n_it) itr -= n_it;
    const int ks0 = (it0 + itr) * BKS;
#pragma unroll
    for (int i = 0; i < AF / 4; ++i) {
      const int f = i * 4 + wave, tile = f / BKS, ksl = f % BKS;
      const int off = ((min(T0 + tile, a.NT - 1) * a.KS) + ks0 + ksl) * 1024 + lane * 16;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (lds_void_t*)(base + f * 1024), 16, off, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < BF / 4; ++i) {
      const int f = i * 4 + wave, ksl = f / BT, tile = f % BT;
      const int off = ((ks0 + ksl) * a.MTc + min(mt0 + tile, a.MTc - 1)) * 1024 + lane * 16;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, (lds_void_t*)(base + (AF + f) * 1024), 16, off, 0, 0, 0);
    }
  };

  f32x4 acc[WN][TW];
#pragma unroll
  for (int i = 0; i < WN; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto compute = [&](int stage) {
    const bf16x8* A = reinterpret_cast<const bf16x8*>(lds + stage * ((AF + BF) * 1024));
    const bf16x8* Bm = A + AF * 64;
#pragma unroll
    for (int ksl = 0; ksl < BKS; ++ksl) {
      bf16x8 af[WN], bfr[TW];
#pragma unroll
      for (int i = 0; i < WN; ++i) af[i] = A[((wn * WN + i) * BKS + ksl) * 64 + lane];
#pragma unroll
      for (int j = 0; j < TW; ++j) bfr[j] = Bm[(ksl * BT + wm * TW + j) * 64 + lane];
#pragma unroll
      for (int i = 0; i < WN; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  };

  for (int it = 0; it < NST - 1 && it < n_it; ++it) issue(it);
  for (int it = 0; it < n_it; ++it) {
    // the loads of iteration `it` are this wavefront's oldest: in the steady state NST - 2 later stages may stay in flight
    if (it + NST - 2 < n_it) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NST - 2) * PER) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // (the bare barrier: __syncthreads() is also a fence, which waits for every load in flight and so would empty
    // the pipeline at every iteration; the waits that matter are the explicit one above and the LDS reads of the last
    // iteration, which the MFMAs that used them have already waited for)
    __builtin_amdgcn_s_barrier();
    if (it + NST - 1 < n_it) issue(it + NST - 1);
    compute(it % NST);
  }
  pf_epilogue<PH, WN, TW>(a, acc, T0, mt0, wn, wm, lane, kz);
}

template <int WN, int BKS, int TW, int NST> constexpr int pf_gemm_direct_lds() { return NST * (2 * WN * BKS + 2 * TW * BKS) * 1024; }

template <int WN, int BKS, int TW> constexpr int pf_gemm_lds() { return 2 * (2 * WN * BKS * 64 + 2 * TW * BKS * 64) * 16; }

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

// Rows of a decode block into the fp32 residual stream: row r takes the embedding of ids[r], or of the mask token
// where mask[r] is set.  With seed arrays (denoising step), position 0 first takes the carried prediction if it is
// still masked, exactly as the prologue of the decode kernels does.
__global__ void pf_block_embed_kernel(float* __restrict__ x, int H, const int* ids, const uint8_t* mask,
                                      int* seed_tokens, uint8_t* seed_mask, DevState* st,
                                      int skippable, int mask_id, const u16* __restrict__ table, int vocab) {
  __shared__ int s_id;
  const int r = blockIdx.x;
  if (skippable && st->skip) return;
  if (threadIdx.x == 0) {
    if (r == 0 && seed_mask != nullptr) {
      st->seeded = 0;
      if (seed_mask[0]) {
        seed_tokens[0] = st->carry_cand;
        seed_mask[0] = 0;
        st->seeded = 1;
      }
    }
    int id = ids[r];
    if (mask != nullptr && mask[r]) id = mask_id;
    s_id = min(max(id, 0), vocab - 1);
  }
  __syncthreads();
  const int id = s_id;
  for (int c = threadIdx.x; c < H; c += blockDim.x) x[(size_t)r * H + c] = bf16_bits_to_f32(table[(size_t)id * H + c]);
}

// ---- rotary table for positions n .. n+M-1: (cos, sin) of pos * theta^(-2i/d), i < d/2 ------------------
// (quad_W > 0: rows are groups of quad_W tokens, row m sits at position n + m / W + m % W, Alg. 2)
__global__ void rope_table_kernel(float2* __restrict__ tab, const DevState* st, int half, float theta, int quad_W = 0) {
  const int m = blockIdx.x;
  const double pos = (double)(st->n + (quad_W > 0 ? m / quad_W + m % quad_W : m));
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double inv = exp2(-log2((double)theta) * (double)i / (double)half);
    const double ang = pos * inv;
    tab[(size_t)m * half + i] = make_float2((float)cos(ang), (float)sin(ang));
  }
}

// One wavefront per row: 1/rms of the fp32 residual row and its bf16 copy in packed order; completes the residual
// row first when the projection before it left its product in K splits (the norm gain lives in
// the weights, the factor is applied by the GEMM epilogue: same arithmetic as the decode path).
__global__ __launch_bounds__(kPfThreads) void pf_norm_kernel(float* __restrict__ x, int H, float eps, u16* __restrict__ xb,
                                                             int MTc, float* __restrict__ rs, const float* __restrict__ gain,
                                                             const float* __restrict__ kparts, int n_kparts,
                                                             const DevState* st = nullptr) {
  if (st != nullptr && st->skip) return;
  // one wavefront per row, four rows per workgroup
  const int token = blockIdx.x * (kPfThreads / 64) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (token >= MTc * 16) return;
  float* row = x + (size_t)token * H;
  float ss = 0.f;
  // eight consecutive columns per lane: two 16-byte loads per source, one 16-byte store of the packed copy
  for (int c = lane * 8; c < H; c += 64 * 8) {
    f32x4 v0 = *reinterpret_cast<const f32x4*>(row + c), v1 = *reinterpret_cast<const f32x4*>(row + c + 4);
    if (n_kparts > 0) {
      // the K splits of the projection before this norm, added in split order
      for (int p = 0; p < n_kparts; ++p) {
        const float* src = kparts + ((size_t)p * MTc * 16 + token) * H + c;
        v0 += *reinterpret_cast<const f32x4*>(src);
        v1 += *reinterpret_cast<const f32x4*>(src + 4);
      }
      *reinterpret_cast<f32x4*>(row + c) = v0;
      *reinterpret_cast<f32x4*>(row + c + 4) = v1;
    }
    union { u16 h[8]; u32x4 q; } o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      ss += v0[e] * v0[e] + v1[e] * v1[e];
      o.h[e] = f32_to_bf16_bits(gain != nullptr ? v0[e] * gain[c + e] : v0[e]);
      o.h[4 + e] = f32_to_bf16_bits(gain != nullptr ? v1[e] * gain[c + 4 + e] : v1[e]);
    }
    *reinterpret_cast<u32x4*>(xb + xp_index(token, c, MTc)) = o.q;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if (lane == 0) rs[token] = rsqrtf(ss / (float)H + eps);
}

// The same for chunks of few rows: one workgroup per row, so that the rows of a 64-row forward spread over 64 CUs
// instead of 16 and every lane has one group of eight columns per pass.  Same sums in the same order per column; the sum
// of squares is reduced over the workgroup's lanes in a fixed order.
__global__ __launch_bounds__(kPfThreads) void pf_norm_row_kernel(float* __restrict__ x, int H, float eps, u16* __restrict__ xb,
                                                                 int MTc, float* __restrict__ rs, const float* __restrict__ gain,
                                                                 const float* __restrict__ kparts, int n_kparts,
                                                                 const DevState* st = nullptr) {
  __shared__ float wsum[kPfThreads / 64];
  if (st != nullptr && st->skip) return;
  const int token = blockIdx.x;
  float* row = x + (size_t)token * H;
  float ss = 0.f;
  for (int c = threadIdx.x * 8; c < H; c += kPfThreads * 8) {
    f32x4 v0 = *reinterpret_cast<const f32x4*>(row + c), v1 = *reinterpret_cast<const f32x4*>(row + c + 4);
    if (n_kparts > 0) {
      for (int p = 0; p < n_kparts; ++p) {
        const float* src = kparts + ((size_t)p * MTc * 16 + token) * H + c;
        v0 += *reinterpret_cast<const f32x4*>(src);
        v1 += *reinterpret_cast<const f32x4*>(src + 4);
      }
      *reinterpret_cast<f32x4*>(row + c) = v0;
      *reinterpret_cast<f32x4*>(row + c + 4) = v1;
    }
    union { u16 h[8]; u32x4 q; } o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      ss += v0[e] * v0[e] + v1[e] * v1[e];
      o.h[e] = f32_to_bf16_bits(gain != nullptr ? v0[e] * gain[c + e] : v0[e]);
      o.h[4 + e] = f32_to_bf16_bits(gain != nullptr ? v1[e] * gain[c + 4 + e] : v1[e]);
    }
    *reinterpret_cast<u32x4*>(xb + xp_index(token, c, MTc)) = o.q;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) rs[token] = rsqrtf((wsum[0] + wsum[1] + wsum[2] + wsum[3]) / (float)H + eps);
}

__global__ __launch_bounds__(kPfThreads) void zero_rows_kernel(float* __restrict__ x, int H, const DevState* st = nullptr) {
  if (st != nullptr && st->skip) return;
  for (int c = threadIdx.x; c < H; c += kPfThreads) x[(size_t)blockIdx.x * H + c] = 0.f;
}

}  // namespace bd
