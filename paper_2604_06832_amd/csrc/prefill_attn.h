// Attention kernel of the large-M path (chunks of prompt rows, decode forwards of more than 32 rows) and of the
// stand-alone attention entry points: templates only, so that several translation units may include it.
#pragma once
#include "prefill_args.h"
#include "stream_fwd.h"

namespace bd {

// Attention of a chunk against the packed cache (which already holds the chunk's own keys and values; among them the
// mode decides what a row sees: causal, all of the chunk, or the groups of a quadratic forward):
// NW (2 or 4) wavefronts per (head, tile of 16 query rows) share out the 32-key blocks up to the last visible key
// round-robin, each with the decode path's block routine, and merge through LDS; with two wavefronts per item the items
// of a workgroup are heads of one kv head; two workgroups fit a CU.  (Measured: a variant that stages every block once
// in LDS for four heads of a kv head, one barrier per block, is slower than these register-buffered walks.)
template <int D, int NW, bool QUAD = false>
__global__ __launch_bounds__(64 * (NW > 4 ? NW : 4), NW > 4 ? 1 : 2) void pf_attn_kernel(PfAttnArgs a) {
  constexpr int DS = D / 32, DT = D / 16;
  constexpr int IPW = NW > 4 ? 1 : 4 / NW;                     // items per workgroup, NW wavefronts per item
  __shared__ f32x4 sO[IPW][NW - 1][DT][64];
  __shared__ float sm[IPW][NW - 1][64], sl[IPW][NW - 1][64];
  if (a.skippable && a.st->skip) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int sub = wave / NW, half = wave % NW;                 // wavefront `half` of item `sub` takes blocks half, half + NW, ..
  const int col = lane & 15, g = lane >> 4;
  const int G = a.n_q / a.n_kv, QT = a.Mc >> 4;
  const int item = blockIdx.x * IPW + sub;
  const bool valid = item < a.n_kv * QT * G;
  const int hq = item % G, qt = (item / G) % QT, kvh = valid ? item / (G * QT) : 0;
  const int head = kvh * G + hq;
  const int row = qt * 16 + col;
  const size_t kv_block = (size_t)32 * D / 8;
  const bf16x8* Kh = reinterpret_cast<const bf16x8*>(a.Kc) + (size_t)kvh * a.max_kb * kv_block;
  const bf16x8* Vh = reinterpret_cast<const bf16x8*>(a.Vc) + (size_t)kvh * a.max_kb * kv_block;
  f32x4 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float mrun = kNegBig, lrun = 0.f;
  if (valid) {
    bf16x8 qf[DS];
    {
      const u16* qp = a.q + ((size_t)row * a.n_q + head) * D + 8 * g;
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8*>(qp + ds * 32);
    }
    // blocks holding a key some row of the tile may see: up to its own last row (causal), else all of the chunk
    const int kb_end = ((a.mode == 1 ? min(a.n0 + qt * 16 + 15, a.n0 + a.Mvalid - 1) : a.n0 + a.Mvalid - 1)) / 32 + 1;
    const int cnt = (kb_end - half + NW - 1) / NW;              // this wavefront's blocks: half, half + NW, ..
    const float c = a.scale_log2e;
    // one register buffer: the other wavefronts of the CU cover the load (a second buffer, loaded one block ahead,
    // costs more in registers than it hides: 25.6 us against 19.3 us per layer at 1024 rows)
    auto block = [&](const KvBlock<D>& b, int kb) {
      if (kb * 32 + 31 >= a.n0) attn_block<D, true, QUAD>(b, qf, O, mrun, lrun, kb, a.n0, a.Mvalid, a.mode, row, g, c);
      else attn_block<D, false>(b, qf, O, mrun, lrun, kb, a.n0, a.Mvalid, a.mode, row, g, c);
    };
    KvBlock<D> b0;
    for (int j = 0; j < cnt; ++j) {
      const int kb = half + NW * j;
      kv_load<D>(b0, Kh, Vh, kb, lane, a.pages);
      asm volatile("" ::: "memory");
      block(b0, kb);
    }
  }
  // wavefronts 1.. of an item hand their (max, sum, O) to wavefront 0 through LDS
  if (half > 0) {
    sm[sub][half - 1][lane] = mrun;
    sl[sub][half - 1][lane] = lrun;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) sO[sub][half - 1][dt][lane] = O[dt];
  }
  __syncthreads();
  if (half == 0 && valid) {
    float m = mrun;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w) m = fmaxf(m, sm[sub][w][lane]);
    const float f0 = __builtin_amdgcn_exp2f(mrun - m);
    float fw[NW - 1];
    float l = lrun * f0;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w) {
      fw[w] = __builtin_amdgcn_exp2f(sm[sub][w][lane] - m);
      l += sl[sub][w][lane] * fw[w];
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      f32x4 o = O[dt] * f0;
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) o += sO[sub][w][dt][lane] * fw[w];
      o *= inv;
      const int fo = head * D + dt * 16 + 4 * g;
      const uint32_t lo = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
      const uint32_t hi = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
      *reinterpret_cast<uint64_t*>(a.out + xp_index(row, fo, a.MTc)) = (uint64_t)lo | ((uint64_t)hi << 32);
    }
  }
}

}  // namespace bd
