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
    // Quadratic forward: most blocks of the forward's own rows hold no key that any row of this tile sees (a row sees
    // its own group, a group's first row the first rows of the groups before it); they would add exact zeros.
    [[maybe_unused]] const int W = (a.mode >> 8) + 1;
    [[maybe_unused]] const int r0 = qt * 16, r1 = min(qt * 16 + 15, a.Mvalid - 1);
    [[maybe_unused]] const int g_lo = r0 / W, g_hi = r1 / W;
    auto needed = [&](int kb) -> bool {
      if constexpr (!QUAD) return true;
      const int jb0 = kb * 32 - a.n0;                              // the block's first key, counted from the forward's first row
      if (jb0 < 0) return true;                                    // keys of the prefix
      if (jb0 < (g_hi + 1) * W && jb0 + 31 >= g_lo * W) return true;   // keys of a group of the tile's rows
      if (g_hi * W < r0) return false;                             // no group's first row in the tile
      const int first = (jb0 + W - 1) / W * W;                     // the first group-first key at or after jb0
      return first <= jb0 + 31 && first <= g_hi * W;
    };
    KvBlock<D> b0;
    for (int j = 0; j < cnt; ++j) {
      const int kb = half + NW * j;
      if (!needed(kb)) continue;
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

// The same for forwards of at most 64 rows, where few items would leave most CUs idle and every item would walk all keys
// of its kv head at one CU's load rate: a workgroup takes JT query tiles of one head (they share every key/value block
// it loads) and one of n_chunks key chunks (block kb belongs to chunk kb mod n_chunks, and inside the workgroup to
// wavefront (kb / n_chunks) mod 4), and leaves an unnormalised partial per tile (sum, maximum, sum of weights) in
// a.part; pf_attn_merge_kernel sums the chunks.  Measured at 64 rows against 2112 keys (split + merge kernel, us per
// layer): 1 tile x 4 chunks 7.6 + 3.2, 1 x 8: 8.4 + 3.4, 2 x 8: 9.8 + 3.7, 4 x 8 and 2 x 16: 14.7 + 4.4, 1 x 2: 12.3 + 3.9;
// the unsplit kernel with eight wavefronts per item: 16.7.  Sharing key/value loads among tiles does not pay: a
// wavefront's time goes into the dependent chain of each block's products and softmax, not into its loads.
template <int D, int JT, bool QUAD = false>
__global__ __launch_bounds__(256, JT > 1 ? 1 : 2) void pf_attn_split_kernel(PfAttnArgs a) {
  constexpr int DS = D / 32, DT = D / 16, NW = 4;
  __shared__ f32x4 sO[NW - 1][DT][64];
  __shared__ float sm[NW - 1][64], sl[NW - 1][64];
  if (a.skippable && a.st->skip) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const int G = a.n_q / a.n_kv, QT = a.Mc >> 4, TG = (QT + JT - 1) / JT;
  const int n_chunks = a.n_chunks;
  const int chunk = blockIdx.x % n_chunks, grp = blockIdx.x / n_chunks;
  const int hq = grp % G, tg = (grp / G) % TG, kvh = grp / (G * TG);
  const int head = kvh * G + hq;
  const size_t kv_block = (size_t)32 * D / 8;
  const bf16x8* Kh = reinterpret_cast<const bf16x8*>(a.Kc) + (size_t)kvh * a.max_kb * kv_block;
  const bf16x8* Vh = reinterpret_cast<const bf16x8*>(a.Vc) + (size_t)kvh * a.max_kb * kv_block;
  bf16x8 qf[JT][DS];
  f32x4 O[JT][DT];
  float mrun[JT], lrun[JT];
  int row[JT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt) {
    const int qt = min(tg * JT + jt, QT - 1);                  // (a group past the last tile repeats it and stores nothing)
    row[jt] = qt * 16 + col;
    const u16* qp = a.q + ((size_t)row[jt] * a.n_q + head) * D + 8 * g;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) qf[jt][ds] = *reinterpret_cast<const bf16x8*>(qp + ds * 32);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[jt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    mrun[jt] = kNegBig;
    lrun[jt] = 0.f;
  }
  {
    // blocks holding a key some row of the group may see: up to its last row (causal), else all of the chunk
    const int last_row = min(min(tg * JT + JT - 1, QT - 1) * 16 + 15, a.Mvalid - 1);
    const int kb_end = (a.n0 + (a.mode == 1 ? last_row : a.Mvalid - 1)) / 32 + 1;
    const int first = wave * n_chunks + chunk, step = NW * n_chunks;
    const int cnt = kb_end > first ? (kb_end - first + step - 1) / step : 0;
    const float c = a.scale_log2e;
    auto block = [&](const KvBlock<D>& b, int kb) {
      if (kb * 32 + 31 >= a.n0) {
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
          attn_block<D, true, QUAD>(b, qf[jt], O[jt], mrun[jt], lrun[jt], kb, a.n0, a.Mvalid, a.mode, row[jt], g, c);
      } else {
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
          attn_block<D, false>(b, qf[jt], O[jt], mrun[jt], lrun[jt], kb, a.n0, a.Mvalid, a.mode, row[jt], g, c);
      }
    };
    // (one register buffer: loading the next block ahead into a second one measured slower here as in pf_attn_kernel)
    KvBlock<D> b0;
    for (int j = 0; j < cnt; ++j) {
      const int kb = first + step * j;
      kv_load<D>(b0, Kh, Vh, kb, lane, a.pages);
      asm volatile("" ::: "memory");
      block(b0, kb);
    }
  }
  // tile by tile: wavefronts 1..3 hand their (max, sum, O) to wavefront 0 through LDS, which stores the chunk's partial
#pragma unroll
  for (int jt = 0; jt < JT; ++jt) {
    if (wave > 0) {
      sm[wave - 1][lane] = mrun[jt];
      sl[wave - 1][lane] = lrun[jt];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) sO[wave - 1][dt][lane] = O[jt][dt];
    }
    __syncthreads();
    const int qt = tg * JT + jt;
    if (wave == 0 && qt < QT) {
      float m = mrun[jt];
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) m = fmaxf(m, sm[w][lane]);
      const float f0 = __builtin_amdgcn_exp2f(mrun[jt] - m);
      float fw[NW - 1];
      float l = lrun[jt] * f0;
#pragma unroll
      for (int w = 0; w < NW - 1; ++w) {
        fw[w] = __builtin_amdgcn_exp2f(sm[w][lane] - m);
        l += sl[w][lane] * fw[w];
      }
      const int item = (kvh * QT + qt) * G + hq;
      float* pp = a.part + (size_t)(item * n_chunks + chunk) * (DT * 256 + 128);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        f32x4 o = O[jt][dt] * f0;
#pragma unroll
        for (int w = 0; w < NW - 1; ++w) o += sO[w][dt][lane] * fw[w];
        *reinterpret_cast<f32x4*>(pp + (dt * 64 + lane) * 4) = o;
      }
      pp[DT * 256 + lane] = m;
      pp[DT * 256 + 64 + lane] = l;
    }
    if (jt + 1 < JT) __syncthreads();
  }
}

// The chunks of every item summed in chunk order (fixed: same bits on every run): one wavefront per (item, d tile),
// all of its loads issued before the first is used.
template <int D, int NC>
__global__ __launch_bounds__(256) void pf_attn_merge_kernel(PfAttnArgs a) {
  constexpr int DT = D / 16;
  if (a.skippable && a.st->skip) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 15, g = lane >> 4;
  const int G = a.n_q / a.n_kv, QT = a.Mc >> 4;
  const int item = blockIdx.x / (DT / 4), dt = (blockIdx.x % (DT / 4)) * 4 + wave;
  const int hq = item % G, qt = (item / G) % QT, kvh = item / (G * QT);
  const int head = kvh * G + hq;
  const int row = qt * 16 + col;
  const float* base = a.part + (size_t)item * NC * (DT * 256 + 128);
  float mc[NC], lc[NC];
  f32x4 oc[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const float* pp = base + (size_t)c * (DT * 256 + 128);
    mc[c] = pp[DT * 256 + lane];
    lc[c] = pp[DT * 256 + 64 + lane];
    oc[c] = *reinterpret_cast<const f32x4*>(pp + (dt * 64 + lane) * 4);
  }
  float m = kNegBig;
#pragma unroll
  for (int c = 0; c < NC; ++c) m = fmaxf(m, mc[c]);
  float l = 0.f;
  f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const float f = __builtin_amdgcn_exp2f(mc[c] - m);
    l += lc[c] * f;
    o += oc[c] * f;
  }
  o *= 1.f / l;
  const int fo = head * D + dt * 16 + 4 * g;
  const uint32_t lo = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
  const uint32_t hi = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
  *reinterpret_cast<uint64_t*>(a.out + xp_index(row, fo, a.MTc)) = (uint64_t)lo | ((uint64_t)hi << 32);
}

}  // namespace bd
