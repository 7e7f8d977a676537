// The whole decoder forward as ONE persistent kernel (one workgroup per compute unit).
//
// Why: a block-denoising step at B<=64 is a chain of ~180 small dependent operations whose only real
// cost is streaming 6.2 GB of weights; launched one by one they spend more time between kernels than
// in them.  Here every compute unit owns a fixed slice of every weight matrix, laid out in HBM in the
// exact order it will read it (one sequential stream per wavefront), and walks through the phases of
// every layer with grid-wide barriers in between.  The first chunk of the next phase's weights is
// requested before a barrier is entered, so HBM keeps streaming while the barrier and the activation
// hand-over are in flight.
//
// Phases of a layer (dependencies force a grid barrier after each):
//   QKV   RMSNorm-on-load + [Q|K|V] projection + rotary + Q store + KV-cache write
//   ATT   block-causal attention over the cache (split over key chunks, last arriver merges)
//   O     output projection + residual + per-tile sum of squares for the next norm
//   GU    RMSNorm-on-load + gate/up projection + SwiGLU
//   DOWN  down projection, K split over workgroups, last arriver reduces + residual + sum of squares
// and after the last layer  LM: RMSNorm-on-load + LM head + per-row (max, argmax, sum exp).
//
// Cross-workgroup data discipline (no cache flushes or invalidations inside the kernel):
//   * every buffer that one workgroup writes and another reads is written with write-through
//     (agent-scope) stores and is written at most once per forward, in a phase that ends before any
//     phase that reads it; so no L1/L2 of any XCD can hold a stale copy, and plain loads are safe;
//   * a workgroup signals (barrier arrival, split-K counters) only after its stores have completed
//     (s_waitcnt on the in-order vector-memory counter).
#pragma once
#include "common.h"
#include "plan.h"

namespace bd {

// ---- write-through stores and ordered waits ---------------------------------------------------------------
__device__ inline void st_wt_u32(void* p, uint32_t v) {
  __hip_atomic_store(reinterpret_cast<uint32_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_wt_u16(void* p, u16 v) {
  __hip_atomic_store(reinterpret_cast<u16*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_wt_u64(void* p, uint64_t v) {
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_wt_f32(void* p, float v) {
  __hip_atomic_store(reinterpret_cast<float*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_wt_f32x4(void* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
// ---- grid barrier --------------------------------------------------------------------------------------
// Two-level arrival counters (groups of 16 workgroups, one 128-byte line per counter), release words per
// group.  Counters only grow; `epoch` numbers the barriers of the whole process.  Bounded spin: on
// time-out the device error flag is set and every later barrier of this launch returns at once.
// Layout of `bar`: [0] top counter, [32*(1+g)] group counters, [32*(1+ng+g)] release words.
__device__ inline bool grid_barrier(unsigned* bar, unsigned epoch, int nwg, DevState* st, int* s_flag) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int ok = 1;
    if (*s_flag != 0) {
      const int ng = (nwg + kBarGroup - 1) / kBarGroup;
      const int g = blockIdx.x / kBarGroup;
      const int gsize = min(kBarGroup, nwg - g * kBarGroup);
      unsigned* gcnt = bar + 32 * (1 + g);
      unsigned* rel = bar + 32 * (1 + ng);
      const unsigned old = __hip_atomic_fetch_add(gcnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == epoch * (unsigned)gsize - 1u) {
        const unsigned o2 = __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (o2 == epoch * (unsigned)ng - 1u)
          for (int r = 0; r < ng; ++r)
            __hip_atomic_store(rel + 32 * r, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      const unsigned* mine = rel + 32 * g;
      int spins = 0;
      while ((int)(__hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) < 0) {
        if (++spins > kSpinLimit) { ok = 0; break; }
        __builtin_amdgcn_s_sleep(2);
      }
      if (!ok) {
        __hip_atomic_store(&st->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = 0;
      }
    }
  }
  __syncthreads();
  return *s_flag != 0;
}

// A launch that is skipped on the device (a step of a block that is already complete) still owes the barrier
// counters the arrivals the host has counted for it: per chip-wide barrier one arrival of every workgroup on its
// group counter and one of every group on the top counter, per XCD barrier one arrival of every workgroup on its XCD's
// counter.  The release words stay behind; the next real barrier overwrites them with a larger epoch.
__device__ inline void skip_barriers(unsigned* bar, unsigned* xbar, unsigned n_global, unsigned n_xcd) {
  if (threadIdx.x != 0) return;
  const int g = blockIdx.x / kBarGroup;
  __hip_atomic_fetch_add(bar + 32 * (1 + g), n_global, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (blockIdx.x % kBarGroup == 0) __hip_atomic_fetch_add(bar, n_global, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (n_xcd != 0u) __hip_atomic_fetch_add(xbar + 32 * (blockIdx.x % 8), n_xcd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- weight stream cursor ----------------------------------------------------------------------------------
// All streamed operands are fetched with raw buffer loads: an out-of-range offset returns zeros and moves
// no data, so the inner loops are straight-line code (every position of a chunk is always "loaded" and
// multiplied; positions a wavefront does not have read as zero) and the compiler's in-order wait counts
// stay exact.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
constexpr int kOob = -1;                                // offset 0xFFFFFFFF: beyond any buffer
constexpr int kAuxNt = 2;                               // non-temporal (streamed once)

__device__ inline rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline bf16x8 buf_load_w(rsrc_t r, int byte_off) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kAuxNt));
}
__device__ inline bf16x8 buf_load_b(rsrc_t r, int byte_off) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
}
__device__ inline f32x4 buf_load_f(rsrc_t r, int byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0));
}

struct ChunkRef {
  int off;             // byte offset of the chunk in this wavefront's stream
  int KW, R0, R1;      // k-steps; rows of the chunk's first / second tile (R1 = 0: single tile); KW = 0: none
};

struct Cursor {
  int pos;             // byte offset in the wavefront's stream
  int l, p, c, wg, w, want_lm;
  __device__ ChunkRef next(const MegaPlan& P) {
    ChunkRef r;
    r.off = 0; r.KW = 0; r.R0 = 0; r.R1 = 0;
    while (p != PH_END) {
      // (the cursor serves the bf16 layers kernel and the LM head: neither sees cut gate/up tiles)
      const WavePhase wp = wave_phase_t<false>(P, p, wg, w);
      const int n_tiles = (wp.rows + 15) >> 4;
      const int n_chunks = (n_tiles + 1) >> 1;
      if (c < n_chunks && wp.KW > 0) {
        r.off = pos;
        r.KW = wp.KW;
        r.R0 = min(16, wp.rows - 32 * c);
        r.R1 = (2 * c + 1 < n_tiles) ? min(16, wp.rows - 32 * c - 16) : 0;
        pos += wp.KW * (r.R0 + r.R1) * 32 * P.ph[p].wbytes;
        ++c;
        return r;
      }
      c = 0;
      if (p == PH_DOWN) {
        ++l;
        p = (l < P.L) ? PH_QKV : (want_lm ? PH_LM : PH_END);
      } else if (p == PH_LM) {
        p = PH_END;
      } else {
        ++p;
      }
    }
    return r;
  }
};

// Per-lane byte offsets of the two tiles of a chunk at k-step 0, and the k-step stride.
struct ChunkLane { int o0, o1, step, KW; };
__device__ inline ChunkLane chunk_lane(const ChunkRef& r, int lane) {
  const int i = lane & 15, kq = lane >> 4;
  ChunkLane cl;
  cl.KW = r.KW;
  cl.step = (r.R0 + r.R1) * 64;
  cl.o0 = r.off + (kq * r.R0 + min(i, max(r.R0 - 1, 0))) * 16;
  cl.o1 = r.R1 > 0 ? r.off + (r.R0 * 4 + kq * r.R1 + min(i, r.R1 - 1)) * 16 : kOob;
  return cl;
}
__device__ inline int chunk_off(const ChunkLane& cl, int ksl, int t) {
  const int base = t ? cl.o1 : cl.o0;
  return (ksl < cl.KW && base != kOob) ? base + ksl * cl.step : kOob;
}

// Always 32 load instructions, whatever the chunk's shape.
__device__ inline void load_chunk(bf16x8 (&buf)[kMaxKW][kT], rsrc_t wr, const ChunkRef& r, int lane) {
  const ChunkLane cl = chunk_lane(r, lane);
#pragma unroll
  for (int ksl = 0; ksl < kMaxKW; ++ksl) {
    buf[ksl][0] = buf_load_w(wr, chunk_off(cl, ksl, 0));
    buf[ksl][1] = buf_load_w(wr, chunk_off(cl, ksl, 1));
  }
}

// ---- activation fragments ----------------------------------------------------------------------------------
// RMSNorm around the GEMM: the gain is folded into the weight columns when they are packed, the bf16
// copy of the residual version is the B operand as it is, and the per-row factor rsqrt(mean square + eps)
// (from the per-tile partial sums of squares) multiplies the accumulators in the epilogue.
// The fragments of a wavefront's k-steps are staged in a wavefront-private LDS region ([k-step][mt][lane]),
// four k-steps per batch (all loads of a batch are in flight together), and read back one k-step at a
// time.  K-steps the wavefront does not have read as zero.
template <int MT>
__device__ inline void stage_x_packed(bf16x8* xs, rsrc_t xr, int ks0, int nk, int slots, int lane) {
  for (int j0 = 0; j0 < slots; j0 += 4) {
    bf16x8 v[4][MT];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        v[jj][mt] = buf_load_b(xr, j0 + jj < nk ? (((ks0 + j0 + jj) * MT + mt) * 64 + lane) * 16 : kOob);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) xs[((j0 + jj) * MT + mt) * 64 + lane] = v[jj][mt];
  }
}

// Store channels r .. r+n-1 (n = 2 or 4) of one token into the packed bf16 copy of a residual version.
__device__ inline void store_xb(u16* xb, int token, int r, int n, const float* o, int MT) {
  if (n == 4 && (r & 3) == 0) {
    const uint32_t lo = (uint32_t)f32_to_bf16_bits(o[0]) | ((uint32_t)f32_to_bf16_bits(o[1]) << 16);
    const uint32_t hi = (uint32_t)f32_to_bf16_bits(o[2]) | ((uint32_t)f32_to_bf16_bits(o[3]) << 16);
    st_wt_u64(xb + xp_index(token, r, MT), (uint64_t)lo | ((uint64_t)hi << 32));
  } else {
    for (int e = 0; e < n; ++e) st_wt_u16(xb + xp_index(token, r + e, MT), f32_to_bf16_bits(o[e]));
  }
}

// ---- one GEMM phase ------------------------------------------------------------------------------------------
struct PhaseCtx {
  int layer, n;             // layer index, committed context length
  int pg[3];                // pages of the blocks that hold positions n .. n+63 (the new rows' keys and values)
  f32x4* red;               // LDS [4][kT*MT][64]
  bf16x8* xstage;           // LDS, activation fragments: [4 wavefronts][XH][MT][64]
  int* s_flags;             // LDS scratch ints
};

// Epilogue operands a caller may have fetched ahead of the product (use_pre false: the epilogue loads them itself).
struct EpiPre {
  float2 cs[2];   // QKV: (cos, sin) of this lane's two rotary pairs
  f32x4 xo;       // O: the four residual values this lane adds to
  f32x4 gn;       // O (fp8 weights): gains of the next norm for this lane's four channels
};

// DC: head dimension when the caller knows it at compile time (0: taken from the plan).
// USE_PRE: `pre` holds this element's operands.  Either way every load of the epilogue is issued before its
// first store: a load behind a write-through store would have to wait for that store's acknowledgement.
template <int MT, int PH, int DC = 0, bool USE_PRE = false>
__device__ inline void gemm_epilogue(const MegaArgs& a, const PhaseCtx& pc, const WavePhase& wp, int c, int t, int mt, f32x4 v, int lane,
                                     float (&rmax)[MT], int (&ridx)[MT], float (&rsum)[MT], const EpiPre pre = EpiPre{}) {
  const MegaPlan& P = a.P;
  const int col = lane & 15, g = lane >> 4;
  const int token = mt * 16 + col;
  const int lr = (2 * c + t) * 16 + 4 * g;               // first of this lane's 4 rows, local to the row range
  const int r = wp.row0 + lr;                             // phase row
  const bool live = token < a.M && lr < wp.rows;          // rows come in pairs/quads only when rows % 4 == 0 ...
  const int nrows = min(4, wp.rows - lr);                 // ... so the last lane group may hold just 2 valid rows
  if constexpr (PH == PH_QKV) {
    if (!live) return;
    const int D = DC ? DC : P.D, half = D >> 1;
    const int rel = ((pc.n + token) >> 5) - (pc.n >> 5);    // which of the (at most three) blocks of the new rows
    const int key = ((rel == 0 ? pc.pg[0] : rel == 1 ? pc.pg[1] : pc.pg[2]) << 5) | ((pc.n + token) & 31);   // in its page
    float2 csv[2];
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      if constexpr (USE_PRE) {
        csv[pr] = pre.cs[pr];
      } else {
        const int rp = r + 2 * pr;
        csv[pr] = (2 * pr < nrows && rp < P.QD + P.KVD) ? a.rope[(size_t)token * half + ((rp % D) >> 1)] : make_float2(0.f, 0.f);
      }
    }
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      if (2 * pr >= nrows) break;
      const int rp = r + 2 * pr;                          // even phase row; (rp, rp+1) is a pair
      if (rp < P.QD + P.KVD) {
        // rotary pair: phase rows (2i, 2i+1) of a head hold dims (i, i + D/2)
        const int dp = rp % D;
        const float2 cs = csv[pr];
        const float lo = v[2 * pr] * cs.x - v[2 * pr + 1] * cs.y;
        const float hi = v[2 * pr + 1] * cs.x + v[2 * pr] * cs.y;
        const uint32_t pk = (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
        if (rp < P.QD) {
          st_wt_u32(a.Q + (((size_t)pc.layer * a.Mp + token) * P.n_q + rp / D) * D + dp, pk);
        } else {
          const int rk = rp - P.QD;
          u16* kc = a.Kc + (size_t)pc.layer * a.kv_layer_elems + (size_t)(rk / D) * a.max_kb * 32 * D;
          st_wt_u32(kc + kp_index(key, dp, D / 32), pk);
        }
      } else {
        const int rv = rp - P.QD - P.KVD;
        u16* vc = a.Vc + (size_t)pc.layer * a.kv_layer_elems + (size_t)(rv / D) * a.max_kb * 32 * D;
        st_wt_u16(vc + vp_index(key, rv % D, D / 16), f32_to_bf16_bits(v[2 * pr]));
        st_wt_u16(vc + vp_index(key, (rv + 1) % D, D / 16), f32_to_bf16_bits(v[2 * pr + 1]));
      }
    }
  } else if constexpr (PH == PH_O) {
    // x_new = x_old + o ; partial sum of squares of this tile's channels
    const int ver = 2 * pc.layer + 1;
    float ss = 0.f;
    if (live) {
      const float* xo = a.xv + ((size_t)(ver - 1) * a.Mp + token) * P.H + r;
      float* xn = a.xv + ((size_t)ver * a.Mp + token) * P.H + r;
      float o[4] = {0.f, 0.f, 0.f, 0.f};
      if (nrows == 4 && (r & 3) == 0) {
        const f32x4 ov = (USE_PRE ? pre.xo : *reinterpret_cast<const f32x4*>(xo)) + v;
        st_wt_f32x4(xn, ov);
        for (int e = 0; e < 4; ++e) o[e] = ov[e];
      } else {
        for (int e = 0; e < nrows; ++e) { o[e] = xo[e] + v[e]; st_wt_f32(xn + e, o[e]); }
      }
      ss = o[0] * o[0] + o[1] * o[1] + o[2] * o[2] + o[3] * o[3];
      if (a.fp8) {
        if constexpr (USE_PRE) { for (int e = 0; e < 4; ++e) o[e] *= pre.gn[e]; }
        else { for (int e = 0; e < nrows; ++e) o[e] *= a.gains[(size_t)ver * P.H + r + e]; }
      }
      store_xb(a.xb + (size_t)ver * a.xb_elems, token, r, nrows, o, a.MT);
    }
    ss += __shfl_xor(ss, 16);
    ss += __shfl_xor(ss, 32);
    if (g == 0)
      st_wt_f32(a.ssq + ((size_t)ver * a.ssq_parts + (size_t)blockIdx.x * phase_tpg(P.ph[PH_O]) + 2 * c + t) * a.Mp + token, ss);
  } else if constexpr (PH == PH_GU) {
    if (!live) return;
    // rows (2f, 2f+1) = (gate f, up f)
    u16* base = a.act + (size_t)pc.layer * a.act_elems;
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      if (2 * pr >= nrows) break;
      const float gt = v[2 * pr], up = v[2 * pr + 1];
      const u16 hv = f32_to_bf16_bits(gt / (1.f + __expf(-gt)) * up);
      if (a.local_gu) base[xp_index(token, (r >> 1) + pr, a.MT)] = hv;      // read only inside this XCD: its L2 is coherent
      else st_wt_u16(base + xp_index(token, (r >> 1) + pr, a.MT), hv);
    }
  } else if constexpr (PH == PH_DOWN) {
    // partial tile of this K group, in fragment order
    if (lr < wp.rows) {
      const int tiles = phase_tile_slots(P, PH_DOWN);
      const int gt = wp.ng * phase_tpg(P.ph[PH_DOWN]) + 2 * c + t;
      float* dst = a.wsD + (size_t)pc.layer * a.wsD_layer_floats +
                   ((((size_t)wp.kg * tiles + gt) * a.MT + mt) * 64 + lane) * 4;
      st_wt_f32x4(dst, v);
    }
  } else {  // PH_LM
    if (lr < wp.rows) {
      if (a.logits != nullptr && token < a.M) {
        float* dst = a.logits + (size_t)token * P.V + r;
        for (int e = 0; e < nrows; ++e) dst[e] = v[e];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (e < nrows) stat_merge(rmax[mt], ridx[mt], rsum[mt], v[e], r + e, 1.f);
    }
  }
}

// Down projection: the last of the ksplit workgroups to finish a tile sums all partials in fixed order,
// adds the residual, stores the new residual version and its per-tile sum of squares.
template <int MT>
__device__ inline bool down_finalize(const MegaArgs& a, const PhaseCtx& pc, const WavePhase& wp, int wave, int lane) {
  const MegaPlan& P = a.P;
  const int ksplit = P.ph[PH_DOWN].ksplit;
  const int tiles = phase_tile_slots(P, PH_DOWN);
  const int my_tiles = (wp.rows + 15) >> 4;
  const int gt0 = wp.ng * phase_tpg(P.ph[PH_DOWN]);
  __syncthreads();
  if ((int)threadIdx.x < my_tiles) {
    int last = 1;
    if (ksplit > 1) {
      const unsigned old = __hip_atomic_fetch_add(a.cntD + (size_t)pc.layer * tiles + gt0 + threadIdx.x, 1u,
                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      last = old == (unsigned)ksplit - 1u;
    }
    pc.s_flags[8 + threadIdx.x] = last;
  }
  __syncthreads();
  const int col = lane & 15, g = lane >> 4;
  const int ver = 2 * pc.layer + 2;
  bool stored = false;
  for (int idx = wave; idx < my_tiles * MT; idx += kWavesPerWG) {
    const int tl = idx / MT, mt = idx % MT;
    if (!pc.s_flags[8 + tl]) continue;
    const int gt = gt0 + tl;
    const float* src = a.wsD + (size_t)pc.layer * a.wsD_layer_floats;
    f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int kg = 0; kg < ksplit; ++kg)
      v += *reinterpret_cast<const f32x4*>(src + ((((size_t)kg * tiles + gt) * a.MT + mt) * 64 + lane) * 4);
    const int token = mt * 16 + col;
    const int lr = tl * 16 + 4 * g;
    const int r = wp.row0 + lr;
    const int nrows = min(4, wp.rows - lr);
    float ss = 0.f;
    if (token < a.M && nrows > 0) {
      const float* xo = a.xv + ((size_t)(ver - 1) * a.Mp + token) * P.H + r;
      float* xn = a.xv + ((size_t)ver * a.Mp + token) * P.H + r;
      float o[4] = {0.f, 0.f, 0.f, 0.f};
      if (nrows == 4 && (r & 3) == 0) {
        const f32x4 ov = *reinterpret_cast<const f32x4*>(xo) + v;
        st_wt_f32x4(xn, ov);
        for (int e = 0; e < 4; ++e) o[e] = ov[e];
      } else {
        for (int e = 0; e < nrows; ++e) { o[e] = xo[e] + v[e]; st_wt_f32(xn + e, o[e]); }
      }
      store_xb(a.xb + (size_t)ver * a.xb_elems, token, r, nrows, o, a.MT);
      ss = o[0] * o[0] + o[1] * o[1] + o[2] * o[2] + o[3] * o[3];
    }
    ss += __shfl_xor(ss, 16);
    ss += __shfl_xor(ss, 32);
    if (g == 0) st_wt_f32(a.ssq + ((size_t)ver * a.ssq_parts + gt) * a.Mp + token, ss);
    stored = true;
  }
  return stored;
}

// Sum the per-tile partial sums of squares of a residual version into rsqrt(mean square + eps) per row,
// with all 256 threads (fixed summation order), result in LDS.
__device__ inline void row_scales_lds(float* s_part, float* s_rs, const float* ssq, int parts, int Mp, int rows, int H,
                                      float eps) {
  const int slices = kWGThreads / rows;                 // rows is 16, 32, 48 or 64
  const int row = threadIdx.x % rows, slice = threadIdx.x / rows;
  if (slice < slices) {
    float s = 0.f;
    for (int p0 = slice; p0 < parts; p0 += 16 * slices) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int p = p0 + u * slices;
        v[u] = ssq[(size_t)min(p, parts - 1) * Mp + row];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) s += (p0 + u * slices < parts) ? v[u] : 0.f;
    }
    s_part[slice * rows + row] = s;
  }
  __syncthreads();
  if ((int)threadIdx.x < rows) {
    float t = 0.f;
    for (int sl = 0; sl < slices; ++sl) t += s_part[sl * rows + threadIdx.x];
    s_rs[threadIdx.x] = rsqrtf(t / (float)H + eps);
  }
  __syncthreads();
}

// One GEMM phase of one workgroup.  `ring` holds the current chunk of this wavefront's weight stream
// (requested earlier).  While a chunk is multiplied, every consumed fragment is at once replaced by the
// same position of the next chunk; only for the last chunk of the phase the refill (first chunk of the
// next GEMM phase) is issued after the epilogue's stores, so that "stores done" can be awaited without
// waiting for it.
template <int MT, int PH>
__device__ inline void gemm_phase(const MegaArgs& a, const PhaseCtx& pc, bf16x8 (&ring)[kMaxKW][kT], Cursor& cur,
                                  int wave, int lane_in) {
  // Re-define the lane id opaquely so that nothing derived from it is hoisted out of the layer loop
  // (five phases' worth of loop-invariant addresses would otherwise live in registers all the time).
  int lane = lane_in;
  asm volatile("" : "+v"(lane));
  constexpr int XH = (MT <= 2) ? kMaxKW : 4;          // k-steps of activation fragments staged at a time
  bf16x8* xs = pc.xstage + (size_t)wave * (XH * MT * 64);
  const MegaPlan& P = a.P;
  const WavePhase wp = wave_phase_t<false>(P, PH, blockIdx.x, wave);
  const int n_tiles = (wp.rows + 15) >> 4;
  const int n_chunks = (n_tiles + 1) >> 1;
  float rmax[MT], rsum[MT];
  int ridx[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) { rmax[mt] = -INFINITY; ridx[mt] = 0x7FFFFFFF; rsum[mt] = 0.f; }

#define BD_SUBTS(k)                                                                                   \
  do {                                                                                                \
    if (a.trace2 != nullptr && pc.layer == 1 && threadIdx.x == 0 && PH < PH_LM)                        \
      a.trace2[(size_t)blockIdx.x * 64 + PH * 12 + (k)] = wall_clock64();                              \
  } while (0)
  BD_SUBTS(0);
  if (n_chunks > 0) {
    // activation source of this phase
    constexpr bool kNorm = (PH == PH_QKV || PH == PH_GU || PH == PH_LM);
    const int ver = (PH == PH_QKV) ? 2 * pc.layer : (PH == PH_GU) ? 2 * pc.layer + 1 : 2 * P.L;
    const rsrc_t wr = make_rsrc(a.wstream + (size_t)(blockIdx.x * kWavesPerWG + wave) * P.wave_stride,
                                (unsigned)(P.wave_stride * 16));
    const rsrc_t xr = kNorm ? make_rsrc(a.xb + (size_t)ver * a.xb_elems, (unsigned)(a.xb_elems * 2))
                            : (PH == PH_O ? make_rsrc(a.ap + (size_t)pc.layer * a.ap_elems, (unsigned)(a.ap_elems * 2))
                                          : make_rsrc(a.act + (size_t)pc.layer * a.act_elems, (unsigned)(a.act_elems * 2)));
    float rs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) rs[mt] = 1.f;
    if constexpr (kNorm) {
      const int parts = ver == 0 ? 1 : phase_tile_slots(P, (ver & 1) ? PH_O : PH_DOWN);
      float* s_part = reinterpret_cast<float*>(pc.red);
      float* s_rs = s_part + kWGThreads;
      row_scales_lds(s_part, s_rs, a.ssq + (size_t)ver * a.ssq_parts * a.Mp, parts, a.Mp, MT * 16, P.H, a.rms_eps);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) rs[mt] = s_rs[mt * 16 + (lane & 15)];
      BD_SUBTS(1);
      if constexpr (XH == kMaxKW) stage_x_packed<MT>(xs, xr, wp.w0, wp.KW, XH, lane);
    } else {
      BD_SUBTS(1);
      if constexpr (XH == kMaxKW) stage_x_packed<MT>(xs, xr, wp.w0, wp.KW, XH, lane);
    }
    BD_SUBTS(2);

    for (int c = 0; c < n_chunks; ++c) {
      const bool last = c == n_chunks - 1;
      const bool two = 2 * c + 1 < n_tiles;
      f32x4 acc[kT][MT];
#pragma unroll
      for (int t = 0; t < kT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (wp.KW > 0) {                                  // a wavefront without k-steps only joins the reduction
        ChunkRef nr;
        nr.off = 0; nr.KW = 0; nr.R0 = 0; nr.R1 = 0;   // last chunk: the in-place refills read nothing
        if (!last) nr = cur.next(P);
        const ChunkLane cl = chunk_lane(nr, lane);
#pragma unroll
        for (int ksl = 0; ksl < kMaxKW; ++ksl) {
          if constexpr (XH < kMaxKW) {
            if (ksl % XH == 0) {
              stage_x_packed<MT>(xs, xr, wp.w0 + ksl, wp.KW - ksl, XH, lane);
            }
          }
          bf16x8 xk[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) xk[mt] = xs[((ksl % XH) * MT + mt) * 64 + lane];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[0][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ring[ksl][0], xk[mt], acc[0][mt], 0, 0, 0);
          ring[ksl][0] = buf_load_w(wr, chunk_off(cl, ksl, 0));
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[1][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ring[ksl][1], xk[mt], acc[1][mt], 0, 0, 0);
          ring[ksl][1] = buf_load_w(wr, chunk_off(cl, ksl, 1));
        }
      }
      if (c < 3) BD_SUBTS(3 + 2 * c);
      // the four wavefronts hold disjoint K ranges: sum them through LDS in fixed order
#pragma unroll
      for (int t = 0; t < kT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) pc.red[(wave * (kT * MT) + t * MT + mt) * 64 + lane] = acc[t][mt];
      __syncthreads();
#pragma unroll
      for (int idx = 0; idx < kT * MT; ++idx) {
        if ((idx & 3) != wave) continue;
        const int t = idx / MT, mt = idx % MT;
        if (t == 1 && !two) continue;
        f32x4 v = pc.red[(0 * (kT * MT) + idx) * 64 + lane];
        v += pc.red[(1 * (kT * MT) + idx) * 64 + lane];
        v += pc.red[(2 * (kT * MT) + idx) * 64 + lane];
        v += pc.red[(3 * (kT * MT) + idx) * 64 + lane];
        if constexpr (kNorm) v *= rs[mt];              // RMSNorm's per-row factor commutes with the product
        gemm_epilogue<MT, PH>(a, pc, wp, c, t, mt, v, lane, rmax, ridx, rsum);
      }
      __syncthreads();
      if (c < 3) BD_SUBTS(4 + 2 * c);
      if (last && wp.KW > 0) {
        // request the first chunk of the next GEMM phase now, after this phase's stores, and wait only
        // for what is older than these 32 loads
        const ChunkRef nr = cur.next(P);
        asm volatile("" ::: "memory");
        load_chunk(ring, wr, nr, lane);
        asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
      }
    }
  }
  BD_SUBTS(9);
  if constexpr (PH == PH_DOWN) {
    if (down_finalize<MT>(a, pc, wp, wave, lane)) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  BD_SUBTS(10);
  if constexpr (PH == PH_LM) {
    // fold lane groups, then wavefronts, into this workgroup's row statistics
    const int col = lane & 15, g = lane >> 4;
    float* s_m = reinterpret_cast<float*>(pc.red);
    int* s_i = reinterpret_cast<int*>(pc.red) + 4 * 64;
    float* s_s = reinterpret_cast<float*>(pc.red) + 8 * 64;
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
        s_m[wave * 64 + mt * 16 + col] = rmax[mt];
        s_i[wave * 64 + mt * 16 + col] = ridx[mt];
        s_s[wave * 64 + mt * 16 + col] = rsum[mt];
      }
    }
    __syncthreads();
    if ((int)threadIdx.x < MT * 16) {
      const int tt = threadIdx.x;
      float m = s_m[tt];
      int i = s_i[tt];
      float s = s_s[tt];
      for (int w = 1; w < kWavesPerWG; ++w) stat_merge(m, i, s, s_m[w * 64 + tt], s_i[w * 64 + tt], s_s[w * 64 + tt]);
      st_wt_f32(a.lm_max + (size_t)blockIdx.x * a.Mp + tt, m);
      st_wt_u32(a.lm_idx + (size_t)blockIdx.x * a.Mp + tt, (uint32_t)i);
      st_wt_f32(a.lm_sum + (size_t)blockIdx.x * a.Mp + tt, s);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
}

// ---- attention phase ------------------------------------------------------------------------------------------
// Items (kv head, group of JT column tiles, key chunk) go round-robin over the workgroups.  Each item
// stores its partial (unnormalised output, running max, running sum); the workgroup that completes the
// last chunk of a (kv head, column group) merges all chunks in fixed order and stores the bf16 result.
template <int D, int JT, bool QUAD>
__device__ inline void attention_phase(const MegaArgs& a, const PhaseCtx& pc, char* lds, int wave, int lane_in) {
  constexpr int DS = D / 32, DT = D / 16;
  int lane = lane_in;
  asm volatile("" : "+v"(lane));
  const MegaPlan& P = a.P;
  f32x4* sO = reinterpret_cast<f32x4*>(lds);                               // [DT*JT][64]
  float* sm = reinterpret_cast<float*>(lds + DT * JT * 64 * 16);           // [4][JT*16]
  float* sl = sm + kWavesPerWG * JT * 16;                                   // [4][JT*16]
  float* wgt = sl + kWavesPerWG * JT * 16;                                  // [max 64 chunks][JT*16]

  const int col = lane & 15, g = lane >> 4;
  const int n = pc.n;
  const int G = P.n_q / P.n_kv;
  const int Mp = a.MT * 16;
  const int n_jg = (G * a.MT) / JT;
  int n_kb, chunk_len, n_chunks;
  attn_chunks(n + a.M, a.attn_max_chunks, n_kb, chunk_len, n_chunks);
  const int n_groups = P.n_kv * n_jg;
  const int n_items = n_groups * n_chunks;
  const size_t kv_block = (size_t)32 * D / 8;
  const u16* Qb = a.Q + (size_t)pc.layer * a.Mp * P.n_q * D;
  float* pO = a.pO + (size_t)pc.layer * a.pO_layer_floats;
  float* pm = a.pm + (size_t)pc.layer * a.pml_layer_floats;
  float* pl = a.pl + (size_t)pc.layer * a.pml_layer_floats;

  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int chunk = item % n_chunks;
    const int grp = item / n_chunks;
    const int jg = grp % n_jg, kvh = grp / n_jg;
    const bf16x8* Kh = reinterpret_cast<const bf16x8*>(a.Kc + (size_t)pc.layer * a.kv_layer_elems) + (size_t)kvh * a.max_kb * kv_block;
    const bf16x8* Vh = reinterpret_cast<const bf16x8*>(a.Vc + (size_t)pc.layer * a.kv_layer_elems) + (size_t)kvh * a.max_kb * kv_block;

    bf16x8 qf[JT][DS];
    int row[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      const int cidx = (jg * JT + jt) * 16 + col;
      const int hq = cidx / Mp, m = cidx - hq * Mp;
      row[jt] = m;
      const u16* qp = Qb + ((size_t)m * P.n_q + kvh * G + hq) * D + 8 * g;
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
      const int pb = page_of_block(a.kv_pages, __builtin_amdgcn_readfirstlane(kb));
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ds = 0; ds < DS; ++ds) kf[t][ds] = Kh[(((size_t)pb * 2 + t) * DS + ds) * 64 + lane];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) vf[dt] = Vh[((size_t)pb * DT + dt) * 64 + lane];
      const bool need_mask = (kb * 32 + 31) >= n;
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
        float v[8];
        bool vis[8];
        float cmax = kNegBig;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          v[e] = s[e >> 2][e & 3] * a.scale_log2e;
          vis[e] = true;
          if (need_mask) {
            const int jb = kb * 32 + 8 * g + e - n;
            vis[e] = (jb < 0) || (jb < a.M && block_key_visible<QUAD>(a.mode, row[jt], jb));
          }
          if (vis[e]) cmax = fmaxf(cmax, v[e]);
        }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32));
        const float mnew = fmaxf(mrun[jt], cmax);
        const float alpha = exp2f(mrun[jt] - mnew);
        float psum = 0.f;
        union { bf16x8 v8; u16 h[8]; } cv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p = vis[e] ? exp2f(v[e] - mnew) : 0.f;
          psum += p;
          cv.h[e] = f32_to_bf16_bits(p);
        }
        psum += __shfl_xor(psum, 16);
        psum += __shfl_xor(psum, 32);
        lrun[jt] = lrun[jt] * alpha + psum;
        mrun[jt] = mnew;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) O[dt][jt] *= alpha;
        pf[jt] = cv.v8;
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
          O[dt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[dt], pf[jt], O[dt][jt], 0, 0, 0);
    }
    // merge the four wavefronts
    if (g == 0) {
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
        sm[wave * JT * 16 + jt * 16 + col] = mrun[jt];
        sl[wave * JT * 16 + jt * 16 + col] = lrun[jt];
      }
    }
    __syncthreads();
    float mall[JT], lall[JT];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
      float mm = sm[jt * 16 + col];
#pragma unroll
      for (int w = 1; w < kWavesPerWG; ++w) mm = fmaxf(mm, sm[w * JT * 16 + jt * 16 + col]);
      float ll = 0.f;
#pragma unroll
      for (int w = 0; w < kWavesPerWG; ++w) ll += sl[w * JT * 16 + jt * 16 + col] * exp2f(sm[w * JT * 16 + jt * 16 + col] - mm);
      mall[jt] = mm;
      lall[jt] = ll;
      const float f = exp2f(mrun[jt] - mm);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) O[dt][jt] *= f;
    }
    for (int w = 0; w < kWavesPerWG; ++w) {
      if (wave == w) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int jt = 0; jt < JT; ++jt) {
            if (w == 0) sO[(dt * JT + jt) * 64 + lane] = O[dt][jt];
            else sO[(dt * JT + jt) * 64 + lane] += O[dt][jt];
          }
      }
      __syncthreads();
    }
    float* po = pO + (size_t)item * (DT * JT) * 64 * 4;
    for (int idx = wave; idx < DT * JT; idx += kWavesPerWG) st_wt_f32x4(po + ((size_t)idx * 64 + lane) * 4, sO[idx * 64 + lane]);
    if (wave == 0 && g == 0) {
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
        st_wt_f32(pm + (size_t)item * (JT * 16) + jt * 16 + col, mall[jt]);
        st_wt_f32(pl + (size_t)item * (JT * 16) + jt * 16 + col, lall[jt]);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
      const unsigned old = __hip_atomic_fetch_add(a.cntA + (size_t)pc.layer * n_groups + grp, 1u, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
      pc.s_flags[4] = old == (unsigned)n_chunks - 1u;
    }
    __syncthreads();
    if (pc.s_flags[4]) {
      // last arriver of this (kv head, column group): merge all chunks, every load of a round in flight at once
      constexpr int NC = JT * 16;                        // columns of the group
      constexpr int SL = kWGThreads / NC;                // threads per column
      const size_t item0 = (size_t)grp * n_chunks;
      float* s_red = wgt + 64 * NC;                      // [SL][NC]
      float* s_inv = s_red + SL * NC;                    // [NC]
      {
        const int cc = threadIdx.x % NC, sl = threadIdx.x / NC;
        constexpr int PER = 64 / SL;                     // chunks per thread (at most 64 chunks)
        float pmv[PER], plv[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
          const int ch = sl + u * SL;
          const int chc = min(ch, n_chunks - 1);
          pmv[u] = pm[(item0 + chc) * NC + cc];
          plv[u] = pl[(item0 + chc) * NC + cc];
        }
        float mx = kNegBig;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
          if (sl + u * SL >= n_chunks) { pmv[u] = kNegBig; plv[u] = 0.f; }
          mx = fmaxf(mx, pmv[u]);
        }
        s_red[sl * NC + cc] = mx;
        __syncthreads();
        float mm = kNegBig;
#pragma unroll
        for (int q = 0; q < SL; ++q) mm = fmaxf(mm, s_red[q * NC + cc]);
        __syncthreads();
        float lp = 0.f;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
          const int ch = sl + u * SL;
          const float w = exp2f(pmv[u] - mm);
          lp += plv[u] * w;
          if (ch < n_chunks) wgt[ch * NC + cc] = w;
        }
        s_red[sl * NC + cc] = lp;
        __syncthreads();
        if (sl == 0) {
          float ll = 0.f;
#pragma unroll
          for (int q = 0; q < SL; ++q) ll += s_red[q * NC + cc];
          s_inv[cc] = 1.f / ll;
        }
        __syncthreads();
      }
      const float* pg = pO + item0 * (DT * JT) * 64 * 4;
      u16* out = a.ap + (size_t)pc.layer * a.ap_elems;
      for (int idx = wave; idx < DT * JT; idx += kWavesPerWG) {
        const int dt = idx / JT, jt = idx % JT;
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int ch0 = 0; ch0 < n_chunks; ch0 += 8) {
          f32x4 v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int chc = min(ch0 + u, n_chunks - 1);
            v[u] = *reinterpret_cast<const f32x4*>(pg + (((size_t)chc * (DT * JT) + idx) * 64 + lane) * 4);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (ch0 + u < n_chunks) acc += v[u] * wgt[(ch0 + u) * NC + jt * 16 + col];
        }
        acc *= s_inv[jt * 16 + col];
        const int cidx = (jg * JT + jt) * 16 + col;
        const int hq = cidx / Mp, m = cidx - hq * Mp;
        if (m < a.M) {
          const int f = (kvh * G + hq) * D + dt * 16 + 4 * g;
          const uint32_t lo = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
          const uint32_t hi = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
          st_wt_u64(out + xp_index(m, f, a.MT), (uint64_t)lo | ((uint64_t)hi << 32));
        }
      }
    }
    __syncthreads();
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// ---- the kernel ------------------------------------------------------------------------------------------------
// Dynamic LDS of the forward kernel: [activation stage | K-reduction buffer]; the attention phase re-uses
// the front of it.
template <int MT> constexpr int mega_xh() { return (MT <= 2) ? kMaxKW : 4; }
template <int MT> constexpr int mega_lds_bytes() {
  return kWavesPerWG * mega_xh<MT>() * MT * 1024 + kWavesPerWG * kT * MT * 1024;
}

template <int MT, int D, int JT, bool QUAD = false>
__global__ __launch_bounds__(kWGThreads, 1) void mega_kernel(MegaArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ int s_flags[16];
  const MegaPlan& P = a.P;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave id in an SGPR: all branches on it are scalar
  if (threadIdx.x == 0) {
    int go = (a.st->error == 0);
    if (go && a.skippable && a.st->skip) {
      skip_barriers(a.bar, nullptr, 5u * (unsigned)P.L, 0u);
      go = 0;
    }
    s_flags[0] = go;
  }
  __syncthreads();
  if (!s_flags[0]) return;

  PhaseCtx pc;
  pc.n = a.st->n;
  for (int i = 0; i < 3; ++i) pc.pg[i] = page_of_block(a.kv_pages, min((pc.n >> 5) + i, a.max_kb - 1));
  pc.xstage = reinterpret_cast<bf16x8*>(lds);
  pc.red = reinterpret_cast<f32x4*>(lds + kWavesPerWG * mega_xh<MT>() * MT * 1024);
  pc.s_flags = s_flags;
  unsigned epoch = a.bar_epoch;

  Cursor cur;
  cur.pos = 0;
  cur.l = 0; cur.p = PH_QKV; cur.c = 0; cur.wg = blockIdx.x; cur.w = wave; cur.want_lm = 0;   // the LM head is its own launch
  bf16x8 ring[kMaxKW][kT];
  {
    const rsrc_t wr = make_rsrc(a.wstream + (size_t)(blockIdx.x * kWavesPerWG + wave) * P.wave_stride,
                                (unsigned)(P.wave_stride * 16));
    const ChunkRef r0 = cur.next(P);
    load_chunk(ring, wr, r0, lane);
  }
  bool alive = true;
  int tsi = 0;
#define BD_TS()                                                                                                  \
  do {                                                                                                           \
    if (a.trace != nullptr && threadIdx.x == 0) a.trace[(size_t)blockIdx.x * (10 * P.L + 4) + tsi] = wall_clock64(); \
    ++tsi;                                                                                                       \
  } while (0)
  BD_TS();
  for (int l = 0; l < P.L && alive; ++l) {
    pc.layer = l;
    gemm_phase<MT, PH_QKV>(a, pc, ring, cur, wave, lane);
    BD_TS();
    alive = grid_barrier(a.bar, ++epoch, P.nwg, a.st, &s_flags[0]);
    BD_TS();
    if (!alive) break;
    attention_phase<D, JT, QUAD>(a, pc, lds, wave, lane);
    BD_TS();
    alive = grid_barrier(a.bar, ++epoch, P.nwg, a.st, &s_flags[0]);
    BD_TS();
    if (!alive) break;
    gemm_phase<MT, PH_O>(a, pc, ring, cur, wave, lane);
    BD_TS();
    alive = grid_barrier(a.bar, ++epoch, P.nwg, a.st, &s_flags[0]);
    BD_TS();
    if (!alive) break;
    gemm_phase<MT, PH_GU>(a, pc, ring, cur, wave, lane);
    BD_TS();
    alive = grid_barrier(a.bar, ++epoch, P.nwg, a.st, &s_flags[0]);
    BD_TS();
    if (!alive) break;
    gemm_phase<MT, PH_DOWN>(a, pc, ring, cur, wave, lane);
    BD_TS();
    alive = grid_barrier(a.bar, ++epoch, P.nwg, a.st, &s_flags[0]);
    BD_TS();
  }
}

// LM head as its own launch of the same machinery: RMSNorm-on-load + LM head + per-row (max, argmax,
// sum exp) per workgroup, a grid barrier, then workgroup r folds row r over all workgroups.
template <int MT>
__global__ __launch_bounds__(kWGThreads, 1) void lm_kernel(MegaArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ int s_flags[16];
  const MegaPlan& P = a.P;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // wave id in an SGPR: all branches on it are scalar
  if (threadIdx.x == 0) {
    int go = (a.st->error == 0);
    if (go && a.skippable && a.st->skip) {
      skip_barriers(a.bar, nullptr, 1u, 0u);
      go = 0;
    }
    s_flags[0] = go;
  }
  __syncthreads();
  if (!s_flags[0]) return;
  PhaseCtx pc;
  pc.n = 0;
  pc.pg[0] = pc.pg[1] = pc.pg[2] = 0;
  pc.layer = P.L;
  pc.xstage = reinterpret_cast<bf16x8*>(lds);
  pc.red = reinterpret_cast<f32x4*>(lds + kWavesPerWG * mega_xh<MT>() * MT * 1024);
  pc.s_flags = s_flags;
  Cursor cur;
  cur.pos = (int)((long long)P.L * wave_layer_units(P, blockIdx.x, wave) * 16);
  cur.l = P.L; cur.p = PH_LM; cur.c = 0; cur.wg = blockIdx.x; cur.w = wave; cur.want_lm = 1;
  bf16x8 ring[kMaxKW][kT];
  {
    const rsrc_t wr = make_rsrc(a.wstream + (size_t)(blockIdx.x * kWavesPerWG + wave) * P.wave_stride,
                                (unsigned)(P.wave_stride * 16));
    const ChunkRef r0 = cur.next(P);
    load_chunk(ring, wr, r0, lane);
  }
  gemm_phase<MT, PH_LM>(a, pc, ring, cur, wave, lane);
  if (!grid_barrier(a.bar, a.bar_epoch + 1u, P.nwg, a.st, &s_flags[0])) return;
  if ((int)blockIdx.x < a.M) {
    const int r = blockIdx.x;
    float m = -INFINITY, s = 0.f;
    int i = 0x7FFFFFFF;
    for (int p = threadIdx.x; p < P.nwg; p += kWGThreads)
      stat_merge(m, i, s, a.lm_max[(size_t)p * a.Mp + r], a.lm_idx[(size_t)p * a.Mp + r], a.lm_sum[(size_t)p * a.Mp + r]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const float m2 = __shfl_xor(m, off);
      const int i2 = __shfl_xor(i, off);
      const float s2 = __shfl_xor(s, off);
      stat_merge(m, i, s, m2, i2, s2);
    }
    float* s_m = reinterpret_cast<float*>(lds);
    int* s_i = reinterpret_cast<int*>(lds) + 8;
    float* s_s = reinterpret_cast<float*>(lds) + 16;
    if (lane == 0) { s_m[wave] = m; s_i[wave] = i; s_s[wave] = s; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < kWavesPerWG; ++w) stat_merge(m, i, s, s_m[w], s_i[w], s_s[w]);
      a.row_cand[r] = i;
      a.row_conf[r] = 1.f / s;
    }
  }
}

}  // namespace bd
