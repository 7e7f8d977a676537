// The decoder forward as one persistent kernel with DECOUPLED weight streaming (block sizes up to 32).
//
// A block-denoising step at B <= 32 is bound by reading 5.5 GB of layer weights, but its ~180 dependent
// phases each end in a cross-chip hand-over (stores -> acknowledgement -> grid barrier -> loads) during
// which a compute wavefront cannot also keep HBM busy.  So every workgroup (one per compute unit) runs
// two kinds of wavefronts:
//   * four PRODUCERS, one per consumer, that do nothing but copy their consumer's weight stream from HBM
//     into a ring of 1-KiB slots in LDS with direct-to-LDS buffer loads (no registers involved).  The
//     stream is the sequence of 16-row x 32-k MFMA A-operand fragments in exactly the order the consumer
//     will multiply them, across all phases and layers, so the producer needs no knowledge of the
//     computation: it runs ahead whenever a slot is free, through barriers and attention phases alike;
//   * four CONSUMERS that hold the activations of their K range in registers, take weight fragments out
//     of the ring, multiply, reduce over the four K ranges through LDS, and run the fused epilogues,
//     the attention phase and the grid barriers.  Their own vector-memory counter only ever tracks the
//     small latency-critical loads and stores of the hand-over, never the bulk stream.
// Producer and consumer talk through two LDS words per ring ("landed", "consumed").  Because the producer
// wavefronts never reach a workgroup barrier, the consumers synchronise among themselves with an LDS
// arrival counter instead of s_barrier.
//
// Weight stream layout, activation buffers, epilogues and the cross-workgroup data discipline (write-once
// buffers, write-through stores, no cache maintenance inside the kernel) are those of mega.h; the two
// kernels are interchangeable on the same context.
#pragma once
#include "attn_plan.h"
#include "mega.h"

namespace bd {

constexpr int kFwdThreads = 512;      // 4 consumer + 4 producer wavefronts
#ifndef BD_SLOTS
#define BD_SLOTS 28
#endif
#ifndef BD_PROD_BATCH
#define BD_PROD_BATCH 4
#endif
#ifndef BD_PROD_DEPTH
#define BD_PROD_DEPTH 6
#endif
constexpr int kSlots = BD_SLOTS;            // 1-KiB ring slots per consumer
constexpr int kProdBatch = BD_PROD_BATCH;   // fragments a producer issues between two publications
constexpr int kProdDepth = BD_PROD_DEPTH;   // loads it leaves in flight when it publishes
constexpr int kLdsSpin = 1 << 22;           // bound of every LDS wait (a timed-out wait marks the context broken)
constexpr int kShareBytes = 40 * 1024;      // K-reduction buffers / attention merge buffers (one region, re-used)

typedef __attribute__((address_space(3))) void lds_void_t;

// words of the LDS synchronisation block
enum { SY_LANDED = 0, SY_CONSUMED = 4, SY_DEAD = 8, SY_CBAR = 9, SY_ARRIVE = 10, SY_EPOCH = 11, SY_XEPOCH = 12, SY_WORDS = 16 };

__device__ inline unsigned lds_addr(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ inline unsigned lds_ld32(unsigned addr) {
  unsigned v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
  return (unsigned)__builtin_amdgcn_readfirstlane((int)v);
}
__device__ inline void lds_st32(unsigned addr, unsigned v) {
  asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ inline void lds_inc(unsigned addr) {
  const unsigned one = 1u;
  asm volatile("ds_add_u32 %0, %1" ::"v"(addr), "v"(one) : "memory");
}

struct FwdSync {
  unsigned base;          // LDS address of the synchronisation block
  unsigned cbar_target;   // arrivals expected at the next consumer barrier
  unsigned arrive_target; // arrivals expected at the next grid barrier
  bool dead;              // a wait timed out somewhere in this workgroup: stop waiting, just finish
};

__device__ inline void mark_dead(FwdSync& sy, DevState* st) {
  sy.dead = true;
  lds_st32(sy.base + SY_DEAD * 4, 1u);
  __hip_atomic_store(&st->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until the LDS word at `addr` has reached `target` (wrap-safe); false on time-out or dead workgroup.
__device__ inline bool lds_wait_ge(FwdSync& sy, unsigned addr, unsigned target, DevState* st) {
  if (sy.dead) return false;
  int spins = 0;
  while ((int)(lds_ld32(addr) - target) < 0) {
    if ((++spins & 63) == 0) {
      if (lds_ld32(sy.base + SY_DEAD * 4) != 0u) { sy.dead = true; return false; }
      if (spins > kLdsSpin) { mark_dead(sy, st); return false; }
    }
  }
  return true;
}

// Barrier of the four consumer wavefronts.  LDS operations of one wavefront execute in order, so whatever
// a wavefront wrote to LDS before its arrival is visible to the others after theirs.
__device__ inline void cbar(FwdSync& sy, int lane, DevState* st) {
  sy.cbar_target += kWavesPerWG;
  if (lane == 0) lds_inc(sy.base + SY_CBAR * 4);
  lds_wait_ge(sy, sy.base + SY_CBAR * 4, sy.cbar_target, st);
  asm volatile("" ::: "memory");
}

// ---- producer ----------------------------------------------------------------------------------------------
// Row ranges are whole tiles, so a consumer's stream is a plain sequence of 1-KiB fragments: fragment q of the
// forward sits at byte q*1024 of the wavefront's stream, lane l's 16 bytes at l*16.
template <bool CUT>
__device__ inline unsigned stream_fragments(const MegaPlan& P, int cw) {
  return (unsigned)((long long)P.L * wave_layer_units_t<CUT>(P, blockIdx.x, cw) / 64);
}

template <bool CUT>
__device__ inline void producer_loop(const MegaArgs& a, int cw, char* ring, unsigned sync_base, int lane) {
  const MegaPlan& P = a.P;
  const unsigned total = stream_fragments<CUT>(P, cw);
  const rsrc_t wr = make_rsrc(a.wstream + (size_t)(blockIdx.x * kWavesPerWG + cw) * P.wave_stride, total * 1024u);
  const unsigned landed_addr = sync_base + (SY_LANDED + cw) * 4;
  const unsigned consumed_addr = sync_base + (SY_CONSUMED + cw) * 4;
  const unsigned dead_addr = sync_base + SY_DEAD * 4;
  unsigned issued = 0, landed = 0, consumed = 0;
  int slot = 0, since = 0;
  while (issued < total) {
    if (issued - consumed >= (unsigned)kSlots) {
      // ring full: publish everything that is under way, then wait for the consumer
      if (landed != issued) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        landed = issued;
        lds_st32(landed_addr, landed);
        since = 0;
      }
      int spins = 0;
      bool ok = true;
      while (issued - (consumed = lds_ld32(consumed_addr)) >= (unsigned)kSlots) {
        __builtin_amdgcn_s_sleep(1);
        if ((++spins & 31) == 0 && (lds_ld32(dead_addr) != 0u || spins > kLdsSpin)) { ok = false; break; }
      }
      if (!ok) break;
    }
    if (!a.no_weights)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (lds_void_t*)(ring + slot * 1024), 16, (int)(issued * 1024u) + lane * 16, 0, 0,
                                               kAuxNt);
    ++issued;
    slot = (slot + 1 == kSlots) ? 0 : slot + 1;
    if (++since == kProdBatch) {
      since = 0;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kProdDepth) : "memory");   // all but the newest kProdDepth are in LDS
      if (issued > (unsigned)kProdDepth && (int)(issued - kProdDepth - landed) > 0) {
        landed = issued - kProdDepth;
        lds_st32(landed_addr, landed);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  lds_st32(landed_addr, issued);
}

// ---- producer with a register stash behind the ring -------------------------------------------------------------
// The ring alone holds 28 KiB per consumer; the phases that stream almost nothing (QKV, attention, O and their
// hand-overs, a third of a layer's time) would leave HBM idle once it is full.  A producer wavefront owns as many
// registers as a consumer and needs none, so it keeps NS further fragments there: every fragment travels
// HBM -> stash register -> ring slot, the stash being a circular buffer of NS / 4 groups of four fragments between the
// two (fragment f in entry f mod NS).  Filling and draining advance independently: a group is moved to the ring as
// soon as the ring has room (at LDS speed, whatever is in flight), and groups are re-loaded at a bounded rate (a token
// bucket on the 100 MHz clock: kStashTicks per fragment, bursts of up to kStashBurst), so that the deep look-ahead
// never shows up as a deep queue in front of the latency-critical loads of the hand-overs.
// Stash entries are registers and can only be named statically, so the loop sweeps over the groups: at group k it
// moves group k if that is the next to move, then re-loads it if it is the next to load.  The loads are issued from
// inline assembly so that the waits stay in our hands (a compiler-placed wait in front of a conditionally loaded
// register can only be a wait for everything): vector-memory loads return in order, hence the group with y younger
// loads behind it has landed once at most y are outstanding.  The build checks that the compiler keeps the entries in
// place (no copy or spill of a register whose load may still be in flight) between the two markers below.
#ifndef BD_STASH
#define BD_STASH 48
#endif
#ifndef BD_STASH_TICKS
#define BD_STASH_TICKS 30
#endif
constexpr int kStash = BD_STASH;                 // fragments a producer keeps in registers (4 registers each); 0: ring only
constexpr int kStashGroup = 4;                   // fragments moved or requested per step
constexpr unsigned kStashTicks = BD_STASH_TICKS; // 10-ns ticks per fragment of the background pace (1 KiB / 300 ns = 3.4 GB/s a wavefront: a layer needs 2.5)
#ifndef BD_STASH_TICKS_FAST
#define BD_STASH_TICKS_FAST 10
#endif
#ifndef BD_STASH_LOW
#define BD_STASH_LOW 24
#endif
constexpr unsigned kStashTicksFast = BD_STASH_TICKS_FAST;   // pace while the consumer is about to run dry
constexpr int kStashLow = BD_STASH_LOW;          // "about to run dry": at most this many fragments requested and not yet consumed
#ifndef BD_STASH_BURST
#define BD_STASH_BURST 16
#endif
constexpr unsigned kStashBurst = BD_STASH_BURST;  // fragments that may be requested back to back
static_assert(kStash % kStashGroup == 0 && kSlots % kStashGroup == 0, "whole groups");

__device__ inline unsigned clock_ticks() { return (unsigned)wall_clock64(); }

// The loads that have `younger` loads issued after them have landed once this returns.
__device__ inline void wait_for_loads(unsigned younger) {
  if (younger >= 32u) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
  else if (younger >= 16u) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else if (younger >= 8u) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if (younger >= 4u) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <bool CUT, int NS>
__device__ inline void producer_loop_stash(const MegaArgs& a, int cw, char* ring, unsigned sync_base, int lane) {
  constexpr int NG = NS / kStashGroup;
  const MegaPlan& P = a.P;
  // (everything the inline assembly takes in scalar registers is made uniform explicitly)
  const unsigned total = (unsigned)__builtin_amdgcn_readfirstlane((int)stream_fragments<CUT>(P, cw));
  const unsigned total_up = (total + kStashGroup - 1) / kStashGroup * kStashGroup;   // (loads past the end read zeros and move no data)
  const size_t wbase = (size_t)(a.wstream + (size_t)(blockIdx.x * kWavesPerWG + cw) * P.wave_stride);
  const unsigned wlo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)wbase);
  const unsigned whi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(wbase >> 32));
  const rsrc_t wr = make_rsrc(reinterpret_cast<const void*>(((size_t)whi << 32) | wlo), total * 1024u);
  const unsigned landed_addr = sync_base + (SY_LANDED + cw) * 4;
  const unsigned consumed_addr = sync_base + (SY_CONSUMED + cw) * 4;
  const unsigned dead_addr = sync_base + SY_DEAD * 4;
  bf16x8 st[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) st[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  unsigned issued = 0, moved = 0, consumed = 0;     // fragments (multiples of the group size)
  int fill_g = 0, move_g = 0;                       // stash groups of fragment `issued` / fragment `moved`
  int slot = 0, spins = 0;
  unsigned t_mark = clock_ticks() - kStashBurst * kStashTicksFast;   // start with a full bucket
  const bool no_w = __builtin_amdgcn_readfirstlane(a.no_weights) != 0;   // measurement only: everything but the loads
  asm volatile("; BD_STASH_BEGIN" ::: "memory");
  while (moved < total_up) {
    // pace of the requests: the background pace while the consumer has plenty buffered, the demand pace once it is
    // about to run dry (what is buffered is what was requested and not yet consumed)
    const unsigned now = clock_ticks();
    consumed = lds_ld32(consumed_addr);
    const unsigned ticks = (issued - consumed <= (unsigned)kStashLow) ? kStashTicksFast : kStashTicks;
    unsigned tokens = (now - t_mark) / ticks;
    if (tokens > kStashBurst || no_w) { tokens = kStashBurst; t_mark = now - kStashBurst * ticks; }
    bool progress = false;
#pragma unroll
    for (int k = 0; k < NG; ++k) {
      if (move_g == k && moved < issued) {
        if (moved + kStashGroup - consumed > (unsigned)kSlots) consumed = lds_ld32(consumed_addr);
        if (moved + kStashGroup - consumed <= (unsigned)kSlots) {
          wait_for_loads(issued - moved - kStashGroup);
          bf16x8* dst = reinterpret_cast<bf16x8*>(ring + slot * 1024 + lane * 16);
#pragma unroll
          for (int j = 0; j < kStashGroup; ++j) dst[j * 64] = st[kStashGroup * k + j];
          asm volatile("" ::: "memory");
          moved += kStashGroup;
          lds_st32(landed_addr, min(moved, total));   // LDS executes a wavefront's operations in order
          slot = (slot + kStashGroup == kSlots) ? 0 : slot + kStashGroup;
          move_g = (k + 1 == NG) ? 0 : k + 1;
          progress = true;
        }
      }
      if (fill_g == k && issued < total_up && issued - moved < (unsigned)NS && tokens >= (unsigned)kStashGroup) {
        const int off = (int)(issued * 1024u) + lane * 16;
        if (!no_w) {
#pragma unroll
          for (int j = 0; j < kStashGroup; ++j)
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen offset:%3 nt"
                         : "+v"(st[kStashGroup * k + j]) : "v"(off), "s"(wr), "n"(j * 1024) : "memory");
        }
        issued += kStashGroup;
        tokens -= kStashGroup;
        t_mark += kStashGroup * ticks;
        fill_g = (k + 1 == NG) ? 0 : k + 1;
        progress = true;
      }
    }
    if (progress) {
      spins = 0;
    } else {
      __builtin_amdgcn_s_sleep(1);
      if ((++spins & 31) == 0 && (lds_ld32(dead_addr) != 0u || spins > kLdsSpin)) break;
    }
  }
  asm volatile("s_waitcnt vmcnt(0)\n\t; BD_STASH_END" ::: "memory");
}

// ---- consumer side of the ring -------------------------------------------------------------------------------
struct Ring {
  const char* base;        // this consumer's slots
  unsigned landed_addr, consumed_addr;
  unsigned have;           // fragments known to have landed
  unsigned taken;          // fragments consumed so far
  int slot;
};

__device__ inline void ring_need(Ring& rg, FwdSync& sy, int nf, DevState* st) {
  const unsigned need = rg.taken + (unsigned)nf;
  if ((int)(rg.have - need) < 0 && !sy.dead) {
    int spins = 0;
    while ((int)((rg.have = lds_ld32(rg.landed_addr)) - need) < 0) {
      if ((++spins & 63) == 0) {
        if (lds_ld32(sy.base + SY_DEAD * 4) != 0u) { sy.dead = true; break; }
        if (spins > kLdsSpin) { mark_dead(sy, st); break; }
      }
    }
  }
  asm volatile("" ::: "memory");
}
__device__ inline bf16x8 ring_take(Ring& rg, int lane) {
  const bf16x8 v = *reinterpret_cast<const bf16x8*>(rg.base + rg.slot * 1024 + lane * 16);
  rg.slot = (rg.slot + 1 == kSlots) ? 0 : rg.slot + 1;
  ++rg.taken;
  return v;
}
__device__ inline void ring_release(Ring& rg) { lds_st32(rg.consumed_addr, rg.taken); }

// One chunk (one or two 16-row tiles x KW k-steps) out of the ring, in batches of kBK k-steps, software
// pipelined over two small register sets: the LDS reads of batch b+1 are issued (and their slots handed back to
// the producer: LDS executes a wavefront's operations in order) before the MFMAs of batch b.
#ifndef BD_BK
#define BD_BK 2
#endif
constexpr int kBK = BD_BK;
template <int NT>
__device__ inline void ring_fetch(Ring& rg, FwdSync& sy, DevState* st, int nk, bf16x8 (&f)[kBK][NT], int lane) {
  ring_need(rg, sy, nk * NT, st);
#pragma unroll
  for (int u = 0; u < kBK; ++u)
    if (u < nk) {
#pragma unroll
      for (int t = 0; t < NT; ++t) f[u][t] = ring_take(rg, lane);
    }
  ring_release(rg);
  asm volatile("" ::: "memory");                            // the reads are issued before anything that follows
}
// The same with the number of k-steps known at compile time: straight-line code, so the compiler's LDS wait
// counts leave the reads of the next batch in flight during the MFMAs of this one.
template <int MT, bool TWO, int K0, int KWC>
__device__ inline void consume_chunk_static(Ring& rg, FwdSync& sy, DevState* st, const bf16x8 (&xk)[kMaxKW][MT],
                                            f32x4 (&acc)[kT][MT], int lane) {
  static_assert(KWC % kBK == 0, "whole batches");
  constexpr int NT = TWO ? 2 : 1;
  static_assert(KWC * NT <= kSlots, "a run must fit the ring");
  bf16x8 f[2][kBK][NT];
  ring_need(rg, sy, KWC * NT, st);                          // one check for the whole run
#pragma unroll
  for (int u = 0; u < kBK; ++u)
#pragma unroll
    for (int t = 0; t < NT; ++t) f[0][u][t] = ring_take(rg, lane);
#pragma unroll
  for (int b = 0; b < KWC / kBK; ++b) {
    if (b + 1 < KWC / kBK) {
#pragma unroll
      for (int u = 0; u < kBK; ++u)
#pragma unroll
        for (int t = 0; t < NT; ++t) f[(b + 1) & 1][u][t] = ring_take(rg, lane);
    }
#pragma unroll
    for (int u = 0; u < kBK; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[b & 1][u][t], xk[K0 + b * kBK + u][mt], acc[t][mt], 0, 0, 0);
  }
  ring_release(rg);
}

template <int MT, bool TWO>
__device__ inline void consume_chunk(Ring& rg, FwdSync& sy, DevState* st, const bf16x8 (&xk)[kMaxKW][MT], int KW,
                                     f32x4 (&acc)[kT][MT], int lane) {
  constexpr int NT = TWO ? 2 : 1;
  if (KW == kMaxKW) {                                       // the common case: a full K range, in runs that fit the ring
    if constexpr (TWO) {
      consume_chunk_static<MT, TWO, 0, kMaxKW / 2>(rg, sy, st, xk, acc, lane);
      consume_chunk_static<MT, TWO, kMaxKW / 2, kMaxKW / 2>(rg, sy, st, xk, acc, lane);
    } else {
      consume_chunk_static<MT, TWO, 0, kMaxKW>(rg, sy, st, xk, acc, lane);
    }
    return;
  }
  bf16x8 f[2][kBK][NT];
  ring_fetch<NT>(rg, sy, st, min(kBK, KW), f[0], lane);
#pragma unroll
  for (int b = 0; b < kMaxKW / kBK; ++b) {
    const int kb = b * kBK;
    if (kb < KW) {
      if (kb + kBK < KW) ring_fetch<NT>(rg, sy, st, min(kBK, KW - kb - kBK), f[(b + 1) & 1], lane);
      const int nk = min(kBK, KW - kb);
#pragma unroll
      for (int u = 0; u < kBK; ++u)
        if (u < nk) {
#pragma unroll
          for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[b & 1][u][t], xk[kb + u][mt], acc[t][mt], 0, 0, 0);
        }
    }
  }
}

// e4m3 weights: one ring fragment holds a 16-row tile for TWO k-steps (lane: 8 codes of the even step, then 8 of
// the odd one).  The codes are widened to bf16 in registers (exact) and multiplied with the bf16 MFMA; the
// per-row scale is applied to the accumulators afterwards.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
__device__ inline void widen_e4m3(const u32x4 raw, bf16x8& even, bf16x8& odd) {
  union { bf16x8 v; bf16x2_t h[4]; } a, b;
  a.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[0], 1.0f, false);
  a.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[0], 1.0f, true);
  a.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[1], 1.0f, false);
  a.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[1], 1.0f, true);
  b.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[2], 1.0f, false);
  b.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[2], 1.0f, true);
  b.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[3], 1.0f, false);
  b.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[3], 1.0f, true);
  even = a.v;
  odd = b.v;
}

template <int MT, bool TWO>
__device__ inline void consume_chunk_fp8(Ring& rg, FwdSync& sy, DevState* st, const bf16x8 (&xk)[kMaxKW][MT], int KW,
                                         f32x4 (&acc)[kT][MT], int lane) {
  constexpr int NT = TWO ? 2 : 1;
#pragma unroll
  for (int kb = 0; kb < kMaxKW; kb += 4) {                // two fragments per tile and batch
    if (kb < KW) {
      const int np = min(2, (KW - kb) >> 1);               // k-step pairs in this batch (KW is even)
      ring_need(rg, sy, np * NT, st);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (u < np) {
          u32x4 raw[NT];
#pragma unroll
          for (int t = 0; t < NT; ++t) raw[t] = __builtin_bit_cast(u32x4, ring_take(rg, lane));
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            bf16x8 we, wo;
            widen_e4m3(raw[t], we, wo);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(we, xk[kb + 2 * u][mt], acc[t][mt], 0, 0, 0);
              acc[t][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wo, xk[kb + 2 * u + 1][mt], acc[t][mt], 0, 0, 0);
            }
          }
        }
      }
      ring_release(rg);
    }
  }
}

struct FwdCtx {
  PhaseCtx pc;            // layer, n, red (LDS), s_flags
  f32x4* red2;            // second K-reduction buffer (chunks alternate)
  float* s_part;          // LDS [4][64] partial sums of squares per consumer
  char* share;            // LDS region shared by the K-reduction and the attention merge
};

// ---- one GEMM phase (consumer wavefronts) ------------------------------------------------------------------------
template <int MT, int PH, int D, bool FP8>
__device__ inline void stream_gemm_phase(const MegaArgs& a, FwdCtx& fc, Ring& rg, FwdSync& sy, int wave, int lane_in) {
  int lane = lane_in;
  asm volatile("" : "+v"(lane));
  const MegaPlan& P = a.P;
  PhaseCtx& pc = fc.pc;
  const WavePhase wp = wave_phase_t<FP8>(P, PH, blockIdx.x, wave);
  const int n_tiles = (wp.rows + 15) >> 4;
  const int n_chunks = (n_tiles + 1) >> 1;
  float rmax[MT], rsum[MT];
  int ridx[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) { rmax[mt] = -INFINITY; ridx[mt] = 0x7FFFFFFF; rsum[mt] = 0.f; }

#define BD_SUBTS2(k)                                                                                  \
  do {                                                                                                \
    if (a.trace2 != nullptr && pc.layer == 1 && threadIdx.x == 0 && PH < PH_LM)                        \
      a.trace2[(size_t)blockIdx.x * 64 + PH * 12 + (k)] = wall_clock64();                              \
  } while (0)
  BD_SUBTS2(0);
  if (n_chunks > 0) {
    constexpr bool kNorm = (PH == PH_QKV || PH == PH_GU || PH == PH_LM);
    const int ver = (PH == PH_QKV) ? 2 * pc.layer : (PH == PH_GU) ? 2 * pc.layer + 1 : 2 * P.L;
    const rsrc_t xr = kNorm ? make_rsrc(a.xb + (size_t)ver * a.xb_elems, (unsigned)(a.xb_elems * 2))
                            : (PH == PH_O ? make_rsrc(a.ap + (size_t)pc.layer * a.ap_elems, (unsigned)(a.ap_elems * 2))
                                          : make_rsrc(a.act + (size_t)pc.layer * a.act_elems, (unsigned)(a.act_elems * 2)));
    // activation fragments of this wavefront's k-steps: one round trip, straight into registers
    bf16x8 xk[kMaxKW][MT];
#pragma unroll
    for (int ksl = 0; ksl < kMaxKW; ++ksl)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        xk[ksl][mt] = buf_load_b(xr, ksl < wp.KW ? (((wp.w0 + ksl) * MT + mt) * 64 + lane) * 16 : kOob);
    if constexpr (kNorm) {
      // this wavefront's share (parts = wave*4 + lane group mod 16) of the sums of squares of every row
      const int parts = ver == 0 ? 1 : phase_tile_slots(P, (ver & 1) ? PH_O : PH_DOWN);
      const rsrc_t sr = make_rsrc(a.ssq + (size_t)ver * a.ssq_parts * a.Mp, (unsigned)((size_t)parts * a.Mp * 4));
      const int col = lane & 15, g = lane >> 4;
      float sv[MT][16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int p = wave * 4 + g + 16 * u;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          sv[mt][u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                    sr, p < parts ? (p * a.Mp + mt * 16 + col) * 4 : kOob, 0, 0));
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        float s = 0.f;
#pragma unroll
        for (int u = 0; u < 16; ++u) s += sv[mt][u];
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (g == 0) fc.s_part[wave * 64 + mt * 16 + col] = s;
      }
    }
    float rs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) rs[mt] = 1.f;
    BD_SUBTS2(1);

    for (int c = 0; c < n_chunks; ++c) {
      const bool two = 2 * c + 1 < n_tiles;
      // operands of this wavefront's epilogue element of the chunk (idx == wave), fetched while the product runs
      EpiPre pre;
      pre.cs[0] = pre.cs[1] = make_float2(0.f, 0.f);
      pre.xo = f32x4{0.f, 0.f, 0.f, 0.f};
      pre.gn = f32x4{1.f, 1.f, 1.f, 1.f};
      f32x4 wsc = f32x4{1.f, 1.f, 1.f, 1.f};                 // fp8: scales of this lane's four output rows
      if constexpr (FP8) {
        static_assert(kT * MT <= kWavesPerWG, "one epilogue element per consumer");
        if (wave < kT * MT) {
          const int lr = (2 * c + wave / MT) * 16 + 4 * (lane >> 4);
          if (lr < wp.rows)
            wsc = *reinterpret_cast<const f32x4*>(a.wscale + (size_t)pc.layer * a.wscale_layer + a.wscale_off[PH] + wp.row0 + lr);
        }
      }
      if constexpr (PH == PH_QKV || PH == PH_O) {
        static_assert(kT * MT <= kWavesPerWG, "one epilogue element per consumer");
        if (wave < kT * MT) {
          const int t = wave / MT, mt = wave % MT;
          const int token = mt * 16 + (lane & 15);
          const int lr = (2 * c + t) * 16 + 4 * (lane >> 4);
          const int r = wp.row0 + lr;
          if (token < a.M && lr < wp.rows) {
            if constexpr (PH == PH_QKV) {
#pragma unroll
              for (int pr = 0; pr < 2; ++pr) {
                const int rp = r + 2 * pr;
                if (2 * pr < min(4, wp.rows - lr) && rp < P.QD + P.KVD)
                  pre.cs[pr] = a.rope[(size_t)token * (D >> 1) + ((rp % D) >> 1)];
              }
            } else {
              if (min(4, wp.rows - lr) == 4 && (r & 3) == 0) {
                pre.xo = *reinterpret_cast<const f32x4*>(a.xv + ((size_t)(2 * pc.layer) * a.Mp + token) * P.H + r);
                if constexpr (FP8) pre.gn = *reinterpret_cast<const f32x4*>(a.gains + (size_t)(2 * pc.layer + 1) * P.H + r);
              }
            }
          }
        }
      }
      f32x4 acc[kT][MT];
#pragma unroll
      for (int t = 0; t < kT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[t][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if constexpr (PH == PH_QKV) {
        if (c == 0) {
          // (trace) the activations have arrived when the first MFMA could start
          unsigned x = __builtin_bit_cast(u32x4, xk[kMaxKW - 1][MT - 1])[0] | __builtin_bit_cast(u32x4, xk[0][0])[0];
          asm volatile("" ::"v"(x));
          BD_SUBTS2(6);
        }
      }
      if (wp.KW > 0) {
        if constexpr (FP8) {
          if (two) consume_chunk_fp8<MT, true>(rg, sy, a.st, xk, wp.KW, acc, lane);
          else consume_chunk_fp8<MT, false>(rg, sy, a.st, xk, wp.KW, acc, lane);
        } else {
          if (two) consume_chunk<MT, true>(rg, sy, a.st, xk, wp.KW, acc, lane);
          else consume_chunk<MT, false>(rg, sy, a.st, xk, wp.KW, acc, lane);
        }
      }
      if (c < 3) BD_SUBTS2(3 + 2 * c);
      // The operands fetched for the epilogue are taken here, before its first store: the vector-memory counter is
      // in order, so a wait for them placed behind a write-through store would also wait for that store's
      // acknowledgement (and after a branch that may have stored, the compiler can only wait for everything).
      asm volatile("" ::"v"(pre.cs[0].x), "v"(pre.cs[0].y), "v"(pre.cs[1].x), "v"(pre.cs[1].y), "v"(pre.xo), "v"(pre.gn), "v"(wsc));
      // the four consumers hold disjoint K ranges: sum them through LDS in fixed order
      f32x4* red = (c & 1) ? fc.red2 : pc.red;
#pragma unroll
      for (int t = 0; t < kT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) red[(wave * (kT * MT) + t * MT + mt) * 64 + lane] = acc[t][mt];
      cbar(sy, lane, a.st);
      if (c == 0) BD_SUBTS2(2);
      if constexpr (kNorm) {
        if (c == 0) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const int r = mt * 16 + (lane & 15);
            const float t = fc.s_part[r] + fc.s_part[64 + r] + fc.s_part[128 + r] + fc.s_part[192 + r];
            rs[mt] = rsqrtf(t / (float)P.H + a.rms_eps);
          }
        }
      }
#pragma unroll
      for (int idx = 0; idx < kT * MT; ++idx) {
        if ((idx & 3) != wave) continue;
        const int t = idx / MT, mt = idx % MT;
        if (t == 1 && !two) continue;
        f32x4 v = red[(0 * (kT * MT) + idx) * 64 + lane];
        v += red[(1 * (kT * MT) + idx) * 64 + lane];
        v += red[(2 * (kT * MT) + idx) * 64 + lane];
        v += red[(3 * (kT * MT) + idx) * 64 + lane];
        if constexpr (kNorm) v *= rs[mt];
        if constexpr (FP8) v *= wsc;
        if constexpr (PH == PH_QKV) { if (c == 0) BD_SUBTS2(5); }
        gemm_epilogue<MT, PH, D, (PH == PH_QKV || PH == PH_O)>(a, pc, wp, c, t, mt, v, lane, rmax, ridx, rsum, pre);
      }
      if (c < 3) BD_SUBTS2(4 + 2 * c);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this wavefront's stores have been acknowledged
  BD_SUBTS2(9);

  if constexpr (PH == PH_DOWN) {
    // the last of the ksplit workgroups to finish a tile sums all partials, adds the residual, stores the new
    // residual version and its sum of squares
    const int ksplit = P.ph[PH_DOWN].ksplit;
    const int tiles = phase_tile_slots(P, PH_DOWN);
    const int my_tiles = (wp.rows + 15) >> 4;
    const int gt0 = wp.ng * phase_tpg(P.ph[PH_DOWN]);
    const int col = lane & 15, g = lane >> 4;
    const int ver = 2 * pc.layer + 2;
    const int n_idx = my_tiles * MT;                          // (tile, row tile of tokens) pairs of this row range
    cbar(sy, lane, a.st);                                    // every consumer's partials are out
    if (wave == 0 && lane < my_tiles) {
      int last = 1;
      if (ksplit > 1) {
        const unsigned old = __hip_atomic_fetch_add(a.cntD + (size_t)pc.layer * tiles + gt0 + lane, 1u, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
        last = old == (unsigned)ksplit - 1u;
      }
      pc.s_flags[8 + lane] = last;
    }
    cbar(sy, lane, a.st);
    const float* src = a.wsD + (size_t)pc.layer * a.wsD_layer_floats;
    for (int idx0 = wave; idx0 < n_idx; idx0 += 2 * kWavesPerWG) {
      // two pairs per round, every load of the round in flight at once
      f32x4 pv[2][8], xov[2], gnv[2];
      bool on[2], vec[2];
      int tok[2], rr[2], nr[2], gtt[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int idx = idx0 + j * kWavesPerWG;
        const int tl = idx / MT, mt = idx % MT;
        on[j] = idx < n_idx && pc.s_flags[8 + min(tl, my_tiles - 1)];
        gtt[j] = gt0 + tl;
        tok[j] = mt * 16 + col;
        const int lr = tl * 16 + 4 * g;
        rr[j] = wp.row0 + lr;
        nr[j] = min(4, wp.rows - lr);
        vec[j] = nr[j] == 4 && (rr[j] & 3) == 0;
        xov[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        gnv[j] = f32x4{1.f, 1.f, 1.f, 1.f};
        if constexpr (FP8) {
          if (on[j] && vec[j] && ver < 2 * P.L) gnv[j] = *reinterpret_cast<const f32x4*>(a.gains + (size_t)ver * P.H + rr[j]);
        }
        if (on[j]) {
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int kg = min(u, ksplit - 1);
            pv[j][u] = *reinterpret_cast<const f32x4*>(src + ((((size_t)kg * tiles + gtt[j]) * a.MT + mt) * 64 + lane) * 4);
          }
          if (tok[j] < a.M && vec[j])
            xov[j] = *reinterpret_cast<const f32x4*>(a.xv + ((size_t)(ver - 1) * a.Mp + tok[j]) * P.H + rr[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (!on[j]) continue;
        const int idx = idx0 + j * kWavesPerWG;
        const int mt = idx % MT;
        f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (u < ksplit) v += pv[j][u];
        for (int kg = 8; kg < ksplit; ++kg)
          v += *reinterpret_cast<const f32x4*>(src + ((((size_t)kg * tiles + gtt[j]) * a.MT + mt) * 64 + lane) * 4);
        const int token = tok[j], r = rr[j], nrows = nr[j];
        float ss = 0.f;
        if (token < a.M && nrows > 0) {
          const float* xo = a.xv + ((size_t)(ver - 1) * a.Mp + token) * P.H + r;
          float* xn = a.xv + ((size_t)ver * a.Mp + token) * P.H + r;
          float o[4] = {0.f, 0.f, 0.f, 0.f};
          if (vec[j]) {
            const f32x4 ov = xov[j] + v;
            st_wt_f32x4(xn, ov);
            for (int e = 0; e < 4; ++e) o[e] = ov[e];
          } else {
            for (int e = 0; e < nrows; ++e) { o[e] = xo[e] + v[e]; st_wt_f32(xn + e, o[e]); }
          }
          ss = o[0] * o[0] + o[1] * o[1] + o[2] * o[2] + o[3] * o[3];
          if constexpr (FP8) {
            if (ver < 2 * P.L)
              for (int e = 0; e < nrows; ++e) o[e] *= gnv[j][e];
          }
          store_xb(a.xb + (size_t)ver * a.xb_elems, token, r, nrows, o, a.MT);
        }
        ss += __shfl_xor(ss, 16);
        ss += __shfl_xor(ss, 32);
        if (g == 0) st_wt_f32(a.ssq + ((size_t)ver * a.ssq_parts + gtt[j]) * a.Mp + token, ss);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    BD_SUBTS2(10);
  }
#undef BD_SUBTS2
}

// ---- attention phase ------------------------------------------------------------------------------------------
// Items (kv head, 16-column tile of (head, token) columns, key chunk).  The four consumers of a workgroup take
// the key blocks of the chunk round-robin, each with its own online softmax, and merge through LDS.  With a
// single chunk (short contexts) the merged result is final and goes straight out; otherwise the partial is
// stored and the workgroup completing the last chunk of a tile merges all chunks in fixed order.
__device__ inline void stream_attn_chunks(int n_keys, int max_chunks, int& n_kb, int& chunk_len, int& n_chunks) {
  n_kb = (n_keys + 31) >> 5;
  int want = n_kb <= 96 ? 1 : (n_kb + 39) / 40;              // short contexts: one chunk (a cross-workgroup merge costs more)
  if (want > max_chunks) want = max_chunks;
  chunk_len = ((n_kb + want - 1) / want + 3) & ~3;
  n_chunks = (n_kb + chunk_len - 1) / chunk_len;
}

// Reductions over the four 16-lane rows of a wavefront (the lanes that share a column of a C fragment), with the
// row-swap instructions of gfx950: two VALU operations per step, no LDS traffic.
__device__ inline float rows_max(float x) {
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ inline float rows_sum(float x) {
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float m = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <int D>
struct KvBlock {
  bf16x8 k[2][D / 32];
  bf16x8 v[D / 16];
};

// Block kb of a kv head (the keys of positions 32 kb .. 32 kb + 31) out of the page that holds it.
template <int D>
__device__ inline void kv_load(KvBlock<D>& b, const bf16x8* Kh, const bf16x8* Vh, int kb_logical, int lane, const int* pages) {
  constexpr int DS = D / 32, DT = D / 16;
  const int kb = page_of_block(pages, __builtin_amdgcn_readfirstlane(kb_logical));
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) b.k[t][ds] = Kh[(((size_t)kb * 2 + t) * DS + ds) * 64 + lane];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) b.v[dt] = Vh[((size_t)kb * DT + dt) * 64 + lane];
}

// One block of 32 keys against one tile of 16 query columns.  Scores stay unscaled until the exponent:
// p = 2^(s*c - m) with c = log2(e)/sqrt(d) folded into one fused multiply-add per score.
template <int D, bool MASKED, bool QUAD = false>
__device__ inline void attn_block(const KvBlock<D>& b, const bf16x8 (&qf)[D / 32], f32x4 (&O)[D / 16], float& mrun, float& lrun,
                                  int kb, int n, int M, int mode, int row, int g, float c) {
  constexpr int DS = D / 32, DT = D / 16;
  f32x4 s[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b.k[t][ds], qf[ds], s[t], 0, 0, 0);
  }
  float v[8];
  bool vis[8];
  float cmax = kNegBig;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] = s[e >> 2][e & 3];
    vis[e] = true;
    if constexpr (MASKED) {
      const int jb = kb * 32 + 8 * g + e - n;
      vis[e] = (jb < 0) || (jb < M && block_key_visible<QUAD>(mode, row, jb));
      if (vis[e]) cmax = fmaxf(cmax, v[e]);
    } else {
      cmax = fmaxf(cmax, v[e]);
    }
  }
  cmax = rows_max(cmax);
  const float mnew = fmaxf(mrun, cmax * c);
  float psum = 0.f;
  bf16x8 p8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float p = __builtin_amdgcn_exp2f(fmaf(v[e], c, -mnew));
    if constexpr (MASKED) p = vis[e] ? p : 0.f;
    psum += p;
    p8[e] = (__bf16)p;
  }
  psum = rows_sum(psum);
  if (__builtin_amdgcn_ballot_w64(mnew != mrun) != 0ull) {          // some column's maximum moved: rescale
    const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
    lrun *= alpha;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] *= alpha;
    mrun = mnew;
  }
  lrun += psum;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b.v[dt], p8, O[dt], 0, 0, 0);
}

template <int D, bool QUAD>
__device__ inline void stream_attention_phase(const MegaArgs& a, FwdCtx& fc, FwdSync& sy, int wave, int lane_in) {
  constexpr int DS = D / 32, DT = D / 16;
  int lane = lane_in;
  asm volatile("" : "+v"(lane));
  const MegaPlan& P = a.P;
  const PhaseCtx& pc = fc.pc;
  f32x4* sO = reinterpret_cast<f32x4*>(fc.share);                        // [4][DT][64]
  float* sm = reinterpret_cast<float*>(fc.share + kWavesPerWG * DT * 1024);   // [4][16]
  float* sl = sm + kWavesPerWG * 16;                                     // [4][16]
  float* wgt = sl + kWavesPerWG * 16;                                    // [64 chunks][16]
  float* s_inv = wgt + 64 * 16;                                          // [16]

  const int col = lane & 15, g = lane >> 4;
  const int n = pc.n;
  const int G = P.n_q / P.n_kv;
  const int Mp = a.MT * 16;
  const int n_ct = G * a.MT;                                             // column tiles per kv head
  int n_kb, chunk_len, n_chunks;
  const int n_groups = P.n_kv * n_ct;
  stream_attn_chunks(n + a.M, a.attn_max_chunks, n_kb, chunk_len, n_chunks);
  const int n_items = n_groups * n_chunks;
  const size_t kv_block = (size_t)32 * D / 8;
  const u16* Qb = a.Q + (size_t)pc.layer * a.Mp * P.n_q * D;
  float* pO = a.pO + (size_t)pc.layer * a.pO_layer_floats;
  float* pm = a.pm + (size_t)pc.layer * a.pml_layer_floats;
  float* pl = a.pl + (size_t)pc.layer * a.pml_layer_floats;
  u16* out = a.ap + (size_t)pc.layer * a.ap_elems;
  const float c = a.scale_log2e;

#define BD_ATS(k)                                                                                     \
  do {                                                                                                \
    if (a.trace2 != nullptr && pc.layer == 1 && threadIdx.x == 0) a.trace2[(size_t)blockIdx.x * 64 + 48 + (k)] = wall_clock64(); \
  } while (0)
  BD_ATS(0);
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int chunk = item % n_chunks;
    const int grp = item / n_chunks;
    const int ct = grp % n_ct, kvh = grp / n_ct;
    const bf16x8* Kh = reinterpret_cast<const bf16x8*>(a.Kc + (size_t)pc.layer * a.kv_layer_elems) + (size_t)kvh * a.max_kb * kv_block;
    const bf16x8* Vh = reinterpret_cast<const bf16x8*>(a.Vc + (size_t)pc.layer * a.kv_layer_elems) + (size_t)kvh * a.max_kb * kv_block;
    const int cidx = ct * 16 + col;
    const int hq = cidx / Mp, row = cidx - hq * Mp;
    bf16x8 qf[DS];
    {
      const u16* qp = Qb + ((size_t)row * P.n_q + kvh * G + hq) * D + 8 * g;
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8*>(qp + ds * 32);
    }
    f32x4 O[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun = kNegBig, lrun = 0.f;
    const int kb_end = min(n_kb, (chunk + 1) * chunk_len);
    const int kb0 = chunk * chunk_len + wave;
    // two register buffers, loads pinned one block ahead of their use
    KvBlock<D> b0, b1;
    if (kb0 < kb_end) kv_load<D>(b0, Kh, Vh, kb0, lane, a.kv_pages);
    asm volatile("" ::: "memory");
    for (int kb = kb0; kb < kb_end; kb += 2 * kWavesPerWG) {
      const int kb1 = kb + kWavesPerWG, kb2 = kb + 2 * kWavesPerWG;
      if (kb1 < kb_end) kv_load<D>(b1, Kh, Vh, kb1, lane, a.kv_pages);
      asm volatile("" ::: "memory");
      if (kb * 32 + 31 >= n) attn_block<D, true, QUAD>(b0, qf, O, mrun, lrun, kb, n, a.M, a.mode, row, g, c);
      else attn_block<D, false>(b0, qf, O, mrun, lrun, kb, n, a.M, a.mode, row, g, c);
      if (kb1 < kb_end) {
        if (kb2 < kb_end) kv_load<D>(b0, Kh, Vh, kb2, lane, a.kv_pages);
        asm volatile("" ::: "memory");
        if (kb1 * 32 + 31 >= n) attn_block<D, true, QUAD>(b1, qf, O, mrun, lrun, kb1, n, a.M, a.mode, row, g, c);
        else attn_block<D, false>(b1, qf, O, mrun, lrun, kb1, n, a.M, a.mode, row, g, c);
      }
    }
    BD_ATS(2);
    // merge the four consumers: everyone publishes (max, sum, O), then each folds a share of the d tiles
    if (g == 0) {
      sm[wave * 16 + col] = mrun;
      sl[wave * 16 + col] = lrun;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) sO[(wave * DT + dt) * 64 + lane] = O[dt];
    cbar(sy, lane, a.st);
    BD_ATS(3);
    float mm = sm[col];
#pragma unroll
    for (int w = 1; w < kWavesPerWG; ++w) mm = fmaxf(mm, sm[w * 16 + col]);
    float f[kWavesPerWG];
    float ll = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerWG; ++w) {
      f[w] = exp2f(sm[w * 16 + col] - mm);
      ll += sl[w * 16 + col] * f[w];
    }
    if (n_chunks == 1) {
      const float inv = 1.f / ll;
      for (int dt = wave; dt < DT; dt += kWavesPerWG) {
        f32x4 acc = sO[(0 * DT + dt) * 64 + lane] * f[0];
#pragma unroll
        for (int w = 1; w < kWavesPerWG; ++w) acc += sO[(w * DT + dt) * 64 + lane] * f[w];
        acc *= inv;
        if (row < a.M) {
          const int fo = (kvh * G + hq) * D + dt * 16 + 4 * g;
          const uint32_t lo = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
          const uint32_t hi = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
          st_wt_u64(out + xp_index(row, fo, a.MT), (uint64_t)lo | ((uint64_t)hi << 32));
        }
      }
      BD_ATS(4);
      cbar(sy, lane, a.st);                                   // the merge buffers are free again
      continue;
    }
    float* po = pO + (size_t)item * DT * 64 * 4;
    for (int dt = wave; dt < DT; dt += kWavesPerWG) {
      f32x4 acc = sO[(0 * DT + dt) * 64 + lane] * f[0];
#pragma unroll
      for (int w = 1; w < kWavesPerWG; ++w) acc += sO[(w * DT + dt) * 64 + lane] * f[w];
      st_wt_f32x4(po + ((size_t)dt * 64 + lane) * 4, acc);
    }
    if (wave == 0 && g == 0) {
      st_wt_f32(pm + (size_t)item * 16 + col, mm);
      st_wt_f32(pl + (size_t)item * 16 + col, ll);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    cbar(sy, lane, a.st);
    if (wave == 0 && lane == 0) {
      const unsigned old = __hip_atomic_fetch_add(a.cntA + (size_t)pc.layer * n_groups + grp, 1u, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
      fc.pc.s_flags[4] = old == (unsigned)n_chunks - 1u;
    }
    cbar(sy, lane, a.st);
    if (fc.pc.s_flags[4]) {
      // last arriver of this (kv head, column tile): merge all chunks in fixed order
      const size_t item0 = (size_t)grp * n_chunks;
      if (wave == 0) {
        // lane (col, g) looks at chunks g, g+4, ...; at most 64 chunks
        float pmv[16], plv[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const int ch = g + 4 * u;
          const int chc = min(ch, n_chunks - 1);
          pmv[u] = pm[(item0 + chc) * 16 + col];
          plv[u] = pl[(item0 + chc) * 16 + col];
        }
        float mx = kNegBig;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          if (g + 4 * u >= n_chunks) { pmv[u] = kNegBig; plv[u] = 0.f; }
          mx = fmaxf(mx, pmv[u]);
        }
        mx = rows_max(mx);
        float lp = 0.f;
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const int ch = g + 4 * u;
          const float w = exp2f(pmv[u] - mx);
          lp += plv[u] * w;
          if (ch < n_chunks) wgt[ch * 16 + col] = w;
        }
        lp = rows_sum(lp);
        if (g == 0) s_inv[col] = 1.f / lp;
      }
      cbar(sy, lane, a.st);
      const float* pg = pO + item0 * DT * 64 * 4;
      for (int dt = wave; dt < DT; dt += kWavesPerWG) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int ch0 = 0; ch0 < n_chunks; ch0 += 8) {
          f32x4 pv[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int chc = min(ch0 + u, n_chunks - 1);
            pv[u] = *reinterpret_cast<const f32x4*>(pg + (((size_t)chc * DT + dt) * 64 + lane) * 4);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (ch0 + u < n_chunks) acc += pv[u] * wgt[(ch0 + u) * 16 + col];
        }
        acc *= s_inv[col];
        if (row < a.M) {
          const int fo = (kvh * G + hq) * D + dt * 16 + 4 * g;
          const uint32_t lo = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
          const uint32_t hi = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
          st_wt_u64(out + xp_index(row, fo, a.MT), (uint64_t)lo | ((uint64_t)hi << 32));
        }
      }
    }
    cbar(sy, lane, a.st);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  BD_ATS(5);
#undef BD_ATS
}

// ---- attention phase kept inside each XCD ------------------------------------------------------------------------
// The split over key chunks above pays only for long contexts, because its merge is a chain of far-memory round trips
// (write-through partials, counter, reload by the last arriver).  When workgroup b runs on XCD b mod 8 (the rule the
// gate/up hand-over already relies on) the whole chip can work on a short context instead: the column tiles
// ((head, token) columns, 16 per tile) are dealt out to the XCDs, CT tiles each, all of one kv head; inside an XCD the
// tile's keys are spread over NCH = (workgroups per XCD) / CT workgroups and their four wavefronts (key block kb goes
// to chunk kb mod NCH, wavefront (kb / NCH) mod 4: every wavefront holds one or two blocks of a 1024-token context).
// Partials go to the XCD's L2 with plain stores, the workgroups of the XCD meet at their own barrier, and the merge is
// shared out again: (column tile, 16-dim slice) items over the XCD's wavefronts, each summing the NCH partials of its
// slice in chunk order.  Only the merged bf16 output is written through, for the O projection of all XCDs.
__device__ inline bool stream_xcd_barrier(const MegaArgs& a, FwdSync& sy, unsigned xepoch, int wave, int lane);

template <int D, bool QUAD>
__device__ inline bool stream_attention_local(const MegaArgs& a, FwdCtx& fc, FwdSync& sy, unsigned xepoch, int wave, int lane_in) {
  constexpr int DS = D / 32, DT = D / 16;
  int lane = lane_in;
  asm volatile("" : "+v"(lane));
  const MegaPlan& P = a.P;
  const PhaseCtx& pc = fc.pc;
  f32x4* sO = reinterpret_cast<f32x4*>(fc.share);                        // [4][DT][64]
  float* sm = reinterpret_cast<float*>(fc.share + kWavesPerWG * DT * 1024);   // [4][16]
  float* sl = sm + kWavesPerWG * 16;                                     // [4][16]
  float* wgt = sl + kWavesPerWG * 16;                                    // [64 chunks][16]
  float* s_inv = wgt + 64 * 16;                                          // [16]

  const int col = lane & 15, g = lane >> 4;
  const int n = pc.n;
  const int G = P.n_q / P.n_kv;
  const int Mp = a.MT * 16;
  const int n_ct = G * a.MT;                                             // column tiles per kv head
  AttnLocalPlan lp;
  attn_local_plan(P.nwg, a.n_xcd, P.n_kv, n_ct, lp);
  const int x = blockIdx.x % a.n_xcd, w = blockIdx.x / a.n_xcd;          // XCD, workgroup inside it
  const int n_kb = (n + a.M + 31) >> 5;
  const size_t kv_block = (size_t)32 * D / 8;
  const u16* Qb = a.Q + (size_t)pc.layer * a.Mp * P.n_q * D;
  float* pO = a.pO + (size_t)pc.layer * a.pO_layer_floats;
  float* pm = a.pm + (size_t)pc.layer * a.pml_layer_floats;
  float* pl = a.pl + (size_t)pc.layer * a.pml_layer_floats;
  u16* out = a.ap + (size_t)pc.layer * a.ap_elems;
  const float c = a.scale_log2e;

#define BD_ATS(k)                                                                                     \
  do {                                                                                                \
    if (a.trace2 != nullptr && pc.layer == 1 && threadIdx.x == 0) a.trace2[(size_t)blockIdx.x * 64 + 48 + (k)] = wall_clock64(); \
  } while (0)
  BD_ATS(0);
  {
    const int ctl = w % lp.CT, chunk = w / lp.CT;
    const int ct = x * lp.CT + ctl;                                      // column tile of this workgroup
    const int kvh = ct / n_ct, ctk = ct - kvh * n_ct;
    const bf16x8* Kh = reinterpret_cast<const bf16x8*>(a.Kc + (size_t)pc.layer * a.kv_layer_elems) + (size_t)kvh * a.max_kb * kv_block;
    const bf16x8* Vh = reinterpret_cast<const bf16x8*>(a.Vc + (size_t)pc.layer * a.kv_layer_elems) + (size_t)kvh * a.max_kb * kv_block;
    const int cidx = ctk * 16 + col;
    const int hq = cidx / Mp, row = cidx - hq * Mp;
    bf16x8 qf[DS];
    {
      const u16* qp = Qb + ((size_t)row * P.n_q + kvh * G + hq) * D + 8 * g;
#pragma unroll
      for (int ds = 0; ds < DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8*>(qp + ds * 32);
    }
    f32x4 O[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun = kNegBig, lrun = 0.f;
    const int stride = kWavesPerWG * lp.NCH;
    const int kb0 = chunk + lp.NCH * wave;
    KvBlock<D> b0, b1;
    if (kb0 < n_kb) kv_load<D>(b0, Kh, Vh, kb0, lane, a.kv_pages);
    asm volatile("" ::: "memory");
    for (int kb = kb0; kb < n_kb; kb += 2 * stride) {
      const int kb1 = kb + stride, kb2 = kb + 2 * stride;
      if (kb1 < n_kb) kv_load<D>(b1, Kh, Vh, kb1, lane, a.kv_pages);
      asm volatile("" ::: "memory");
      if (kb * 32 + 31 >= n) attn_block<D, true, QUAD>(b0, qf, O, mrun, lrun, kb, n, a.M, a.mode, row, g, c);
      else attn_block<D, false>(b0, qf, O, mrun, lrun, kb, n, a.M, a.mode, row, g, c);
      if (kb1 < n_kb) {
        if (kb2 < n_kb) kv_load<D>(b0, Kh, Vh, kb2, lane, a.kv_pages);
        asm volatile("" ::: "memory");
        if (kb1 * 32 + 31 >= n) attn_block<D, true, QUAD>(b1, qf, O, mrun, lrun, kb1, n, a.M, a.mode, row, g, c);
        else attn_block<D, false>(b1, qf, O, mrun, lrun, kb1, n, a.M, a.mode, row, g, c);
      }
    }
    BD_ATS(2);
    // merge the four consumers through LDS, each folding a share of the d tiles; the result is this workgroup's partial
    if (g == 0) {
      sm[wave * 16 + col] = mrun;
      sl[wave * 16 + col] = lrun;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) sO[(wave * DT + dt) * 64 + lane] = O[dt];
    cbar(sy, lane, a.st);
    float mm = sm[col];
#pragma unroll
    for (int wv = 1; wv < kWavesPerWG; ++wv) mm = fmaxf(mm, sm[wv * 16 + col]);
    float f[kWavesPerWG];
    float ll = 0.f;
#pragma unroll
    for (int wv = 0; wv < kWavesPerWG; ++wv) {
      f[wv] = exp2f(sm[wv * 16 + col] - mm);
      ll += sl[wv * 16 + col] * f[wv];
    }
    float* po = pO + (size_t)blockIdx.x * DT * 64 * 4;
    for (int dt = wave; dt < DT; dt += kWavesPerWG) {
      f32x4 acc = sO[(0 * DT + dt) * 64 + lane] * f[0];
#pragma unroll
      for (int wv = 1; wv < kWavesPerWG; ++wv) acc += sO[(wv * DT + dt) * 64 + lane] * f[wv];
      *reinterpret_cast<f32x4*>(po + ((size_t)dt * 64 + lane) * 4) = acc;   // read only inside this XCD: its L2 is coherent
    }
    if (wave == 0 && g == 0) {
      pm[(size_t)blockIdx.x * 16 + col] = mm;
      pl[(size_t)blockIdx.x * 16 + col] = ll;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    BD_ATS(3);
  }
  if (!stream_xcd_barrier(a, sy, xepoch, wave, lane)) return false;
  BD_ATS(4);
  // merge: item (column tile ctl, d tile dt) -> workgroup item mod WX, wavefront item / WX
  for (int item = w + lp.WX * wave; item < lp.CT * DT; item += lp.WX * kWavesPerWG) {
    const int ctl = item / DT, dt = item - ctl * DT;
    const int ct = x * lp.CT + ctl;
    const int kvh = ct / n_ct, ctk = ct - kvh * n_ct;
    const int cidx = ctk * 16 + col;
    const int hq = cidx / Mp, row = cidx - hq * Mp;
    // partial of chunk ch of this tile: the workgroup with w = ch * CT + ctl of this XCD
    float mx = kNegBig;
    for (int ch = 0; ch < lp.NCH; ++ch) mx = fmaxf(mx, pm[(size_t)((ch * lp.CT + ctl) * a.n_xcd + x) * 16 + col]);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f;
    for (int ch0 = 0; ch0 < lp.NCH; ch0 += 8) {
      f32x4 pv[8];
      float pmv[8], plv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int chc = min(ch0 + u, lp.NCH - 1);
        const size_t it = (size_t)((chc * lp.CT + ctl) * a.n_xcd + x);
        pv[u] = *reinterpret_cast<const f32x4*>(pO + (it * DT + dt) * 64 * 4 + (size_t)lane * 4);
        pmv[u] = pm[it * 16 + col];
        plv[u] = pl[it * 16 + col];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (ch0 + u < lp.NCH) {
          const float wq = exp2f(pmv[u] - mx);
          acc += pv[u] * wq;
          lsum += plv[u] * wq;
        }
    }
    acc *= 1.f / lsum;
    if (row < a.M) {
      const int fo = (kvh * G + hq) * D + dt * 16 + 4 * g;
      const uint32_t lo = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
      const uint32_t hi = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
      st_wt_u64(out + xp_index(row, fo, a.MT), (uint64_t)lo | ((uint64_t)hi << 32));
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  BD_ATS(5);
#undef BD_ATS
  (void)wgt; (void)s_inv;
  return true;
}

// ---- grid barrier of the consumer wavefronts ---------------------------------------------------------------------
// Every consumer has waited for its own stores (each phase ends with that wait).  Consumer 0 collects the four
// arrivals, takes part in the chip-wide barrier (two-level counters of mega.h) and hands the new epoch to the
// others through LDS.
__device__ inline bool stream_grid_barrier(const MegaArgs& a, FwdSync& sy, unsigned epoch, int wave, int lane) {
  const int nwg = a.P.nwg;
  sy.arrive_target += kWavesPerWG;
  if (lane == 0) lds_inc(sy.base + SY_ARRIVE * 4);
  if (wave == 0) {
    bool ok = lds_wait_ge(sy, sy.base + SY_ARRIVE * 4, sy.arrive_target, a.st);
    if (ok && lane == 0) {
      const int ng = (nwg + kBarGroup - 1) / kBarGroup;
      const int g = blockIdx.x / kBarGroup;
      const int gsize = min(kBarGroup, nwg - g * kBarGroup);
      unsigned* gcnt = a.bar + 32 * (1 + g);
      unsigned* rel = a.bar + 32 * (1 + ng);
      const unsigned old = __hip_atomic_fetch_add(gcnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == epoch * (unsigned)gsize - 1u) {
        const unsigned o2 = __hip_atomic_fetch_add(a.bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (o2 == epoch * (unsigned)ng - 1u)
          for (int r = 0; r < ng; ++r) __hip_atomic_store(rel + 32 * r, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      const unsigned* mine = rel + 32 * g;
      int spins = 0;
      while ((int)(__hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) < 0) {
        if (++spins > kSpinLimit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      if (ok) lds_st32(sy.base + SY_EPOCH * 4, epoch);
      else {
        lds_st32(sy.base + SY_DEAD * 4, 1u);
        __hip_atomic_store(&a.st->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  const bool ok = lds_wait_ge(sy, sy.base + SY_EPOCH * 4, epoch, a.st);
  asm volatile("" ::: "memory");
  return ok;
}

// ---- barrier of the workgroups of one XCD ------------------------------------------------------------------------
// Workgroup b runs on XCD b mod 8 (checked when the kernel starts), and the CUs of one XCD share one L2.  Between
// workgroups of one XCD a hand-over therefore needs no write-through: plain stores are complete (s_waitcnt) once that
// L2 holds them, and every later load from a CU of the same XCD that misses its L1 reads them there.  The arrival
// counter of XCD x is touched by the workgroups of XCD x only, through read-modify-write atomics, which never execute
// in an L1.
__device__ inline unsigned xcc_id() {
  unsigned x;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
  return x & 15u;
}
__device__ inline unsigned l2_atomic_peek(unsigned* p) {
  unsigned v;
  const unsigned zero = 0u;
  asm volatile("global_atomic_or %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p), "v"(zero) : "memory");
  return v;
}
__device__ inline bool stream_xcd_barrier(const MegaArgs& a, FwdSync& sy, unsigned xepoch, int wave, int lane) {
  sy.arrive_target += kWavesPerWG;
  if (lane == 0) lds_inc(sy.base + SY_ARRIVE * 4);
  if (wave == 0) {
    bool ok = lds_wait_ge(sy, sy.base + SY_ARRIVE * 4, sy.arrive_target, a.st);
    if (ok && lane == 0) {
      const int nx = a.n_xcd;
      unsigned* cnt = a.xbar + 32 * (blockIdx.x % nx);
      const unsigned target = xepoch * (unsigned)(a.P.nwg / nx);
      __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      int spins = 0;
      while ((int)(l2_atomic_peek(cnt) - target) < 0) {
        if (++spins > kSpinLimit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      if (ok) lds_st32(sy.base + SY_XEPOCH * 4, xepoch);
      else {
        lds_st32(sy.base + SY_DEAD * 4, 1u);
        __hip_atomic_store(&a.st->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  const bool ok = lds_wait_ge(sy, sy.base + SY_XEPOCH * 4, xepoch, a.st);
  asm volatile("" ::: "memory");
  return ok;
}

// ---- the kernel ------------------------------------------------------------------------------------------------
template <int MT> constexpr int stream_lds_bytes() { return kWavesPerWG * kSlots * 1024 + kShareBytes; }

template <int MT, int D, bool FP8, bool QUAD = false>
__global__ __launch_bounds__(kFwdThreads, 1) void stream_fwd_kernel(MegaArgs a) {
  static_assert(2 * kWavesPerWG * kT * MT * 1024 <= kShareBytes, "K-reduction buffers exceed the shared region");
  static_assert(kWavesPerWG * (D / 16) * 1024 + (8 * 16 + 64 * 16 + 16) * 4 <= kShareBytes, "attention merge buffers exceed the shared region");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ unsigned s_sync[SY_WORDS];
  __shared__ int s_flags[16];
  __shared__ float s_part[kWavesPerWG * 64];
  const MegaPlan& P = a.P;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (threadIdx.x < SY_WORDS) s_sync[threadIdx.x] = 0u;
  if (threadIdx.x == 0) {
    int go = (a.st->error == 0);
    if (go && a.skippable && a.st->skip) {
      skip_barriers(a.bar, a.xbar, (a.local_gu ? 4u : 5u) * (unsigned)P.L, ((a.local_gu ? 1u : 0u) + (a.attn_local ? 1u : 0u)) * (unsigned)P.L);
      go = 0;
    }
    if (go && (a.local_gu || a.attn_local) && xcc_id() != blockIdx.x % 8u) {   // the XCD-local hand-overs would be unsafe
      __hip_atomic_store(&a.st->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      go = 0;
    }
    s_flags[0] = go;
  }
  __syncthreads();                                       // the only workgroup barrier: all eight wavefronts are still here
  if (!s_flags[0]) return;
  const unsigned sync_base = lds_addr(s_sync);

  if (wave >= kWavesPerWG) {
    const int cw = wave - kWavesPerWG;
    if constexpr (kStash > 0) producer_loop_stash<FP8, kStash>(a, cw, lds + cw * kSlots * 1024, sync_base, lane);
    else producer_loop<FP8>(a, cw, lds + cw * kSlots * 1024, sync_base, lane);
    return;
  }

  FwdSync sy;
  sy.base = sync_base; sy.cbar_target = 0u; sy.arrive_target = 0u; sy.dead = false;
  Ring rg;
  rg.base = lds + wave * kSlots * 1024;
  rg.landed_addr = sync_base + (SY_LANDED + wave) * 4;
  rg.consumed_addr = sync_base + (SY_CONSUMED + wave) * 4;
  rg.have = 0u; rg.taken = 0u; rg.slot = 0;
  FwdCtx fc;
  fc.share = lds + kWavesPerWG * kSlots * 1024;
  fc.pc.n = a.st->n;
  for (int i = 0; i < 3; ++i) fc.pc.pg[i] = page_of_block(a.kv_pages, min((fc.pc.n >> 5) + i, a.max_kb - 1));
  fc.pc.xstage = nullptr;
  fc.pc.red = reinterpret_cast<f32x4*>(fc.share);
  fc.red2 = fc.pc.red + kWavesPerWG * kT * MT * 64;
  fc.pc.s_flags = s_flags;
  fc.s_part = s_part;
  unsigned epoch = a.bar_epoch, xepoch = a.xbar_epoch;

  int tsi = 0;
#define BD_TS2()                                                                                                  \
  do {                                                                                                            \
    if (a.trace != nullptr && threadIdx.x == 0) a.trace[(size_t)blockIdx.x * (10 * P.L + 4) + tsi] = wall_clock64(); \
    ++tsi;                                                                                                        \
  } while (0)
  BD_TS2();
  bool alive = true;
  for (int l = 0; l < P.L && alive; ++l) {
    fc.pc.layer = l;
    stream_gemm_phase<MT, PH_QKV, D, FP8>(a, fc, rg, sy, wave, lane);
    BD_TS2();
    alive = stream_grid_barrier(a, sy, ++epoch, wave, lane);
    BD_TS2();
    if (!alive) break;
    if (a.attn_local) {
      alive = stream_attention_local<D, QUAD>(a, fc, sy, ++xepoch, wave, lane);
      if (!alive) break;
    } else {
      stream_attention_phase<D, QUAD>(a, fc, sy, wave, lane);
    }
    BD_TS2();
    alive = stream_grid_barrier(a, sy, ++epoch, wave, lane);
    BD_TS2();
    if (!alive) break;
    stream_gemm_phase<MT, PH_O, D, FP8>(a, fc, rg, sy, wave, lane);
    BD_TS2();
    alive = stream_grid_barrier(a, sy, ++epoch, wave, lane);
    BD_TS2();
    if (!alive) break;
    stream_gemm_phase<MT, PH_GU, D, FP8>(a, fc, rg, sy, wave, lane);
    BD_TS2();
    if (a.local_gu) alive = stream_xcd_barrier(a, sy, ++xepoch, wave, lane);
    else alive = stream_grid_barrier(a, sy, ++epoch, wave, lane);
    BD_TS2();
    if (!alive) break;
    stream_gemm_phase<MT, PH_DOWN, D, FP8>(a, fc, rg, sy, wave, lane);
    BD_TS2();
    alive = stream_grid_barrier(a, sy, ++epoch, wave, lane);
    BD_TS2();
  }
  if (!alive && lane == 0) lds_st32(sync_base + SY_DEAD * 4, 1u);   // let the producers go
#undef BD_TS2
}

}  // namespace bd
