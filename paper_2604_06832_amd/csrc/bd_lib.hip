// Host side of the C ABI declared in include/bd.h: context, weight upload and packing, launch
// sequencing of one decoder forward, and the decode calls built on it.
#include "../../include/bd.h"
#include "../../include/bd_kernels.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <string>
#include <vector>

#include <cstdarg>

#include "common.h"
#include "launch.h"
#include "attn_plan.h"
#include "misc.h"
#include "pack.h"
#include "plan.h"
#include "prefill_args.h"

using namespace bd;

static char g_last_error[512] = "";

namespace bd {
void set_last_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
  va_end(ap);
}
}  // namespace bd

namespace {

enum KClass { KC_PROLOGUE = 0, KC_LAYERS, KC_LMHEAD, KC_FINISH, KC_COUNT };

}  // namespace

struct bd_ctx {
  bd_config cfg;
  hipStream_t stream = nullptr;
  int device = 0, num_cus = 256;
  int H, QD, KVD, NQKV, F, V, D, L, G;
  int Mp_max, max_kb;
  // paged cache: block kb of the sequence lives in page page_of[kb] (-1: none yet); pages come off the back of `free_pages`
  int* kv_pages = nullptr; std::vector<int> page_of, free_pages; int blocks_in_use = 0;
  int scattered = 0;               // blocks in use that do not sit in the page of their own number (0: the cache is contiguous)
  int rows_max = 0;                // most rows any forward can have: Mp_max, or the rows of a quadratic forward through the large-M kernels
  MegaPlan plan;
  // weights
  u16* wstream = nullptr;          // all matrices, in per-wavefront streaming order
  u16* embed = nullptr;            // bf16 [V][H] row-major (gathered, not streamed)
  float* gains = nullptr;          // [2L+1][H]
  std::vector<unsigned> loaded;    // per layer bit mask; last entry = top-level tensors
  // KV cache, packed: [L][n_kv][max_kb][32*D] bf16 each
  u16* Kc = nullptr;
  u16* Vc = nullptr;
  size_t kv_layer_elems = 0;
  // write-once activations of a forward
  float* xv = nullptr; float* ssq = nullptr; int ssq_parts = 0;
  u16* xb = nullptr; size_t xb_elems = 0;
  float2* rope = nullptr;
  u16* q = nullptr; u16* ap = nullptr; u16* act = nullptr;
  size_t ap_elems = 0, act_elems = 0;
  float* wsD = nullptr; size_t wsD_layer_floats = 0;
  unsigned* counters = nullptr; int n_cntD = 0, n_cntA = 0;
  float* pO = nullptr; float* pm = nullptr; float* pl = nullptr;
  size_t pO_layer_floats = 0, pml_layer_floats = 0;
  float* lm_max = nullptr; int* lm_idx = nullptr; float* lm_sum = nullptr;
  float* logits = nullptr; int logits_on = 0; int last_rows = 0; int last_had_logits = 0;
  int* row_cand = nullptr; float* row_conf = nullptr;
  // large-M prefill (prefill.h): tile-major copy of the decoder weights and the activations of one chunk
  bool pf_on = false; int pf_rows = 0;   // large-M kernels in use; rows of a prompt chunk
  int pf_cap = 0;                        // rows their working buffers hold: a prompt chunk, or the largest quadratic forward
  u16* pf_w = nullptr; size_t pf_layer_elems = 0; size_t pf_off[4] = {0, 0, 0, 0};
  float* pf_x = nullptr; u16* pf_xb = nullptr; float* pf_rs = nullptr; float2* pf_rope = nullptr;
  u16* pf_q = nullptr; u16* pf_ap = nullptr; u16* pf_act = nullptr;
  bool pf_staged = false;
  float* pf_apart = nullptr;       // attention partials of forwards of at most 64 rows through the large-M kernels
  float* pf_part = nullptr;        // [kPfSplit][pf_cap][H] K splits of the down projection
  int32_t* spec_tokens = nullptr; uint8_t* spec_mask = nullptr; int32_t* spec_k = nullptr;   // bd_speculative_step, bd_decode_block, bd_quad_*
  int32_t* quad_ids = nullptr;     // rows of the quadratic forward
  DevState* st = nullptr;
  unsigned* bar = nullptr; unsigned bar_epoch = 0;
  unsigned* xbar = nullptr; unsigned xbar_epoch = 0;   // barriers among the workgroups of one XCD (stream_fwd.h)
  int xcds = 0;                    // XCDs, if workgroup b of a forward-shaped launch runs on XCD b mod xcds (probed); else 0
  unsigned long long* trace = nullptr; int trace_on = 0;
  // host mirror of the decode state
  int n = 0;
  bool prefilled = false, carry_valid = false;
  bool use_stream = true;          // forwards of up to 32 rows run the kernel with decoupled weight streaming
  bool fp8 = false;                // decoder linears stored as e4m3 codes + per-row scales
  float* wscale = nullptr; int wscale_layer = 0; int wscale_off[4] = {0, 0, 0, 0};
  // per-launch timing (bd_k_profile)
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;   // pairs
  std::vector<int> prof_cls;
  std::vector<void*> allocs;
};

namespace {

int dev_alloc(bd_ctx* c, void** p, size_t bytes) {
  HIP_TRY(hipMalloc(p, bytes));
  HIP_TRY(hipMemsetAsync(*p, 0, bytes, c->stream));
  c->allocs.push_back(*p);
  return BD_OK;
}

struct Prof {
  bd_ctx* c; int cls; hipEvent_t e0 = nullptr, e1 = nullptr;
  Prof(bd_ctx* c_, int cls_) : c(c_), cls(cls_) {
    if (c->prof_on) {
      (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
      (void)hipEventRecord(e0, c->stream);
    }
  }
  ~Prof() {
    if (c->prof_on) {
      (void)hipEventRecord(e1, c->stream);
      c->prof_ev.push_back(e0); c->prof_ev.push_back(e1); c->prof_cls.push_back(cls);
    }
  }
};

// Row ranges and K splits of every GEMM phase; fails if a wavefront would have to hold more than
// kMaxKW k-steps of activations.
int make_plan(bd_ctx* c) {
  MegaPlan& P = c->plan;
  P.nwg = c->num_cus; P.L = c->L; P.H = c->H; P.QD = c->QD; P.KVD = c->KVD; P.F = c->F; P.V = c->V; P.D = c->D;
  P.n_q = c->cfg.n_q_heads; P.n_kv = c->cfg.n_kv_heads;
  const bool fp8 = c->cfg.weight_dtype == BD_FP8_E4M3;
  auto set = [&](int p, int N, int K, bool may_split) -> bool {
    PhasePlan& ph = P.ph[p];
    ph.N = N; ph.KS = ceil_div(K, 32); ph.ksplit = 1;
    ph.kgran = (fp8 && p != PH_LM) ? 2 : 1;
    ph.wbytes = (fp8 && p != PH_LM) ? 1 : 2;
    while (ph.kgran * ceil_div(ceil_div(ceil_div(ph.KS, ph.kgran), ph.ksplit), kWavesPerWG) > kMaxKW) {
      if (!may_split || P.nwg % (ph.ksplit * 2) != 0) return false;
      ph.ksplit *= 2;
    }
    const int groups = P.nwg / ph.ksplit;
    if (N % 16 != 0) return false;
    ph.RW = 16 * ceil_div(N / 16, groups);
    return true;
  };
  if (!set(PH_QKV, c->NQKV, c->H, false) || !set(PH_O, c->H, c->QD, false) || !set(PH_GU, 2 * c->F, c->H, false) ||
      !set(PH_DOWN, c->H, c->F, true) || !set(PH_LM, c->V, c->H, false))
    return BD_E_ARG;
  // QKV and O: at most one tile per workgroup -> tile j on workgroup j / nwg-1-j (see MegaPlan::single)
  P.single = 0;
  for (int p : {PH_QKV, PH_O})
    if (P.ph[p].ksplit == 1 && P.ph[p].N / 16 <= P.nwg) { P.single |= 1 << p; P.ph[p].RW = 16; }
  // Gate/up rows dealt out per XCD so that the SwiGLU output never leaves the XCD that produced it: needs the K slices
  // of the down projection to coincide with XCDs (workgroup b holds K slice b mod ksplit and runs on XCD b mod xcds).
  P.xcd_gu = 0;
  // (F a whole number of K units, so that every K slice of the down projection is a whole number of gate/up tiles;
  // bf16: slices of equal size, so that the even spread of the tiles is also the spread per XCD.)
  P.gu_cut = 0;
  if (c->xcds > 0 && P.nwg % c->xcds == 0 && P.ph[PH_DOWN].ksplit == c->xcds && P.ph[PH_GU].ksplit == 1 &&
      c->F == P.ph[PH_DOWN].KS * 32 && P.ph[PH_DOWN].KS % P.ph[PH_DOWN].kgran == 0 &&
      P.ph[PH_DOWN].KS / P.ph[PH_DOWN].kgran >= c->xcds && (fp8 || P.ph[PH_DOWN].KS % c->xcds == 0)) {
    P.xcd_gu = c->xcds;
    P.gu_cut = fp8 ? 1 : 0;
    int most = 0;
    for (int g = 0; g < P.nwg; ++g) most = std::max(most, phase_tile0(P, PH_GU, g + 1) - phase_tile0(P, PH_GU, g));
    P.ph[PH_GU].RW = 16 * most;
  }
  long long mx = 0;
  for (int wg = 0; wg < P.nwg; ++wg)
    for (int w = 0; w < kWavesPerWG; ++w) {
      long long u = (long long)P.L * wave_layer_units(P, wg, w) + wave_phase_units(P.ph[PH_LM], wave_phase(P, PH_LM, wg, w));
      mx = std::max(mx, u);
    }
  P.wave_stride = (mx + 63) / 64 * 64 + 64;            // a little slack: partial-tile lanes read clamped addresses only
  return BD_OK;
}

// Column tiles per attention item of the register-ring kernel: its register budget is shared with the prefetched
// weights, so it works on pairs.
int attn_jt(const bd_ctx*, int) { return 2; }

int attn_max_chunks(const bd_ctx* c, int MT) {
  const int JT = attn_jt(c, MT);
  const int groups = c->cfg.n_kv_heads * (c->G * MT / JT);
  int mc = (2 * c->num_cus) / groups;
  return std::max(1, std::min(mc, 64));
}

// Does workgroup b of a launch shaped like the streaming forward kernel's run on XCD b mod 8?  Returns 8 if so, else 0.
int probe_xcds(bd_ctx* c) {
  if (c->cfg.flags & BD_FLAG_CHIP_WIDE_HANDOVER) return 0;
  const int nwg = c->num_cus, nx = 8;
  if (nwg % nx != 0) return 0;
  unsigned* d = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&d), (size_t)nwg * 4) != hipSuccess) { (void)hipGetLastError(); return 0; }
  std::vector<unsigned> h((size_t)nwg, ~0u);
  bool ok = true;
  for (int rep = 0; rep < 2 && ok; ++rep) {
    ok = launch_xcc_probe(c->stream, nwg, d) == BD_OK &&
         hipMemcpyAsync(h.data(), d, (size_t)nwg * 4, hipMemcpyDeviceToHost, c->stream) == hipSuccess &&
         hipStreamSynchronize(c->stream) == hipSuccess;
    for (int b = 0; b < nwg && ok; ++b) ok = h[(size_t)b] == (unsigned)(b % nx);
  }
  (void)hipFree(d);
  (void)hipGetLastError();
  return ok ? nx : 0;
}

int stream_attn_max_chunks(const bd_ctx* c, int MT) {
  const int groups = c->cfg.n_kv_heads * c->G * MT;
  return std::max(1, std::min(c->num_cus / groups, 64));
}

// The layers kernel (streaming kernel for forwards of up to 32 rows, register-ring kernel beyond) and the LM head.
int launch_forward_kernels(bd_ctx* c, int MT, MegaArgs& a, bool lm_only = false) {
  const bool streamed = MT <= 2 && c->use_stream;
  if (!lm_only) {
    Prof pr(c, KC_LAYERS);
    const bool quad = a.mode >= 2;                           // quadratic mask (Alg. 2): its own instantiations
    if (streamed) {
      a.attn_max_chunks = stream_attn_max_chunks(c, MT);
      a.local_gu = c->plan.xcd_gu > 0 ? 1 : 0;
      a.n_xcd = c->xcds;
      AttnLocalPlan lp;
      a.attn_local = (!(c->cfg.flags & BD_FLAG_ATTENTION_KEY_SPLIT) &&
                      attn_local_plan(c->plan.nwg, c->xcds, c->cfg.n_kv_heads, c->G * MT, lp)) ? 1 : 0;
      a.xbar = c->xbar; a.xbar_epoch = c->xbar_epoch;
      a.no_weights = (c->cfg.flags & BD_FLAG_MEASURE_NO_WEIGHTS) ? 1 : 0;
      BD_TRY(launch_stream_fwd(c->stream, MT, c->D, c->fp8, quad, a));
      c->bar_epoch += (a.local_gu ? 4u : 5u) * (unsigned)c->L;
      c->xbar_epoch += (unsigned)((a.local_gu ? 1 : 0) + (a.attn_local ? 1 : 0)) * (unsigned)c->L;
      a.local_gu = 0; a.attn_local = 0;
    } else {
      if (c->fp8) return BD_E_ARG;                           // e4m3 weights are only streamed by the kernel above
      BD_TRY(launch_mega_fwd(c->stream, MT, c->D, quad, a));
      c->bar_epoch += 5u * (unsigned)c->L;
    }
  }
  if (a.want_lm) {
    Prof pr(c, KC_LMHEAD);
    a.bar_epoch = c->bar_epoch;
    BD_TRY(launch_lm_head(c->stream, MT, a));
    c->bar_epoch += 1u;
  }
  return BD_OK;
}

constexpr int kQuadMaxB = 32;      // largest block of a quadratic step: B (B + 1) = 1056 rows
constexpr int kStreamRows = 32;    // rows of a forward the decode kernels stream the weights against (two token tiles)

// ---- paged cache: the host owns the page list, the device holds a copy that the kernels index ---------------------
// Pages for every block that holds a position below `upto`, taken off the free list in order; the device table follows
// in stream order.
int ensure_pages(bd_ctx* c, int upto) {
  const int need = std::min(ceil_div(upto, 32), c->max_kb);
  while (c->blocks_in_use < need) {
    PageVals pv{};
    const int kb0 = c->blocks_in_use;
    int cnt = 0;
    while (cnt < 16 && kb0 + cnt < need) {
      if (c->free_pages.empty()) { set_last_error("paged cache: no free page for block %d", kb0 + cnt); return BD_E_CAPACITY; }
      const int pg = c->free_pages.back();
      c->free_pages.pop_back();
      c->page_of[(size_t)(kb0 + cnt)] = pg;
      c->scattered += pg != kb0 + cnt;
      pv.v[cnt++] = pg;
    }
    hipLaunchKernelGGL(set_pages_kernel, dim3(1), dim3(64), 0, c->stream, c->kv_pages, kb0, cnt, pv);
    BD_TRY(check_launch());
    c->blocks_in_use += cnt;
  }
  return BD_OK;
}

// Truncate the page list to the blocks that hold positions below `len`: the others go back to the free list, last
// block first (so that growing again hands them out in the same order).
void release_pages(bd_ctx* c, int len) {
  const int keep = ceil_div(len, 32);
  while (c->blocks_in_use > keep) {
    const int kb = --c->blocks_in_use;
    c->scattered -= c->page_of[(size_t)kb] != kb;
    c->free_pages.push_back(c->page_of[(size_t)kb]);
    c->page_of[(size_t)kb] = -1;
  }
}

// The table the kernels follow: none while every block in use sits in the page of its own number (the default hand-out
// order on a single sequence: the cache is contiguous and the kernels skip the look-ups).
const int* page_table(const bd_ctx* c) { return c->scattered ? c->kv_pages : nullptr; }

// What every chunk through the large-M kernels shares: shapes, weights, cache and working buffers of the context.
PfChunk chunk_args(bd_ctx* c) {
  PfChunk p{};
  p.n0 = c->n;
  p.table = c->embed; p.vocab = c->V; p.mask_id = c->cfg.mask_token_id;
  p.L = c->L; p.H = c->H; p.QD = c->QD; p.KVD = c->KVD; p.NQKV = c->NQKV; p.F = c->F; p.D = c->D;
  p.n_q = c->cfg.n_q_heads; p.n_kv = c->cfg.n_kv_heads; p.max_kb = c->max_kb;
  p.rms_eps = c->cfg.rms_eps; p.rope_theta = c->cfg.rope_theta;
  p.st = c->st;
  p.fp8 = c->fp8; p.staged = c->pf_staged;
  p.gains = c->gains; p.wscale = c->wscale; p.wscale_layer = c->wscale_layer;
  for (int i = 0; i < 4; ++i) { p.wscale_off[i] = c->wscale_off[i]; p.w_off[i] = c->pf_off[i]; }
  p.w = c->pf_w; p.layer_elems = c->pf_layer_elems;
  p.Kc = c->Kc; p.Vc = c->Vc; p.kv_layer_elems = c->kv_layer_elems; p.pages = page_table(c);
  p.x = c->pf_x; p.xb = c->pf_xb; p.rs = c->pf_rs; p.rope = c->pf_rope; p.q = c->pf_q; p.ap = c->pf_ap; p.act = c->pf_act;
  p.part = c->pf_part; p.apart = c->pf_apart;
  p.mode = BD_MODE_CAUSAL;
  return p;
}

// One chunk of `rows` prompt rows starting at prompt row `off` = cache position c->n through the large-M kernels.
int prefill_chunk(bd_ctx* c, const float* dev_embeds, int n_embed, const int32_t* dev_ids, int off, int rows) {
  BD_TRY(ensure_pages(c, c->n + rows));
  PfChunk p = chunk_args(c);
  p.rows = rows; p.off = off;
  p.embeds = dev_embeds; p.n_embed = n_embed; p.ids = dev_ids;
  return launch_prefill_chunk(c->stream, p);
}

int forward(bd_ctx* c, int M, int mode, bool want_lm, const float* embeds, int n_embed, const int32_t* ids, int off,
            int32_t* seed_tokens, uint8_t* seed_mask, const uint8_t* mask, bool skippable = false, int quad_B = 0,
            bool lm_only = false, int row0 = 0);

// Rows of the large-M kernels' residual stream [0, M) to the final norm + LM head of the decode kernels (all of them,
// or only the last one as row 0), and the clean-up afterwards.
int lm_head_of_rows(bd_ctx* c, const float* xrows, int M, int mode, bool skippable, int quad_B) {
  hipStream_t s = c->stream;
  const int ver = 2 * c->L, parts = phase_tile_slots(c->plan, PH_DOWN);
  const DevState* skip = skippable ? c->st : nullptr;
  float* ssq = c->ssq + (size_t)ver * c->ssq_parts * c->Mp_max;
  // (the LM head takes as many rows at a time as the decode kernels' buffers hold)
  for (int r0 = 0; r0 < M; r0 += c->Mp_max) {
    const int rows = std::min(c->Mp_max, M - r0), MT = ceil_div(rows, 16);
    hipLaunchKernelGGL(pf_rows_to_lm_kernel, dim3(MT * 16), dim3(kPfThreads), 0, s, xrows + (size_t)r0 * c->H, c->H, rows, MT,
                       c->xb + (size_t)ver * c->xb_elems, ssq, parts, c->Mp_max, skip);
    BD_TRY(check_launch());
    BD_TRY(forward(c, rows, mode, true, nullptr, 0, nullptr, 0, nullptr, nullptr, nullptr, skippable, quad_B, true, r0));
    hipLaunchKernelGGL(pf_clear_ssq_kernel, dim3(4), dim3(256), 0, s, ssq, parts, c->Mp_max, MT * 16, skip);
    BD_TRY(check_launch());
  }
  c->last_rows = M;
  return BD_OK;
}

// A forward of more than 32 rows: the decode kernels stream the weights against at most two token tiles, so these go
// through the large-M kernels (whole-chip tiled GEMMs per phase, attention with the forward's own visibility among the
// new rows), then the decode path's LM head over all rows.
int forward_large(bd_ctx* c, int M, int mode, bool want_lm, const float* embeds, int n_embed, const int32_t* ids, int off,
                  int32_t* seed_tokens, uint8_t* seed_mask, const uint8_t* mask, bool skippable, int quad_B) {
  PfChunk p = chunk_args(c);
  p.rows = M; p.off = off;
  p.embeds = embeds; p.n_embed = n_embed; p.ids = ids;
  p.block = mask != nullptr || seed_mask != nullptr;
  if (p.block && (embeds != nullptr || n_embed != 0 || off != 0)) return BD_E_ARG;
  p.seed_tokens = seed_tokens; p.seed_mask = seed_mask; p.mask = mask;
  p.mode = mode; p.quad_W = quad_B > 0 ? quad_B + 1 : 0; p.skippable = skippable ? 1 : 0;
  {
    Prof pr(c, KC_LAYERS);
    BD_TRY(launch_prefill_chunk(c->stream, p));
  }
  c->last_rows = M;
  c->last_had_logits = 0;
  if (want_lm) BD_TRY(lm_head_of_rows(c, c->pf_x, M, mode, skippable, quad_B));
  return BD_OK;
}

// One decoder forward over M rows: prologue (block assembly) + the persistent forward kernel.
// Source of the rows: prompt rows [off, off+M) (embeds then ids), or block tokens with an optional mask.
int forward(bd_ctx* c, int M, int mode, bool want_lm, const float* embeds, int n_embed, const int32_t* ids, int off,
            int32_t* seed_tokens, uint8_t* seed_mask, const uint8_t* mask, bool skippable, int quad_B, bool lm_only, int row0) {
  if (!lm_only) BD_TRY(ensure_pages(c, c->n + M));          // the new rows' keys and values land at [n, n + M)
  if (!lm_only && M > kStreamRows && c->pf_on && M <= std::max(c->Mp_max, c->rows_max))
    return forward_large(c, M, mode, want_lm, embeds, n_embed, ids, off, seed_tokens, seed_mask, mask, skippable, quad_B);
  // lm_only: the last residual version of the rows (bf16 copy and sums of squares) is already in place; only the final
  // norm + LM head run (the large-M prefill hands its last row over this way)
  const int MT = ceil_div(M, 16);
  const int Mp = c->Mp_max;
  hipStream_t s = c->stream;
  if (!lm_only) {
    PrologueArgs p{};
    p.x0 = c->xv; p.ssq0 = c->ssq; p.H = c->H; p.Mp = Mp; p.xb0 = c->xb; p.MT = MT;
    p.embeds = embeds; p.n_embed = n_embed; p.ids = ids; p.off = off;
    p.seed_tokens = seed_tokens; p.seed_mask = seed_mask; p.mask = mask;
    p.mask_id = c->cfg.mask_token_id; p.table = c->embed; p.vocab = c->V; p.st = c->st;
    p.rope = c->rope; p.half = c->D / 2; p.theta = c->cfg.rope_theta;
    p.counters = c->counters; p.n_counters = c->n_cntD + c->n_cntA;
    p.gain0 = c->fp8 ? c->gains : nullptr;
    p.skippable = skippable ? 1 : 0;
    p.quad_W = quad_B > 0 ? quad_B + 1 : 0;
    Prof pr(c, KC_PROLOGUE);
    hipLaunchKernelGGL(prologue_kernel, dim3(M), dim3(kWGThreads), 0, s, p);
    BD_TRY(check_launch());
  }
  MegaArgs a{};
  a.P = c->plan;
  a.wstream = reinterpret_cast<const bf16x8*>(c->wstream);
  a.st = c->st; a.bar = c->bar; a.bar_epoch = c->bar_epoch;
  a.M = M; a.MT = MT; a.mode = mode; a.want_lm = want_lm ? 1 : 0;
  a.skippable = skippable ? 1 : 0;
  a.xv = c->xv; a.xb = c->xb; a.xb_elems = c->xb_elems; a.ssq = c->ssq; a.ssq_parts = c->ssq_parts; a.Mp = Mp; a.gains = c->gains; a.rms_eps = c->cfg.rms_eps;
  a.fp8 = c->fp8 ? 1 : 0; a.wscale = c->wscale; a.wscale_layer = c->wscale_layer;
  for (int i = 0; i < 4; ++i) a.wscale_off[i] = c->wscale_off[i];
  a.rope = c->rope; a.Q = c->q; a.Kc = c->Kc; a.Vc = c->Vc; a.kv_layer_elems = c->kv_layer_elems; a.max_kb = c->max_kb;
  a.kv_pages = page_table(c);
  a.ap = c->ap; a.ap_elems = c->ap_elems; a.act = c->act; a.act_elems = c->act_elems;
  a.wsD = c->wsD; a.wsD_layer_floats = c->wsD_layer_floats; a.cntD = c->counters;
  a.pO = c->pO; a.pm = c->pm; a.pl = c->pl; a.pO_layer_floats = c->pO_layer_floats; a.pml_layer_floats = c->pml_layer_floats;
  a.cntA = c->counters + c->n_cntD;
  a.attn_max_chunks = attn_max_chunks(c, MT);
  a.scale_log2e = 1.4426950408889634f / std::sqrt((float)c->D);
  a.lm_max = c->lm_max; a.lm_idx = c->lm_idx; a.lm_sum = c->lm_sum;
  // (lm_only: the rows are rows row0 .. of a larger forward, and so are their results)
  a.logits = (want_lm && c->logits_on) ? c->logits + (size_t)row0 * c->V : nullptr;
  a.row_cand = c->row_cand + row0; a.row_conf = c->row_conf + row0;
  a.trace = c->trace_on ? c->trace : nullptr;
  a.trace2 = c->trace_on ? c->trace + (size_t)c->plan.nwg * (10 * c->L + 4) : nullptr;
  BD_TRY(launch_forward_kernels(c, MT, a, lm_only));
  c->last_rows = M;
  c->last_had_logits = (want_lm && c->logits_on) ? 1 : 0;
  return BD_OK;
}

bool all_loaded(const bd_ctx* c) {
  for (int l = 0; l < c->L; ++l)
    if (c->loaded[l] != 0x1FFu) return false;
  return c->loaded[c->L] == 7u;
}

int check_decode_call(const bd_ctx* c, int B) {
  if (c == nullptr) return BD_E_ARG;
  if (B < 1 || B > c->cfg.max_block) return BD_E_ARG;
  if (!c->prefilled) return BD_E_STATE;
  if (c->n + B > c->cfg.max_seq) return BD_E_CAPACITY;
  return BD_OK;
}

// The accept length of a speculative or quadratic step, read back together with the device state: a forward that
// gave up at a barrier leaves the previous call's length behind, so the call fails unless the device reports no error
// and its context length has advanced by exactly that many tokens.
int read_accept_length(bd_ctx* c, int B, const char* what, int32_t* k_out) {
  int32_t k = 0;
  DevState h;
  HIP_TRY(hipMemcpyAsync(&k, c->spec_k, 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipMemcpyAsync(&h, c->st, sizeof h, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (h.error != 0) {
    snprintf(g_last_error, sizeof g_last_error, "a grid barrier of the forward kernel timed out; the context is unusable");
    return BD_E_HIP;
  }
  if (k < 1 || k > B || h.n != c->n + k) {
    snprintf(g_last_error, sizeof g_last_error, "%s step returned an accept length of %d for a block of %d (device length %d, host length %d)",
             what, (int)k, B, h.n, c->n);
    return BD_E_HIP;
  }
  *k_out = k;
  return BD_OK;
}

FinishArgs finish_args(bd_ctx* c, int B) {
  FinishArgs f{};
  f.B = B; f.st = c->st; f.row_cand = c->row_cand; f.row_conf = c->row_conf;
  return f;
}

}  // namespace

namespace {

}  // namespace

extern "C" {

const char* bd_strerror(int code) {
  switch (code) {
    case BD_OK: return "ok";
    case BD_E_ARG: return "bad argument";
    case BD_E_STATE: return "call out of order";
    case BD_E_CAPACITY: return "KV cache capacity exceeded";
    case BD_E_DTYPE: return "unsupported dtype";
    case BD_E_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char* bd_last_error(void) { return g_last_error; }

int bd_create(const bd_config* cfg, void* hip_stream, bd_ctx** out) {
  if (cfg == nullptr || out == nullptr) return BD_E_ARG;
  const bd_config& k = *cfg;
  if (k.n_layers < 1 || k.hidden < 32 || k.n_q_heads < 1 || k.n_kv_heads < 1 || k.ffn < 16 || k.vocab < 16)
    return BD_E_ARG;
  if (k.head_dim != 64 && k.head_dim != 128) return BD_E_ARG;
  if (k.n_q_heads % k.n_kv_heads != 0) return BD_E_ARG;
  if (k.hidden % 32 != 0 || k.ffn % 16 != 0 || k.vocab % 16 != 0) return BD_E_ARG;
  if (k.max_block < 1 || k.max_block > 64 || k.max_seq < k.max_block) return BD_E_ARG;
  if (k.mask_token_id >= k.vocab) return BD_E_ARG;
  if (!(k.rope_theta > 0.f) || !(k.rms_eps > 0.f)) return BD_E_ARG;
  {
    // the attention phase works on groups of 2 or 4 column tiles (16 query columns each)
    // the attention phase works on pairs of column tiles (16 query columns each)
    const int G = k.n_q_heads / k.n_kv_heads;
    if (G % 2 != 0) return BD_E_ARG;
  }
  if (k.weight_dtype != BD_BF16 && k.weight_dtype != BD_FP8_E4M3) return BD_E_DTYPE;
  if (k.flags & ~(BD_FLAG_CHIP_WIDE_HANDOVER | BD_FLAG_REGISTER_RING | BD_FLAG_PREFILL_DECODE | BD_FLAG_PREFILL_STAGED | BD_FLAG_ATTENTION_KEY_SPLIT | BD_FLAG_MEASURE_NO_WEIGHTS)) return BD_E_ARG;
  // e4m3 weights: the streaming kernel takes forwards of up to 32 rows, larger ones need the large-M kernels
  if (k.weight_dtype == BD_FP8_E4M3 && k.max_block > 32 && !(k.max_seq > kPfTokens && !(k.flags & BD_FLAG_PREFILL_DECODE))) return BD_E_ARG;

  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, dev));

  bd_ctx* c = new bd_ctx();
  c->cfg = k;
  if (c->cfg.mask_token_id < 0) c->cfg.mask_token_id = k.vocab - 1;
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->device = dev;
  c->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  c->fp8 = k.weight_dtype == BD_FP8_E4M3;
  c->use_stream = c->fp8 || !(k.flags & BD_FLAG_REGISTER_RING);
  c->H = k.hidden; c->D = k.head_dim; c->QD = k.n_q_heads * k.head_dim; c->KVD = k.n_kv_heads * k.head_dim;
  c->NQKV = c->QD + 2 * c->KVD; c->F = k.ffn; c->V = k.vocab; c->L = k.n_layers; c->G = k.n_q_heads / k.n_kv_heads;
  c->Mp_max = ceil_div(k.max_block, 16) * 16;
  c->max_kb = ceil_div(k.max_seq, 32);
  // Large-M kernels for contexts whose cache can hold a chunk of 128 rows plus the prompt's last rows.
  c->pf_on = k.max_seq > kPfTokens && !(k.flags & BD_FLAG_PREFILL_DECODE);
  c->pf_rows = c->pf_on ? std::min(1024, (k.max_seq - 1) / kPfTokens * kPfTokens) : 0;
  {
    // the largest quadratic forward of this context: B (B + 1) rows for B = min(max_block, 32), if the cache can hold them
    const int Bq = std::min(k.max_block, kQuadMaxB);
    const int quad_rows = std::min(Bq * (Bq + 1), k.max_seq - 1);
    c->pf_cap = c->pf_on ? std::max(c->pf_rows, ceil_div(quad_rows, 16) * 16) : 0;
    c->rows_max = c->pf_on ? std::max(c->Mp_max, quad_rows) : c->Mp_max;
  }
  c->loaded.assign(c->L + 1, 0u);
  c->kv_layer_elems = (size_t)k.n_kv_heads * c->max_kb * 32 * c->D;
  c->xcds = c->use_stream ? probe_xcds(c) : 0;
  if (make_plan(c) != BD_OK) { delete c; return BD_E_ARG; }
  const MegaPlan& P = c->plan;

  auto fail = [&](int rc) { bd_destroy(c); return rc; };
#define A(ptr, bytes) { int rc_ = dev_alloc(c, reinterpret_cast<void**>(&(ptr)), (bytes)); if (rc_ != BD_OK) return fail(rc_); }
  const size_t Mp = c->Mp_max, L = c->L;
  A(c->wstream, (size_t)P.nwg * kWavesPerWG * P.wave_stride * 16);
  A(c->embed, (size_t)c->V * c->H * 2);
  A(c->gains, (2 * L + 1) * c->H * 4);
  if (c->fp8) {
    c->wscale_off[0] = 0; c->wscale_off[1] = c->NQKV; c->wscale_off[2] = c->NQKV + c->H; c->wscale_off[3] = c->NQKV + c->H + 2 * c->F;
    c->wscale_layer = c->NQKV + 2 * c->H + 2 * c->F;
    A(c->wscale, L * (size_t)c->wscale_layer * 4);
  }
  A(c->Kc, c->kv_layer_elems * L * 2);
  A(c->Vc, c->kv_layer_elems * L * 2);
  A(c->xv, (2 * L + 1) * Mp * c->H * 4);
  c->xb_elems = (size_t)c->H * Mp;
  A(c->xb, (2 * L + 1) * c->xb_elems * 2);
  c->ssq_parts = std::max(phase_tile_slots(P, PH_O), phase_tile_slots(P, PH_DOWN));
  A(c->ssq, (2 * L + 1) * (size_t)c->ssq_parts * Mp * 4);
  A(c->rope, Mp * (c->D / 2) * sizeof(float2));
  A(c->q, L * Mp * c->QD * 2);
  c->ap_elems = (size_t)ceil_div(c->QD, 32) * 32 * Mp;
  A(c->ap, L * c->ap_elems * 2);
  c->act_elems = (size_t)ceil_div(c->F, 32) * 32 * Mp;
  A(c->act, L * c->act_elems * 2);
  c->wsD_layer_floats = (size_t)P.ph[PH_DOWN].ksplit * phase_tile_slots(P, PH_DOWN) * (Mp / 16) * 64 * 4;
  A(c->wsD, L * c->wsD_layer_floats * 4);
  {
    // attention partials of one layer: sized for the largest item count any (M, n) can produce
    size_t tiles = 0; int groups_max = 0;
    for (int MT = 1; MT <= (int)Mp / 16; ++MT) {
      const int JT = attn_jt(c, MT);
      const int groups = k.n_kv_heads * (c->G * MT / JT);
      tiles = std::max(tiles, (size_t)groups * attn_max_chunks(c, MT) * JT);
      groups_max = std::max(groups_max, groups);
      if (MT <= 2) {   // the streaming kernel works on single column tiles (one partial per workgroup when it keeps the phase inside the XCDs)
        const int sg = k.n_kv_heads * c->G * MT;
        tiles = std::max(tiles, (size_t)P.nwg);
        tiles = std::max(tiles, (size_t)sg * stream_attn_max_chunks(c, MT));
        groups_max = std::max(groups_max, sg);
      }
    }
    c->pO_layer_floats = tiles * (c->D / 16) * 64 * 4;
    c->pml_layer_floats = tiles * 16;
    A(c->pO, L * c->pO_layer_floats * 4);
    A(c->pm, L * c->pml_layer_floats * 4);
    A(c->pl, L * c->pml_layer_floats * 4);
    c->n_cntD = (int)L * phase_tile_slots(P, PH_DOWN);
    c->n_cntA = (int)L * groups_max;
    A(c->counters, (size_t)(c->n_cntD + c->n_cntA) * 4);
  }
  A(c->lm_max, (size_t)P.nwg * Mp * 4);
  A(c->lm_idx, (size_t)P.nwg * Mp * 4);
  A(c->lm_sum, (size_t)P.nwg * Mp * 4);
  A(c->row_cand, (size_t)c->rows_max * 4);
  A(c->row_conf, (size_t)c->rows_max * 4);
  A(c->spec_tokens, Mp * 4);
  A(c->spec_mask, Mp);
  A(c->spec_k, 4);
  A(c->quad_ids, (size_t)c->rows_max * 4);
  {
    // Large-M prefill for contexts whose cache can hold a chunk of 128 rows plus the prompt's last rows.  (e4m3
    // decoder linears are widened into the bf16 copy, exactly; their row scales stay in the epilogue.)
    c->pf_staged = (k.flags & BD_FLAG_PREFILL_STAGED) != 0;     // register-staged GEMMs only (else: the fallback for K tails)
    if (c->pf_on) {
      const size_t R = (size_t)c->pf_cap;
      const int NP[4] = {c->NQKV, c->H, 2 * c->F, c->H};
      const int KP[4] = {c->H, c->QD, c->H, c->F};
      size_t off = 0;
      for (int ph = 0; ph < 4; ++ph) { c->pf_off[ph] = off; off += (size_t)NP[ph] * ceil_div(KP[ph], 32) * 32; }
      c->pf_layer_elems = off;
      A(c->pf_w, L * c->pf_layer_elems * 2);
      A(c->pf_x, R * c->H * 4);
      A(c->pf_xb, R * c->H * 2);
      A(c->pf_rs, R * 4);
      A(c->pf_rope, R * (c->D / 2) * sizeof(float2));
      A(c->pf_q, R * c->QD * 2);
      A(c->pf_ap, R * (size_t)ceil_div(c->QD, 32) * 32 * 2);
      A(c->pf_act, R * (size_t)ceil_div(c->F, 32) * 32 * 2);
      A(c->pf_part, (size_t)kPfSplit * R * c->H * 4);
      A(c->pf_apart, (size_t)k.n_q_heads * 4 * kPfAttnChunks * ((size_t)(c->D / 16) * 256 + 128) * 4);
    }
  }
  {
    // page table of the cache: every block is a page; none is in use yet, and the free list hands them out in
    // ascending order unless bd_kv_page_order says otherwise.  (The device copy starts as the identity: an entry of a
    // block that is not in use is never followed, but it always names an existing page.)
    A(c->kv_pages, (size_t)c->max_kb * 4);
    c->page_of.assign((size_t)c->max_kb, -1);
    c->free_pages.resize((size_t)c->max_kb);
    for (int i = 0; i < c->max_kb; ++i) c->free_pages[(size_t)i] = c->max_kb - 1 - i;
    hipLaunchKernelGGL(iota_kernel, dim3(ceil_div(c->max_kb, 256)), dim3(256), 0, c->stream, c->kv_pages, c->max_kb);
  }
  A(c->st, sizeof(DevState));
  A(c->bar, (size_t)(1 + 2 * ceil_div(P.nwg, kBarGroup)) * 32 * 4);
  A(c->xbar, (size_t)8 * 32 * 4);
#undef A
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) {
    snprintf(g_last_error, sizeof g_last_error, "hipStreamSynchronize failed: %s", hipGetErrorString(e));
    return fail(BD_E_HIP);
  }
  *out = c;
  return BD_OK;
}

void bd_destroy(bd_ctx* c) {
  if (c == nullptr) return;
  (void)hipStreamSynchronize(c->stream);
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->logits) (void)hipFree(c->logits);
  delete c;
}

int bd_load_weight(bd_ctx* c, const char* name, const void* host_ptr, size_t bytes, int dtype,
                   const float* host_scales) {
  if (c == nullptr || name == nullptr || host_ptr == nullptr) return BD_E_ARG;
  std::string nm(name);
  int layer = -1;
  std::string base = nm;
  if (nm.size() > 1 && nm[0] == 'l' && nm[1] >= '0' && nm[1] <= '9') {
    size_t dot = nm.find('.');
    if (dot == std::string::npos) return BD_E_ARG;
    layer = atoi(nm.substr(1, dot - 1).c_str());
    base = nm.substr(dot + 1);
    if (layer < 0 || layer >= c->L) return BD_E_ARG;
  }
  // logical shape and where the rows go in the weight stream
  int rows = 0, K = 0, ph = -1, row_base = 0, row_map = 0, bit = -1;
  int norm_ver = -1;              // residual version whose RMSNorm gain is folded into this matrix
  float* gain_dst = nullptr;
  bool is_embed = false;
  if (layer < 0) {
    if (base == "embed") { rows = c->V; K = c->H; is_embed = true; bit = 0; }
    else if (base == "lm_head") { rows = c->V; K = c->H; ph = PH_LM; bit = 1; norm_ver = 2 * c->L; }
    else if (base == "final_norm") { rows = c->H; gain_dst = c->gains + (size_t)(2 * c->L) * c->H; bit = 2; }
    else return BD_E_ARG;
  } else {
    if (base == "attn_norm") { rows = c->H; gain_dst = c->gains + (size_t)(2 * layer) * c->H; bit = 0; }
    else if (base == "ffn_norm") { rows = c->H; gain_dst = c->gains + (size_t)(2 * layer + 1) * c->H; bit = 1; }
    else if (base == "wq") { rows = c->QD; K = c->H; ph = PH_QKV; row_base = 0; row_map = 1; bit = 2; norm_ver = 2 * layer; }
    else if (base == "wk") { rows = c->KVD; K = c->H; ph = PH_QKV; row_base = c->QD; row_map = 1; bit = 3; norm_ver = 2 * layer; }
    else if (base == "wv") { rows = c->KVD; K = c->H; ph = PH_QKV; row_base = c->QD + c->KVD; bit = 4; norm_ver = 2 * layer; }
    else if (base == "wo") { rows = c->H; K = c->QD; ph = PH_O; bit = 5; }
    else if (base == "w_gate") { rows = c->F; K = c->H; ph = PH_GU; row_base = 0; row_map = 2; bit = 6; norm_ver = 2 * layer + 1; }
    else if (base == "w_up") { rows = c->F; K = c->H; ph = PH_GU; row_base = 1; row_map = 2; bit = 7; norm_ver = 2 * layer + 1; }
    else if (base == "w_down") { rows = c->H; K = c->F; ph = PH_DOWN; bit = 8; }
    else return BD_E_ARG;
  }
  if (gain_dst != nullptr) {
    if (dtype != BD_F32) return BD_E_DTYPE;
    if (bytes != (size_t)rows * 4) return BD_E_ARG;
    {
      const unsigned used_by = layer < 0 ? 2u : (base == "attn_norm" ? 0x1Cu : 0xC0u);   // lm_head | wq,wk,wv | gate,up
      if (c->loaded[layer < 0 ? c->L : layer] & used_by) return BD_E_STATE;
    }
    HIP_TRY(hipMemcpy(gain_dst, host_ptr, bytes, hipMemcpyHostToDevice));
  } else if (c->fp8 && ph >= 0 && ph != PH_LM) {
    // one of the seven decoder linears of an e4m3 context: codes + one fp32 scale per output row
    if (dtype != BD_FP8_E4M3) return BD_E_DTYPE;
    if (host_scales == nullptr || bytes != (size_t)rows * K) return BD_E_ARG;
    void* stage = nullptr;
    float* sc = nullptr;
    HIP_TRY(hipMalloc(&stage, bytes));
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&sc), (size_t)rows * 4);
    if (e == hipSuccess) e = hipMemcpy(stage, host_ptr, bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(sc, host_scales, (size_t)rows * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
      hipLaunchKernelGGL(pack_stream_fp8_kernel, dim3(4096), dim3(256), 0, c->stream, (const uint8_t*)stage, rows, K, c->plan,
                         ph, layer, row_base, row_map, c->D, reinterpret_cast<uint8_t*>(c->wstream));
      hipLaunchKernelGGL(scatter_scales_kernel, dim3(64), dim3(256), 0, c->stream, sc, rows, row_base, row_map, c->D,
                         c->wscale + (size_t)layer * c->wscale_layer + c->wscale_off[ph]);
      if (c->pf_on)
        hipLaunchKernelGGL(pack_tiles_kernel<uint8_t>, dim3(4096), dim3(256), 0, c->stream, (const uint8_t*)stage, rows, K,
                           ceil_div(K, 32), row_base, row_map, c->D, (const float*)nullptr,
                           c->pf_w + (size_t)layer * c->pf_layer_elems + c->pf_off[ph]);
      e = hipGetLastError();
      if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    }
    (void)hipFree(stage);
    if (sc) (void)hipFree(sc);
    if (e != hipSuccess) {
      snprintf(g_last_error, sizeof g_last_error, "weight upload failed: %s", hipGetErrorString(e));
      return BD_E_HIP;
    }
  } else {
    if (dtype != BD_F32 && dtype != BD_BF16) return BD_E_DTYPE;
    const float* col_gain = nullptr;
    if (norm_ver >= 0) {
      // the gain of the norm in front of this matrix is folded into its columns, so it must be here already
      const bool have = norm_ver == 2 * c->L ? (c->loaded[c->L] & 4u) != 0
                                             : (c->loaded[norm_ver / 2] & (1u << (norm_ver & 1))) != 0;
      if (!have) return BD_E_STATE;
      col_gain = c->gains + (size_t)norm_ver * c->H;
    }
    const size_t esz = dtype == BD_F32 ? 4 : 2;
    if (bytes != (size_t)rows * K * esz) return BD_E_ARG;
    void* stage = nullptr;
    HIP_TRY(hipMalloc(&stage, bytes));
    hipError_t e = hipMemcpy(stage, host_ptr, bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
      if (is_embed) {
        if (dtype == BD_F32)
          hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(2048), dim3(256), 0, c->stream, (const float*)stage, c->embed,
                             (size_t)rows * K);
        else
          e = hipMemcpyAsync(c->embed, stage, bytes, hipMemcpyDeviceToDevice, c->stream);
      } else if (dtype == BD_F32) {
        hipLaunchKernelGGL(pack_stream_kernel<float>, dim3(4096), dim3(256), 0, c->stream, (const float*)stage, rows, K,
                           c->plan, ph, std::max(layer, 0), row_base, row_map, c->D, col_gain, c->wstream);
      } else {
        hipLaunchKernelGGL(pack_stream_kernel<u16>, dim3(4096), dim3(256), 0, c->stream, (const u16*)stage, rows, K,
                           c->plan, ph, std::max(layer, 0), row_base, row_map, c->D, col_gain, c->wstream);
      }
      if (c->pf_on && !is_embed && ph >= 0 && ph != PH_LM) {
        u16* dst = c->pf_w + (size_t)layer * c->pf_layer_elems + c->pf_off[ph];
        if (dtype == BD_F32)
          hipLaunchKernelGGL(pack_tiles_kernel<float>, dim3(4096), dim3(256), 0, c->stream, (const float*)stage, rows, K,
                             ceil_div(K, 32), row_base, row_map, c->D, col_gain, dst);
        else
          hipLaunchKernelGGL(pack_tiles_kernel<u16>, dim3(4096), dim3(256), 0, c->stream, (const u16*)stage, rows, K,
                             ceil_div(K, 32), row_base, row_map, c->D, col_gain, dst);
      }
      if (e == hipSuccess) e = hipGetLastError();
      if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    }
    (void)hipFree(stage);
    if (e != hipSuccess) {
      snprintf(g_last_error, sizeof g_last_error, "weight upload failed: %s", hipGetErrorString(e));
      return BD_E_HIP;
    }
  }
  c->loaded[layer < 0 ? c->L : layer] |= 1u << bit;
  return BD_OK;
}

int bd_prefill(bd_ctx* c, const float* dev_embeds, int n_embed, const int32_t* dev_ids, int n_ids) {
  if (c == nullptr || n_embed < 0 || n_ids < 0 || n_embed + n_ids < 1) return BD_E_ARG;
  if ((n_embed > 0 && dev_embeds == nullptr) || (n_ids > 0 && dev_ids == nullptr)) return BD_E_ARG;
  if (!all_loaded(c)) return BD_E_STATE;
  const int total = n_embed + n_ids;
  if (total > c->cfg.max_seq) return BD_E_CAPACITY;
  hipStream_t s = c->stream;
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, s, c->st, 0, 1);
  BD_TRY(check_launch());
  c->n = 0; c->prefilled = false; c->carry_valid = false;
  release_pages(c, 0);
  const int step = c->cfg.max_block;                   // (at most 32 with e4m3 weights, checked at creation)
  int off0 = 0;
  if (c->pf_on && total > kPfTokens) {
    // The whole prompt in large chunks; the last row's residual stream is then handed to the final norm + LM head.
    while (off0 < total) {
      int rows = std::min(c->pf_rows, total - off0);
      if (total - off0 - rows > 0 && total - off0 - rows < kPfTokens && rows > kPfTokens) rows -= kPfTokens;   // no sliver
      BD_TRY(prefill_chunk(c, dev_embeds, n_embed, dev_ids, off0, rows));
      const bool last = off0 + rows >= total;
      hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(1), 0, s, c->st, last ? rows - 1 : rows);
      BD_TRY(check_launch());
      if (last) {
        c->n += rows - 1;
        BD_TRY(lm_head_of_rows(c, c->pf_x + (size_t)(rows - 1) * c->H, 1, BD_MODE_CAUSAL, false, 0));
        FinishArgs f = finish_args(c, 1);
        f.commit = 1;
        hipLaunchKernelGGL(finish_causal_kernel, dim3(1), dim3(64), 0, s, f);
        BD_TRY(check_launch());
        c->n += 1;
      } else {
        c->n += rows;
      }
      off0 += rows;
    }
    c->prefilled = true; c->carry_valid = true;
    return BD_OK;
  }
  for (int off = off0; off < total; off += step) {
    const int M = std::min(step, total - off);
    const bool last = off + M >= total;
    BD_TRY(forward(c, M, BD_MODE_CAUSAL, last, dev_embeds, n_embed, dev_ids, off, nullptr, nullptr, nullptr));
    if (last) {
      FinishArgs f = finish_args(c, M);
      f.commit = 1;
      hipLaunchKernelGGL(finish_causal_kernel, dim3(1), dim3(64), 0, s, f);
    } else {
      hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(1), 0, s, c->st, M);
    }
    BD_TRY(check_launch());
    c->n += M;
  }
  c->prefilled = true; c->carry_valid = true;
  return BD_OK;
}

int bd_denoise_step(bd_ctx* c, int32_t* dev_block_tokens, uint8_t* dev_mask, int B, float threshold, int fixed_k,
                    int32_t* dev_n_unmasked, float* dev_conf_out) {
  BD_TRY(check_decode_call(c, B));
  if (dev_block_tokens == nullptr || dev_mask == nullptr || fixed_k < 0) return BD_E_ARG;
  hipStream_t s = c->stream;
  if (B == 1) {
    hipLaunchKernelGGL(seed_kernel, dim3(1), dim3(64), 0, s, dev_block_tokens, dev_mask, c->st);
    BD_TRY(check_launch());
    hipLaunchKernelGGL(finish_seed_only_kernel, dim3(1), dim3(64), 0, s, c->st, dev_n_unmasked, dev_conf_out);
    return check_launch();
  }
  BD_TRY(forward(c, B, BD_MODE_BIDIR, true, nullptr, 0, dev_block_tokens, 0, dev_block_tokens, dev_mask, dev_mask));
  FinishArgs f = finish_args(c, B);
  f.tokens = dev_block_tokens; f.mask = dev_mask; f.threshold = threshold; f.fixed_k = fixed_k;
  f.n_unmasked = dev_n_unmasked; f.conf_out = dev_conf_out;
  Prof pr(c, KC_FINISH);
  hipLaunchKernelGGL(finish_denoise_kernel, dim3(1), dim3(64), 0, s, f);
  return check_launch();
}

static int causal_pass(bd_ctx* c, const int32_t* dev_tokens, int B, int commit, int32_t* dev_ar_pred,
                       int32_t* dev_n_accept, const int32_t* draft) {
  hipStream_t s = c->stream;
  BD_TRY(forward(c, B, BD_MODE_CAUSAL, true, nullptr, 0, dev_tokens, 0, nullptr, nullptr, nullptr));
  FinishArgs f = finish_args(c, B);
  f.draft = draft; f.commit = commit; f.ar_pred = dev_ar_pred; f.n_accept = dev_n_accept;
  {
    Prof pr(c, KC_FINISH);
    hipLaunchKernelGGL(finish_causal_kernel, dim3(1), dim3(64), 0, s, f);
    BD_TRY(check_launch());
  }
  if (commit) { c->n += B; c->carry_valid = true; }
  return BD_OK;
}

int bd_commit_block(bd_ctx* c, const int32_t* dev_block_tokens, int B) {
  BD_TRY(check_decode_call(c, B));
  if (dev_block_tokens == nullptr) return BD_E_ARG;
  return causal_pass(c, dev_block_tokens, B, 1, nullptr, nullptr, nullptr);
}

int bd_verify_block(bd_ctx* c, const int32_t* dev_draft, int B, int commit, int32_t* dev_ar_pred,
                    int32_t* dev_n_accept) {
  BD_TRY(check_decode_call(c, B));
  if (dev_draft == nullptr) return BD_E_ARG;
  if (dev_n_accept != nullptr && !c->carry_valid) return BD_E_STATE;
  return causal_pass(c, dev_draft, B, commit ? 1 : 0, dev_ar_pred, dev_n_accept, dev_draft);
}

int bd_decode_block(bd_ctx* c, int B, float threshold, int fixed_k, int32_t* dev_tokens_out, int32_t* dev_steps_out) {
  BD_TRY(check_decode_call(c, B));
  if (dev_tokens_out == nullptr || fixed_k < 0) return BD_E_ARG;
  if (!c->carry_valid) return BD_E_STATE;
  hipStream_t s = c->stream;
  hipLaunchKernelGGL(fill_masked_kernel, dim3(1), dim3(64), 0, s, c->spec_tokens, c->spec_mask, B, c->cfg.mask_token_id, c->st, 0);
  BD_TRY(check_launch());
  if (B == 1) {
    hipLaunchKernelGGL(seed_kernel, dim3(1), dim3(64), 0, s, c->spec_tokens, c->spec_mask, c->st);
    BD_TRY(check_launch());
  } else {
    // every step reveals at least one position (min(fixed_k, left) under the fixed schedule), so this many complete
    // any block; the steps after the last useful one find DevState::skip set and do nothing
    const int steps = fixed_k > 0 ? ceil_div(B - 1, fixed_k) : B - 1;
    for (int i = 0; i < steps; ++i) {
      BD_TRY(forward(c, B, BD_MODE_BIDIR, true, nullptr, 0, c->spec_tokens, 0, c->spec_tokens, c->spec_mask, c->spec_mask, true));
      FinishArgs f = finish_args(c, B);
      f.tokens = c->spec_tokens; f.mask = c->spec_mask; f.threshold = threshold; f.fixed_k = fixed_k; f.skippable = 1;
      Prof pr(c, KC_FINISH);
      hipLaunchKernelGGL(finish_denoise_kernel, dim3(1), dim3(64), 0, s, f);
      BD_TRY(check_launch());
    }
  }
  BD_TRY(causal_pass(c, c->spec_tokens, B, 1, nullptr, nullptr, nullptr));
  HIP_TRY(hipMemcpyAsync(dev_tokens_out, c->spec_tokens, (size_t)B * 4, hipMemcpyDeviceToDevice, s));
  if (dev_steps_out != nullptr) {
    hipLaunchKernelGGL(read_steps_kernel, dim3(1), dim3(1), 0, s, c->st, dev_steps_out);
    BD_TRY(check_launch());
  }
  return BD_OK;
}

int bd_quad_draft(bd_ctx* c, int B, int32_t* dev_draft_out) {
  BD_TRY(check_decode_call(c, B));
  if (dev_draft_out == nullptr) return BD_E_ARG;
  if (!c->carry_valid) return BD_E_STATE;
  hipStream_t s = c->stream;
  if (B > 1) {
    // B mask tokens, none of them seeded: position 0 is handed over as already revealed but holds the mask id
    hipLaunchKernelGGL(fill_masked_kernel, dim3(1), dim3(64), 0, s, c->spec_tokens, c->spec_mask, B, c->cfg.mask_token_id, c->st, 1);
    BD_TRY(check_launch());
    BD_TRY(forward(c, B, BD_MODE_BIDIR, true, nullptr, 0, c->spec_tokens, 0, c->spec_tokens, c->spec_mask, c->spec_mask));
    FinishArgs f = finish_args(c, B);
    f.tokens = c->spec_tokens; f.mask = c->spec_mask; f.threshold = 2.f; f.fixed_k = B - 1;
    hipLaunchKernelGGL(finish_denoise_kernel, dim3(1), dim3(64), 0, s, f);
    BD_TRY(check_launch());
  }
  hipLaunchKernelGGL(quad_first_kernel, dim3(1), dim3(1), 0, s, c->spec_tokens, c->st);
  BD_TRY(check_launch());
  HIP_TRY(hipMemcpyAsync(dev_draft_out, c->spec_tokens, (size_t)B * 4, hipMemcpyDeviceToDevice, s));
  return BD_OK;
}

int bd_quad_step(bd_ctx* c, int B, const int32_t* dev_draft, int32_t* dev_next_draft, int32_t* host_n_accepted) {
  if (c == nullptr || B < 1 || dev_draft == nullptr || dev_next_draft == nullptr || host_n_accepted == nullptr) return BD_E_ARG;
  const int M = B * (B + 1);
  if (B > c->cfg.max_block || B > kQuadMaxB) return BD_E_ARG;
  // B (B + 1) rows: within max_block through the decode kernels, beyond (up to 1056) through the large-M kernels
  if (M > c->cfg.max_block && !(c->pf_on && M <= c->rows_max)) return BD_E_ARG;
  if (!c->prefilled) return BD_E_STATE;
  if (c->n + M > c->cfg.max_seq) return BD_E_CAPACITY;   // the forward parks its rows at [cache_len, cache_len + M)
  hipStream_t s = c->stream;
  hipLaunchKernelGGL(quad_assemble_kernel, dim3(ceil_div(M, 64)), dim3(64), 0, s, dev_draft, B, c->cfg.mask_token_id, c->quad_ids);
  BD_TRY(check_launch());
  BD_TRY(forward(c, M, 2 | (B << 8), true, nullptr, 0, c->quad_ids, 0, nullptr, nullptr, nullptr, false, B));
  {
    FinishArgs f = finish_args(c, B);
    f.draft = dev_draft; f.n_accept = c->spec_k;
    Prof pr(c, KC_FINISH);
    hipLaunchKernelGGL(finish_quad_kernel, dim3(1), dim3(64), 0, s, f, dev_next_draft);
    BD_TRY(check_launch());
    hipLaunchKernelGGL(quad_compact_kv_kernel, dim3(c->L * c->cfg.n_kv_heads), dim3(256), 0, s, c->Kc, c->Vc, c->kv_layer_elems,
                       c->cfg.n_kv_heads, c->D, c->max_kb, c->st, c->spec_k, B, page_table(c));
    BD_TRY(check_launch());
  }
  int32_t k = 0;
  BD_TRY(read_accept_length(c, B, "quadratic", &k));
  c->n += k;
  c->carry_valid = true;
  release_pages(c, c->n);                               // the rows beyond the accepted ones are gone: so are their pages
  *host_n_accepted = k;
  return BD_OK;
}

int bd_speculative_step(bd_ctx* c, int B, int32_t* dev_tokens_out, int32_t* host_n_accepted) {
  BD_TRY(check_decode_call(c, B));
  if (dev_tokens_out == nullptr || host_n_accepted == nullptr) return BD_E_ARG;
  if (!c->carry_valid) return BD_E_STATE;
  hipStream_t s = c->stream;
  // draft: [x_n, MASK, ...] -> every masked position filled by the argmax of the row before it, in one pass
  hipLaunchKernelGGL(fill_masked_kernel, dim3(1), dim3(64), 0, s, c->spec_tokens, c->spec_mask, B, c->cfg.mask_token_id, c->st, 0);
  BD_TRY(check_launch());
  if (B == 1) {
    hipLaunchKernelGGL(seed_kernel, dim3(1), dim3(64), 0, s, c->spec_tokens, c->spec_mask, c->st);
    BD_TRY(check_launch());
  } else {
    BD_TRY(forward(c, B, BD_MODE_BIDIR, true, nullptr, 0, c->spec_tokens, 0, c->spec_tokens, c->spec_mask, c->spec_mask));
    FinishArgs f = finish_args(c, B);
    f.tokens = c->spec_tokens; f.mask = c->spec_mask; f.threshold = 2.f; f.fixed_k = B - 1;
    Prof pr(c, KC_FINISH);
    hipLaunchKernelGGL(finish_denoise_kernel, dim3(1), dim3(64), 0, s, f);
    BD_TRY(check_launch());
  }
  // verify: causal forward with cache update; accept and crop on the device
  BD_TRY(forward(c, B, BD_MODE_CAUSAL, true, nullptr, 0, c->spec_tokens, 0, nullptr, nullptr, nullptr));
  {
    FinishArgs f = finish_args(c, B);
    f.draft = c->spec_tokens; f.commit = 2; f.ar_pred = dev_tokens_out; f.n_accept = c->spec_k;
    Prof pr(c, KC_FINISH);
    hipLaunchKernelGGL(finish_causal_kernel, dim3(1), dim3(64), 0, s, f);
    BD_TRY(check_launch());
  }
  int32_t k = 0;
  BD_TRY(read_accept_length(c, B, "speculative", &k));
  c->n += k;
  c->carry_valid = true;
  release_pages(c, c->n);                               // the rows beyond the accepted ones are gone: so are their pages
  *host_n_accepted = k;
  return BD_OK;
}

int bd_crop(bd_ctx* c, int new_len) {
  if (c == nullptr) return BD_E_ARG;
  if (!c->prefilled) return BD_E_STATE;
  if (new_len < 0 || new_len > c->n) return BD_E_ARG;
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, c->stream, c->st, new_len, 1);
  BD_TRY(check_launch());
  c->n = new_len;
  c->carry_valid = false;
  release_pages(c, new_len);                            // the page list is cut where the context is
  return BD_OK;
}

int bd_kv_page_order(bd_ctx* c, const int32_t* host_order, int n_pages) {
  if (c == nullptr || host_order == nullptr || n_pages != c->max_kb) return BD_E_ARG;
  if (c->blocks_in_use != 0) return BD_E_STATE;
  std::vector<char> seen((size_t)n_pages, 0);
  for (int i = 0; i < n_pages; ++i) {
    const int pg = host_order[i];
    if (pg < 0 || pg >= n_pages || seen[(size_t)pg]) return BD_E_ARG;
    seen[(size_t)pg] = 1;
  }
  for (int i = 0; i < n_pages; ++i) c->free_pages[(size_t)(n_pages - 1 - i)] = host_order[i];   // the back is handed out first
  return BD_OK;
}

int bd_kv_pages(const bd_ctx* c, int32_t* host_out, int capacity) {
  if (c == nullptr || (host_out == nullptr && capacity > 0) || capacity < 0) return BD_E_ARG;
  for (int i = 0; i < c->blocks_in_use && i < capacity; ++i) host_out[i] = c->page_of[(size_t)i];
  return c->blocks_in_use;
}

int bd_cache_len(const bd_ctx* c) { return c == nullptr ? BD_E_ARG : c->n; }

int bd_status(bd_ctx* c) {
  if (c == nullptr) return BD_E_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  DevState h;
  HIP_TRY(hipMemcpy(&h, c->st, sizeof h, hipMemcpyDeviceToHost));
  if (h.error != 0) {
    snprintf(g_last_error, sizeof g_last_error, "a grid barrier of the forward kernel timed out; the context is unusable");
    return BD_E_HIP;
  }
  return BD_OK;
}

int bd_debug_logits(bd_ctx* c, int enable) {
  if (c == nullptr) return BD_E_ARG;
  if (enable && c->logits == nullptr) HIP_TRY(hipMalloc(reinterpret_cast<void**>(&c->logits), (size_t)c->rows_max * c->V * 4));
  c->logits_on = enable ? 1 : 0;
  return BD_OK;
}

int bd_read_logits(bd_ctx* c, float* dev_out, int rows) {
  if (c == nullptr || dev_out == nullptr || rows < 1) return BD_E_ARG;
  if (!c->last_had_logits || rows > c->last_rows) return BD_E_STATE;
  HIP_TRY(hipMemcpyAsync(dev_out, c->logits, (size_t)rows * c->V * 4, hipMemcpyDeviceToDevice, c->stream));
  return BD_OK;
}

int bd_read_kv(bd_ctx* c, int layer, int pos0, int count, float* dev_k_out, float* dev_v_out) {
  if (c == nullptr || layer < 0 || layer >= c->L || pos0 < 0 || count < 1) return BD_E_ARG;
  if (pos0 + count > c->cfg.max_seq) return BD_E_ARG;
  hipLaunchKernelGGL(read_kv_kernel, dim3(256), dim3(256), 0, c->stream, c->Kc + (size_t)layer * c->kv_layer_elems,
                     c->Vc + (size_t)layer * c->kv_layer_elems, c->cfg.n_kv_heads, c->D, c->max_kb, pos0, count,
                     dev_k_out, dev_v_out, 1, page_table(c));
  return check_launch();
}

int bd_read_carry(bd_ctx* c, int32_t* dev_cand, float* dev_conf) {
  if (c == nullptr) return BD_E_ARG;
  if (!c->carry_valid) return BD_E_STATE;
  if (dev_cand) HIP_TRY(hipMemcpyAsync(dev_cand, &c->st->carry_cand, 4, hipMemcpyDeviceToDevice, c->stream));
  if (dev_conf) HIP_TRY(hipMemcpyAsync(dev_conf, &c->st->carry_conf, 4, hipMemcpyDeviceToDevice, c->stream));
  return BD_OK;
}

int bd_read_rows(bd_ctx* c, int32_t* dev_cand, float* dev_conf, int rows) {
  if (c == nullptr || rows < 1 || rows > c->last_rows) return BD_E_ARG;
  if (dev_cand) HIP_TRY(hipMemcpyAsync(dev_cand, c->row_cand, (size_t)rows * 4, hipMemcpyDeviceToDevice, c->stream));
  if (dev_conf) HIP_TRY(hipMemcpyAsync(dev_conf, c->row_conf, (size_t)rows * 4, hipMemcpyDeviceToDevice, c->stream));
  return BD_OK;
}

int64_t bd_forward_bytes(const bd_ctx* c) {
  if (c == nullptr) return BD_E_ARG;
  const int64_t per_layer = (int64_t)c->H * c->NQKV + (int64_t)c->QD * c->H + 3ll * c->H * c->F;
  const int64_t w = c->fp8 ? (per_layer + 4ll * c->wscale_layer) * c->L + (int64_t)c->V * c->H * 2
                           : (per_layer * c->L + (int64_t)c->V * c->H) * 2;
  const int64_t kv = (int64_t)c->n * c->L * 2 * c->KVD * 2;
  return w + kv;
}

// ---- kernel-level entry points (include/bd_kernels.h) ---------------------------------------------------

int bd_k_profile(bd_ctx* c, int enable) {
  if (c == nullptr) return BD_E_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
  c->prof_ev.clear(); c->prof_cls.clear();
  c->prof_on = enable != 0;
  return BD_OK;
}

int bd_k_profile_read(bd_ctx* c, int kclass, double* total_ms, int* launches) {
  if (c == nullptr || kclass < 0 || kclass >= KC_COUNT) return BD_E_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  double tot = 0; int cnt = 0;
  for (size_t i = 0; i < c->prof_cls.size(); ++i) {
    if (c->prof_cls[i] != kclass) continue;
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
    tot += ms; ++cnt;
  }
  if (total_ms) *total_ms = tot;
  if (launches) *launches = cnt;
  return BD_OK;
}

int bd_k_stream_floor(bd_ctx* c, int repeats, double* host_ms, int64_t* host_bytes) {
  if (c == nullptr || repeats < 1 || host_ms == nullptr || !c->use_stream) return BD_E_ARG;
  const MegaPlan& P = c->plan;
  const int nw = P.nwg * kWavesPerWG;
  std::vector<unsigned> frags((size_t)nw);
  int64_t bytes = 0;
  for (int wg = 0; wg < P.nwg; ++wg)
    for (int w = 0; w < kWavesPerWG; ++w) {
      frags[(size_t)wg * kWavesPerWG + w] = (unsigned)((long long)P.L * wave_layer_units(P, wg, w) / 64);
      bytes += (int64_t)frags[(size_t)wg * kWavesPerWG + w] * 1024;
    }
  unsigned* d = nullptr;
  HIP_TRY(hipMalloc(reinterpret_cast<void**>(&d), (size_t)nw * 8));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = BD_OK;
  float ms = 0.f;
  auto run = [&]() -> int {
    HIP_TRY(hipMemcpyAsync(d, frags.data(), (size_t)nw * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    HIP_TRY(hipEventCreate(&e0));
    HIP_TRY(hipEventCreate(&e1));
    for (int i = 0; i < repeats + 1; ++i) {
      if (i == 1) HIP_TRY(hipEventRecord(e0, c->stream));      // (the first launch warms up)
      hipLaunchKernelGGL(stream_floor_kernel, dim3(P.nwg), dim3(256), 0, c->stream, reinterpret_cast<const floor_u32x4*>(c->wstream),
                         (long long)P.wave_stride, d, d + nw);
      BD_TRY(check_launch());
    }
    HIP_TRY(hipEventRecord(e1, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
    return BD_OK;
  };
  rc = run();
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(d);
  if (rc != BD_OK) return rc;
  *host_ms = (double)ms / repeats;
  if (host_bytes) *host_bytes = bytes;
  return BD_OK;
}

int bd_k_raise_device_error(bd_ctx* c) {
  if (c == nullptr) return BD_E_ARG;
  hipLaunchKernelGGL(raise_error_kernel, dim3(1), dim3(1), 0, c->stream, c->st);
  return check_launch();
}

int bd_k_trace(bd_ctx* c, int enable) {
  if (c == nullptr) return BD_E_ARG;
  const size_t n = (size_t)c->plan.nwg * (10 * c->L + 4 + 64);
  if (enable && c->trace == nullptr) {
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&c->trace), n * 8));
    c->allocs.push_back(c->trace);
  }
  if (enable) HIP_TRY(hipMemsetAsync(c->trace, 0, n * 8, c->stream));
  c->trace_on = enable ? 1 : 0;
  return BD_OK;
}

int bd_k_trace_read(bd_ctx* c, unsigned long long* host_out, int capacity, int* n_wg, int* per_wg) {
  if (c == nullptr || host_out == nullptr || c->trace == nullptr) return BD_E_ARG;
  const size_t n = (size_t)c->plan.nwg * (10 * c->L + 4 + 64);
  if ((size_t)capacity < n) return BD_E_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  HIP_TRY(hipMemcpy(host_out, c->trace, n * 8, hipMemcpyDeviceToHost));
  if (n_wg) *n_wg = c->plan.nwg;
  if (per_wg) *per_wg = 10 * c->L + 4;   /* followed by [n_wg][64] in-phase stamps of layer 1 */
  return BD_OK;
}

const char* bd_k_class_name(int kclass) {
  static const char* names[KC_COUNT] = {"prologue", "layers", "lm_head", "finish"};
  return (kclass >= 0 && kclass < KC_COUNT) ? names[kclass] : nullptr;
}

int bd_k_class_count(void) { return KC_COUNT; }

int64_t bd_k_class_bytes(const bd_ctx* c, int kclass) {
  if (c == nullptr) return BD_E_ARG;
  const int64_t lm = (int64_t)c->V * c->H * 2;
  if (kclass == KC_LAYERS) return bd_forward_bytes(c) - lm;
  if (kclass == KC_LMHEAD) return lm;
  return 0;
}

}  // extern "C"

