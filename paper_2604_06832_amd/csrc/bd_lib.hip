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

#include "attention.h"
#include "common.h"
#include "gemm.h"
#include "misc.h"

using namespace bd;

static char g_last_error[512] = "";

#define HIP_TRY(expr)                                                                                   \
  do {                                                                                                  \
    hipError_t e__ = (expr);                                                                            \
    if (e__ != hipSuccess) {                                                                            \
      snprintf(g_last_error, sizeof g_last_error, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), \
               __FILE__, __LINE__);                                                                     \
      return BD_E_HIP;                                                                                  \
    }                                                                                                   \
  } while (0)

#define BD_TRY(expr)            \
  do {                          \
    int rc__ = (expr);          \
    if (rc__ != BD_OK) return rc__; \
  } while (0)

namespace {

enum KClass {
  KC_GEMM_QKV = 0, KC_QKV_POST, KC_ATTN_PARTIAL, KC_ATTN_COMBINE, KC_GEMM_O, KC_RESID_NORM, KC_GEMM_GATEUP,
  KC_GEMM_DOWN, KC_GEMM_LMHEAD, KC_MISC, KC_COUNT
};

struct Layer {
  u16* wqkv = nullptr;   // packed [q|k|v] x hidden
  u16* wo = nullptr;     // packed hidden x q_dim
  u16* wgu = nullptr;    // packed, gate/up tiles interleaved, 2*ffn x hidden
  u16* wdown = nullptr;  // packed hidden x ffn
  float* g_attn = nullptr;
  float* g_ffn = nullptr;
  unsigned loaded = 0;   // bit per tensor
};

struct GemmPlan { int NT, ksplit, grid; };

}  // namespace

struct bd_ctx {
  bd_config cfg;
  hipStream_t stream = nullptr;
  int device = 0, num_cus = 256;
  int H, QD, KVD, NQKV, F, V, D, L, G;
  int Mp_max, max_kb;
  std::vector<Layer> layers;
  u16* embed = nullptr;
  u16* lm_head = nullptr;
  float* g_final = nullptr;
  unsigned loaded_top = 0;
  // KV cache, packed: [L][n_kv][max_kb][32*D] bf16 each
  u16* Kc = nullptr;
  u16* Vc = nullptr;
  size_t kv_layer_elems = 0;
  // workspaces
  float* x = nullptr;      // residual stream fp32 [Mp_max][H]
  u16* xp = nullptr;       // packed normalised activations (K = H)
  u16* q = nullptr;        // [Mp_max][n_q][D]
  u16* ap = nullptr;       // packed attention output (K = QD)
  u16* act = nullptr;      // packed SwiGLU output (K = F)
  float* ws = nullptr;     // split-K partials
  size_t ws_floats = 0;
  float2* rope = nullptr;
  float* pO = nullptr; float* pm = nullptr; float* pl = nullptr;
  int attn_items_max = 0;
  float* lm_max = nullptr; int* lm_idx = nullptr; float* lm_sum = nullptr;
  int lm_parts_max = 0;
  float* logits = nullptr; int logits_on = 0; int last_rows = 0; int last_had_logits = 0;
  int* row_cand = nullptr; float* row_conf = nullptr;
  DevState* st = nullptr;
  // host mirror of the decode state
  int n = 0;
  bool prefilled = false, carry_valid = false;
  // per-kernel-class timing (bd_k_profile)
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
      hipEventCreate(&e0); hipEventCreate(&e1);
      hipEventRecord(e0, c->stream);
    }
  }
  ~Prof() {
    if (c->prof_on) {
      hipEventRecord(e1, c->stream);
      c->prof_ev.push_back(e0); c->prof_ev.push_back(e1); c->prof_cls.push_back(cls);
    }
  }
};

int check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    snprintf(g_last_error, sizeof g_last_error, "kernel launch failed: %s", hipGetErrorString(e));
    return BD_E_HIP;
  }
  return BD_OK;
}

GemmPlan plan_gemm(const bd_ctx* c, int epi, int n_tiles, int KS, int MT) {
  GemmPlan p;
  if (epi == EPI_LMHEAD) {
    p.NT = (MT <= 2 && n_tiles % 4 == 0) ? 4 : ((n_tiles % 2 == 0) ? 2 : 1);
    p.ksplit = 1;
    p.grid = std::min(n_tiles / p.NT, std::min(c->lm_parts_max, 4 * c->num_cus));
    return p;
  }
  if (epi == EPI_SWIGLU) {
    p.NT = 2; p.ksplit = 1; p.grid = n_tiles / 2;
    return p;
  }
  p.NT = (n_tiles % 2 == 0) ? 2 : 1;
  const int groups = n_tiles / p.NT;
  int ks = (3 * c->num_cus / 2 + groups - 1) / groups;
  ks = std::max(1, std::min(ks, std::max(1, KS / 8)));
  ks = std::min(ks, 16);
  p.ksplit = ks;
  p.grid = groups * ks;
  return p;
}

template <int MT, int NT, int EPI>
void launch_gemm_t(const GemmArgs& a, int grid, hipStream_t s) {
  hipLaunchKernelGGL((gemm_kernel<MT, NT, EPI>), dim3(grid), dim3(kWGThreads), 0, s, a);
}

template <int EPI>
int launch_gemm_epi(const GemmArgs& a, int MT, int NT, int grid, hipStream_t s) {
#define BD_CASE(mt, nt) \
  if (MT == mt && NT == nt) { launch_gemm_t<mt, nt, EPI>(a, grid, s); return check_launch(); }
  if constexpr (EPI != EPI_SWIGLU) { BD_CASE(1, 1) BD_CASE(2, 1) BD_CASE(3, 1) BD_CASE(4, 1) }
  BD_CASE(1, 2) BD_CASE(2, 2) BD_CASE(3, 2) BD_CASE(4, 2)
  if constexpr (EPI == EPI_LMHEAD) { BD_CASE(1, 4) BD_CASE(2, 4) }
#undef BD_CASE
  snprintf(g_last_error, sizeof g_last_error, "no GEMM instance for MT=%d NT=%d", MT, NT);
  return BD_E_HIP;
}

// Y partials = Xp * Wp^T into c->ws; returns the split count used.
int gemm_partial(bd_ctx* c, int cls, const u16* Wp, const u16* Xp, int N, int K, int M, int* S_out) {
  const int MT = ceil_div(M, 16), KS = ceil_div(K, 32);
  GemmPlan p = plan_gemm(c, EPI_PARTIAL, N / 16, KS, MT);
  if ((size_t)p.ksplit * MT * 16 * N > c->ws_floats) {
    snprintf(g_last_error, sizeof g_last_error, "split-K workspace too small");
    return BD_E_HIP;
  }
  GemmArgs a{};
  a.Wp = reinterpret_cast<const bf16x8*>(Wp); a.Xp = reinterpret_cast<const bf16x8*>(Xp);
  a.n_tiles = N / 16; a.KS = KS; a.ksplit = p.ksplit; a.M = M; a.N = N; a.partial = c->ws;
  Prof pr(c, cls);
  BD_TRY(launch_gemm_epi<EPI_PARTIAL>(a, MT, p.NT, p.grid, c->stream));
  *S_out = p.ksplit;
  return BD_OK;
}

int resid_norm(bd_ctx* c, int S, int M, const float* gain) {
  const int MT = ceil_div(M, 16);
  Prof pr(c, KC_RESID_NORM);
  hipLaunchKernelGGL(resid_norm_kernel, dim3(M), dim3(kWGThreads), 0, c->stream, c->x, c->ws, S, MT * 16, c->H, gain,
                     c->cfg.rms_eps, c->xp, MT);
  return check_launch();
}

int attn_jt(const bd_ctx* c, int MT) {
  const int jt_total = c->G * MT;
  return (jt_total % 4 == 0) ? 4 : ((jt_total % 2 == 0) ? 2 : 1);
}

int attn_max_chunks(const bd_ctx* c, int MT) {
  const int JT = attn_jt(c, MT);
  const int groups = c->cfg.n_kv_heads * (c->G * MT / JT);
  int mc = (2 * c->num_cus) / groups;
  return std::max(1, std::min(mc, 128));
}

template <int D>
int launch_attention_d(bd_ctx* c, const AttnArgs& a, int JT, int grid_p, int grid_c) {
#define BD_ATT(jt)                                                                                             \
  if (JT == jt) {                                                                                              \
    { Prof pr(c, KC_ATTN_PARTIAL);                                                                             \
      hipLaunchKernelGGL((attn_partial_kernel<D, jt>), dim3(grid_p), dim3(kWGThreads), 0, c->stream, a);        \
      BD_TRY(check_launch()); }                                                                                \
    { Prof pr(c, KC_ATTN_COMBINE);                                                                             \
      hipLaunchKernelGGL((attn_combine_kernel<D, jt>), dim3(grid_c), dim3(kWGThreads), 0, c->stream, a);        \
      BD_TRY(check_launch()); }                                                                                \
    return BD_OK;                                                                                              \
  }
  BD_ATT(1) BD_ATT(2) BD_ATT(4)
#undef BD_ATT
  return BD_E_ARG;
}

int attention(bd_ctx* c, int layer, int M, int mode) {
  const int MT = ceil_div(M, 16);
  const int JT = attn_jt(c, MT);
  const int groups = c->cfg.n_kv_heads * (c->G * MT / JT);
  AttnArgs a{};
  a.Q = c->q;
  a.Kc = reinterpret_cast<const bf16x8*>(c->Kc + (size_t)layer * c->kv_layer_elems);
  a.Vc = reinterpret_cast<const bf16x8*>(c->Vc + (size_t)layer * c->kv_layer_elems);
  a.st = c->st;
  a.M = M; a.MT = MT; a.n_q = c->cfg.n_q_heads; a.n_kv = c->cfg.n_kv_heads; a.mode = mode; a.max_kb = c->max_kb;
  a.max_chunks = attn_max_chunks(c, MT);
  a.scale_log2e = 1.4426950408889634f / std::sqrt((float)c->D);
  a.pO = c->pO; a.pm = c->pm; a.pl = c->pl; a.out = c->ap;
  // the grid covers the chunks the current context length needs (the kernels recompute the same geometry)
  const int n_kb = ceil_div(c->n + M, 32);
  int chunk_len = std::max(kWavesPerWG, ceil_div(n_kb, a.max_chunks));
  const int n_chunks = ceil_div(n_kb, chunk_len);
  const int grid_p = groups * n_chunks;
  if (grid_p > c->attn_items_max) {
    snprintf(g_last_error, sizeof g_last_error, "attention partial buffer too small");
    return BD_E_HIP;
  }
  if (c->D == 128) return launch_attention_d<128>(c, a, JT, grid_p, groups);
  return launch_attention_d<64>(c, a, JT, grid_p, groups);
}

// One decoder forward over the M rows already sitting in c->x (fp32), positions n .. n+M-1.
// Writes the rows' K/V into the cache at those positions (the context length is not advanced here).
int forward(bd_ctx* c, int M, int mode, bool want_lm) {
  const int MT = ceil_div(M, 16);
  hipStream_t s = c->stream;
  {
    Prof pr(c, KC_MISC);
    hipLaunchKernelGGL(rope_table_kernel, dim3(M), dim3(64), 0, s, c->rope, c->st, c->D / 2, c->cfg.rope_theta);
    BD_TRY(check_launch());
  }
  BD_TRY(resid_norm(c, 0, M, c->layers[0].g_attn));
  for (int l = 0; l < c->L; ++l) {
    Layer& ly = c->layers[l];
    int S = 0;
    BD_TRY(gemm_partial(c, KC_GEMM_QKV, ly.wqkv, c->xp, c->NQKV, c->H, M, &S));
    {
      QkvPostArgs qa{};
      qa.partial = c->ws; qa.S = S; qa.Mp = MT * 16; qa.n_q = c->cfg.n_q_heads; qa.n_kv = c->cfg.n_kv_heads;
      qa.D = c->D; qa.max_kb = c->max_kb; qa.rope = c->rope; qa.st = c->st; qa.Q = c->q;
      qa.Kc = c->Kc + (size_t)l * c->kv_layer_elems; qa.Vc = c->Vc + (size_t)l * c->kv_layer_elems;
      Prof pr(c, KC_QKV_POST);
      hipLaunchKernelGGL(qkv_post_kernel, dim3(M), dim3(kWGThreads), 0, s, qa);
      BD_TRY(check_launch());
    }
    BD_TRY(attention(c, l, M, mode));
    BD_TRY(gemm_partial(c, KC_GEMM_O, ly.wo, c->ap, c->H, c->QD, M, &S));
    BD_TRY(resid_norm(c, S, M, ly.g_ffn));
    {
      GemmArgs a{};
      a.Wp = reinterpret_cast<const bf16x8*>(ly.wgu); a.Xp = reinterpret_cast<const bf16x8*>(c->xp);
      a.n_tiles = 2 * c->F / 16; a.KS = ceil_div(c->H, 32); a.ksplit = 1; a.M = M; a.N = 2 * c->F; a.act_out = c->act;
      GemmPlan p = plan_gemm(c, EPI_SWIGLU, a.n_tiles, a.KS, MT);
      Prof pr(c, KC_GEMM_GATEUP);
      BD_TRY(launch_gemm_epi<EPI_SWIGLU>(a, MT, p.NT, p.grid, s));
    }
    BD_TRY(gemm_partial(c, KC_GEMM_DOWN, ly.wdown, c->act, c->H, c->F, M, &S));
    BD_TRY(resid_norm(c, S, M, l + 1 < c->L ? c->layers[l + 1].g_attn : c->g_final));
  }
  c->last_rows = M;
  c->last_had_logits = 0;
  if (want_lm) {
    GemmArgs a{};
    a.Wp = reinterpret_cast<const bf16x8*>(c->lm_head); a.Xp = reinterpret_cast<const bf16x8*>(c->xp);
    a.n_tiles = c->V / 16; a.KS = ceil_div(c->H, 32); a.ksplit = 1; a.M = M; a.N = c->V;
    a.lm_max = c->lm_max; a.lm_idx = c->lm_idx; a.lm_sum = c->lm_sum;
    a.logits = c->logits_on ? c->logits : nullptr;
    GemmPlan p = plan_gemm(c, EPI_LMHEAD, a.n_tiles, a.KS, MT);
    Prof pr(c, KC_GEMM_LMHEAD);
    BD_TRY(launch_gemm_epi<EPI_LMHEAD>(a, MT, p.NT, p.grid, s));
    c->last_had_logits = c->logits_on;
  }
  return BD_OK;
}

int lm_parts(const bd_ctx* c, int M) {
  const int MT = ceil_div(M, 16);
  return plan_gemm(c, EPI_LMHEAD, c->V / 16, ceil_div(c->H, 32), MT).grid;
}

bool all_loaded(const bd_ctx* c) {
  if (c->loaded_top != 7u) return false;
  for (const Layer& l : c->layers)
    if (l.loaded != 0x1FFu) return false;
  return true;
}

int check_decode_call(const bd_ctx* c, int B) {
  if (c == nullptr) return BD_E_ARG;
  if (B < 1 || B > c->cfg.max_block) return BD_E_ARG;
  if (!c->prefilled) return BD_E_STATE;
  if (c->n + B > c->cfg.max_seq) return BD_E_CAPACITY;
  return BD_OK;
}

FinishArgs finish_args(bd_ctx* c, int B) {
  FinishArgs f{};
  f.lm_max = c->lm_max; f.lm_idx = c->lm_idx; f.lm_sum = c->lm_sum;
  f.n_parts = lm_parts(c, B); f.Mp = ceil_div(B, 16) * 16; f.B = B; f.st = c->st;
  f.row_cand = c->row_cand; f.row_conf = c->row_conf;
  return f;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------------
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
  if (k.weight_dtype == BD_FP8_E4M3) return BD_E_DTYPE;   // fp8 weight streaming is not built yet
  if (k.weight_dtype != BD_BF16) return BD_E_DTYPE;

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
  c->H = k.hidden; c->D = k.head_dim; c->QD = k.n_q_heads * k.head_dim; c->KVD = k.n_kv_heads * k.head_dim;
  c->NQKV = c->QD + 2 * c->KVD; c->F = k.ffn; c->V = k.vocab; c->L = k.n_layers; c->G = k.n_q_heads / k.n_kv_heads;
  c->Mp_max = ceil_div(k.max_block, 16) * 16;
  c->max_kb = ceil_div(k.max_seq, 32);
  c->layers.resize(c->L);
  c->kv_layer_elems = (size_t)k.n_kv_heads * c->max_kb * 32 * c->D;

  auto fail = [&](int rc) { bd_destroy(c); return rc; };
#define A(ptr, bytes) { int rc_ = dev_alloc(c, reinterpret_cast<void**>(&(ptr)), (bytes)); if (rc_ != BD_OK) return fail(rc_); }
  const size_t Mp = c->Mp_max;
  A(c->Kc, c->kv_layer_elems * c->L * 2);
  A(c->Vc, c->kv_layer_elems * c->L * 2);
  A(c->x, Mp * c->H * 4);
  A(c->xp, (size_t)ceil_div(c->H, 32) * 32 * Mp * 2);
  A(c->q, Mp * c->QD * 2);
  A(c->ap, (size_t)ceil_div(c->QD, 32) * 32 * Mp * 2);
  A(c->act, (size_t)ceil_div(c->F, 32) * 32 * Mp * 2);
  c->ws_floats = (size_t)16 * Mp * std::max(c->NQKV, c->H);
  A(c->ws, c->ws_floats * 4);
  A(c->rope, Mp * (c->D / 2) * sizeof(float2));
  {
    // attention partials: sized for the largest item count any (M, n) can produce
    int items = 0;
    for (int MT = 1; MT <= (int)Mp / 16; ++MT) {
      const int JT = attn_jt(c, MT);
      const int groups = k.n_kv_heads * (c->G * MT / JT);
      const int mc = attn_max_chunks(c, MT);
      items = std::max(items, groups * mc * JT);           // in units of one column tile
    }
    c->attn_items_max = items;                             // conservative: counts JT=1-sized items
    A(c->pO, (size_t)items * (c->D / 16) * 64 * 16);
    A(c->pm, (size_t)items * 16 * 4);
    A(c->pl, (size_t)items * 16 * 4);
  }
  c->lm_parts_max = 4 * c->num_cus;
  A(c->lm_max, (size_t)c->lm_parts_max * Mp * 4);
  A(c->lm_idx, (size_t)c->lm_parts_max * Mp * 4);
  A(c->lm_sum, (size_t)c->lm_parts_max * Mp * 4);
  A(c->row_cand, Mp * 4);
  A(c->row_conf, Mp * 4);
  A(c->st, sizeof(DevState));
  // weights
  A(c->embed, (size_t)c->V * c->H * 2);
  A(c->lm_head, (size_t)c->V * ceil_div(c->H, 32) * 32 * 2);
  A(c->g_final, (size_t)c->H * 4);
  for (Layer& l : c->layers) {
    A(l.wqkv, (size_t)c->NQKV * ceil_div(c->H, 32) * 32 * 2);
    A(l.wo, (size_t)c->H * ceil_div(c->QD, 32) * 32 * 2);
    A(l.wgu, (size_t)2 * c->F * ceil_div(c->H, 32) * 32 * 2);
    A(l.wdown, (size_t)c->H * ceil_div(c->F, 32) * 32 * 2);
    A(l.g_attn, (size_t)c->H * 4);
    A(l.g_ffn, (size_t)c->H * 4);
  }
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
  hipStreamSynchronize(c->stream);
  for (hipEvent_t e : c->prof_ev) hipEventDestroy(e);
  for (void* p : c->allocs) hipFree(p);
  if (c->logits) hipFree(c->logits);
  delete c;
}

int bd_load_weight(bd_ctx* c, const char* name, const void* host_ptr, size_t bytes, int dtype,
                   const float* host_scales) {
  if (c == nullptr || name == nullptr || host_ptr == nullptr) return BD_E_ARG;
  (void)host_scales;
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
  // destination, logical shape, packing placement
  int rows = 0, K = 0, tile_off = 0, tile_stride = 1, bit = -1;
  u16* dst = nullptr;
  float* gain_dst = nullptr;
  bool row_major_bf16 = false;
  if (layer < 0) {
    if (base == "embed") { rows = c->V; K = c->H; dst = c->embed; row_major_bf16 = true; bit = 0; }
    else if (base == "lm_head") { rows = c->V; K = c->H; dst = c->lm_head; bit = 1; }
    else if (base == "final_norm") { rows = c->H; gain_dst = c->g_final; bit = 2; }
    else return BD_E_ARG;
  } else {
    Layer& l = c->layers[layer];
    if (base == "attn_norm") { rows = c->H; gain_dst = l.g_attn; bit = 0; }
    else if (base == "ffn_norm") { rows = c->H; gain_dst = l.g_ffn; bit = 1; }
    else if (base == "wq") { rows = c->QD; K = c->H; dst = l.wqkv; tile_off = 0; bit = 2; }
    else if (base == "wk") { rows = c->KVD; K = c->H; dst = l.wqkv; tile_off = c->QD / 16; bit = 3; }
    else if (base == "wv") { rows = c->KVD; K = c->H; dst = l.wqkv; tile_off = (c->QD + c->KVD) / 16; bit = 4; }
    else if (base == "wo") { rows = c->H; K = c->QD; dst = l.wo; bit = 5; }
    else if (base == "w_gate") { rows = c->F; K = c->H; dst = l.wgu; tile_off = 0; tile_stride = 2; bit = 6; }
    else if (base == "w_up") { rows = c->F; K = c->H; dst = l.wgu; tile_off = 1; tile_stride = 2; bit = 7; }
    else if (base == "w_down") { rows = c->H; K = c->F; dst = l.wdown; bit = 8; }
    else return BD_E_ARG;
  }
  if (gain_dst != nullptr) {
    if (dtype != BD_F32) return BD_E_DTYPE;
    if (bytes != (size_t)rows * 4) return BD_E_ARG;
    HIP_TRY(hipMemcpy(gain_dst, host_ptr, bytes, hipMemcpyHostToDevice));
  } else {
    if (dtype != BD_F32 && dtype != BD_BF16) return BD_E_DTYPE;
    const size_t esz = dtype == BD_F32 ? 4 : 2;
    if (bytes != (size_t)rows * K * esz) return BD_E_ARG;
    void* stage = nullptr;
    HIP_TRY(hipMalloc(&stage, bytes));
    hipError_t e = hipMemcpy(stage, host_ptr, bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
      if (row_major_bf16) {
        if (dtype == BD_F32)
          hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(2048), dim3(256), 0, c->stream, (const float*)stage, dst,
                             (size_t)rows * K);
        else
          e = hipMemcpyAsync(dst, stage, bytes, hipMemcpyDeviceToDevice, c->stream);
      } else {
        const int KS = ceil_div(K, 32);
        if (dtype == BD_F32)
          hipLaunchKernelGGL(pack_weight_kernel<float>, dim3(2048), dim3(256), 0, c->stream, (const float*)stage,
                             (const float*)nullptr, rows, K, KS, dst, tile_off, tile_stride);
        else
          hipLaunchKernelGGL(pack_weight_kernel<u16>, dim3(2048), dim3(256), 0, c->stream, (const u16*)stage,
                             (const float*)nullptr, rows, K, KS, dst, tile_off, tile_stride);
      }
      if (e == hipSuccess) e = hipGetLastError();
      if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    }
    hipFree(stage);
    if (e != hipSuccess) {
      snprintf(g_last_error, sizeof g_last_error, "weight upload failed: %s", hipGetErrorString(e));
      return BD_E_HIP;
    }
  }
  if (layer < 0) c->loaded_top |= 1u << bit;
  else c->layers[layer].loaded |= 1u << bit;
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
  const int step = c->cfg.max_block;
  for (int off = 0; off < total; off += step) {
    const int M = std::min(step, total - off);
    const bool last = off + M >= total;
    hipLaunchKernelGGL(embed_kernel, dim3(M), dim3(256), 0, s, c->x, c->H, dev_embeds, n_embed, dev_ids, off,
                       (const uint8_t*)nullptr, c->cfg.mask_token_id, c->embed, c->V);
    BD_TRY(check_launch());
    BD_TRY(forward(c, M, BD_MODE_CAUSAL, last));
    if (last) {
      FinishArgs f = finish_args(c, M);
      f.commit = 1;
      hipLaunchKernelGGL(finish_causal_kernel, dim3(1), dim3(kWGThreads), 0, s, f);
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
  hipLaunchKernelGGL(seed_kernel, dim3(1), dim3(64), 0, s, dev_block_tokens, dev_mask, c->st);
  BD_TRY(check_launch());
  if (B == 1) {
    hipLaunchKernelGGL(finish_seed_only_kernel, dim3(1), dim3(64), 0, s, c->st, dev_n_unmasked, dev_conf_out);
    return check_launch();
  }
  hipLaunchKernelGGL(embed_kernel, dim3(B), dim3(256), 0, s, c->x, c->H, (const float*)nullptr, 0, dev_block_tokens, 0,
                     dev_mask, c->cfg.mask_token_id, c->embed, c->V);
  BD_TRY(check_launch());
  BD_TRY(forward(c, B, BD_MODE_BIDIR, true));
  FinishArgs f = finish_args(c, B);
  f.tokens = dev_block_tokens; f.mask = dev_mask; f.threshold = threshold; f.fixed_k = fixed_k;
  f.n_unmasked = dev_n_unmasked; f.conf_out = dev_conf_out;
  Prof pr(c, KC_MISC);
  hipLaunchKernelGGL(finish_denoise_kernel, dim3(1), dim3(kWGThreads), 0, s, f);
  return check_launch();
}

static int causal_pass(bd_ctx* c, const int32_t* dev_tokens, int B, int commit, int32_t* dev_ar_pred,
                       int32_t* dev_n_accept, const int32_t* draft) {
  hipStream_t s = c->stream;
  hipLaunchKernelGGL(embed_kernel, dim3(B), dim3(256), 0, s, c->x, c->H, (const float*)nullptr, 0, dev_tokens, 0,
                     (const uint8_t*)nullptr, c->cfg.mask_token_id, c->embed, c->V);
  BD_TRY(check_launch());
  BD_TRY(forward(c, B, BD_MODE_CAUSAL, true));
  FinishArgs f = finish_args(c, B);
  f.draft = draft; f.commit = commit; f.ar_pred = dev_ar_pred; f.n_accept = dev_n_accept;
  {
    Prof pr(c, KC_MISC);
    hipLaunchKernelGGL(finish_causal_kernel, dim3(1), dim3(kWGThreads), 0, s, f);
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

int bd_crop(bd_ctx* c, int new_len) {
  if (c == nullptr) return BD_E_ARG;
  if (!c->prefilled) return BD_E_STATE;
  if (new_len < 0 || new_len > c->n) return BD_E_ARG;
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, c->stream, c->st, new_len, 1);
  BD_TRY(check_launch());
  c->n = new_len;
  c->carry_valid = false;
  return BD_OK;
}

int bd_cache_len(const bd_ctx* c) { return c == nullptr ? BD_E_ARG : c->n; }

int bd_debug_logits(bd_ctx* c, int enable) {
  if (c == nullptr) return BD_E_ARG;
  if (enable && c->logits == nullptr) HIP_TRY(hipMalloc(reinterpret_cast<void**>(&c->logits), (size_t)c->Mp_max * c->V * 4));
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
                     dev_k_out, dev_v_out);
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
  const int64_t w = (per_layer * c->L + (int64_t)c->V * c->H) * 2;
  const int64_t kv = (int64_t)c->n * c->L * 2 * c->KVD * 2;
  return w + kv;
}

// ---- kernel-level entry points (include/bd_kernels.h) ---------------------------------------------------

int bd_k_profile(bd_ctx* c, int enable) {
  if (c == nullptr) return BD_E_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (hipEvent_t e : c->prof_ev) hipEventDestroy(e);
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

const char* bd_k_class_name(int kclass) {
  static const char* names[KC_COUNT] = {"gemm_qkv", "qkv_post", "attn_partial", "attn_combine", "gemm_o", "resid_norm",
                                        "gemm_gateup_swiglu", "gemm_down", "gemm_lmhead", "misc"};
  return (kclass >= 0 && kclass < KC_COUNT) ? names[kclass] : nullptr;
}

int bd_k_class_count(void) { return KC_COUNT; }

int64_t bd_k_class_bytes(const bd_ctx* c, int kclass) {
  if (c == nullptr) return BD_E_ARG;
  switch (kclass) {
    case KC_GEMM_QKV: return (int64_t)c->H * c->NQKV * 2;
    case KC_GEMM_O: return (int64_t)c->QD * c->H * 2;
    case KC_GEMM_GATEUP: return 2ll * c->H * c->F * 2;
    case KC_GEMM_DOWN: return (int64_t)c->H * c->F * 2;
    case KC_GEMM_LMHEAD: return (int64_t)c->V * c->H * 2;
    case KC_ATTN_PARTIAL: return (int64_t)c->n * 2 * c->KVD * 2;
    default: return 0;
  }
}

}  // extern "C"

namespace {
struct TmpBufs {
  std::vector<void*> p;
  ~TmpBufs() { for (void* q : p) hipFree(q); }
  template <typename T> int get(T** out, size_t bytes) {
    void* q = nullptr;
    HIP_TRY(hipMalloc(&q, bytes));
    HIP_TRY(hipMemset(q, 0, bytes));
    p.push_back(q);
    *out = static_cast<T*>(q);
    return BD_OK;
  }
};

int timed_loop(hipStream_t s, int iters, float* avg_ms, const std::function<int()>& body) {
  hipEvent_t e0, e1;
  HIP_TRY(hipEventCreate(&e0));
  HIP_TRY(hipEventCreate(&e1));
  int rc = body();                                   // first launch also serves as warm-up
  if (rc == BD_OK && iters > 1) {
    hipEventRecord(e0, s);
    for (int i = 0; i < iters && rc == BD_OK; ++i) rc = body();
    hipEventRecord(e1, s);
  }
  hipError_t e = hipStreamSynchronize(s);
  if (rc == BD_OK && e != hipSuccess) {
    snprintf(g_last_error, sizeof g_last_error, "kernel failed: %s", hipGetErrorString(e));
    rc = BD_E_HIP;
  }
  if (rc == BD_OK && avg_ms != nullptr) {
    float ms = 0.f;
    if (iters > 1) { hipEventElapsedTime(&ms, e0, e1); ms /= (float)iters; }
    *avg_ms = ms;
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  return rc;
}
}  // namespace

extern "C" int bd_k_gemm(void* hip_stream, const uint16_t* dev_w, const float* dev_x, int M, int N, int K,
                         float* dev_y, int iters, float* avg_ms) {
  if (dev_w == nullptr || dev_x == nullptr || dev_y == nullptr) return BD_E_ARG;
  if (M < 1 || M > 64 || N < 16 || N % 16 != 0 || K < 1 || iters < 1) return BD_E_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int MT = ceil_div(M, 16), KS = ceil_div(K, 32);
  bd_ctx fake;                                       // only the fields the planner reads
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, dev));
  fake.num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  GemmPlan p = plan_gemm(&fake, EPI_PARTIAL, N / 16, KS, MT);
  TmpBufs t;
  u16 *wp, *xp; float* ws;
  BD_TRY(t.get(&wp, (size_t)N * KS * 32 * 2));
  BD_TRY(t.get(&xp, (size_t)KS * 32 * MT * 16 * 2));
  BD_TRY(t.get(&ws, (size_t)p.ksplit * MT * 16 * N * 4));
  hipLaunchKernelGGL(pack_weight_kernel<u16>, dim3(2048), dim3(256), 0, s, dev_w, (const float*)nullptr, N, K, KS, wp, 0, 1);
  hipLaunchKernelGGL(pack_x_kernel, dim3(256), dim3(256), 0, s, dev_x, M, K, xp, MT);
  BD_TRY(check_launch());
  GemmArgs a{};
  a.Wp = reinterpret_cast<const bf16x8*>(wp); a.Xp = reinterpret_cast<const bf16x8*>(xp);
  a.n_tiles = N / 16; a.KS = KS; a.ksplit = p.ksplit; a.M = M; a.N = N; a.partial = ws;
  BD_TRY(timed_loop(s, iters, avg_ms, [&]() { return launch_gemm_epi<EPI_PARTIAL>(a, MT, p.NT, p.grid, s); }));
  hipLaunchKernelGGL(reduce_partial_kernel, dim3(512), dim3(256), 0, s, ws, p.ksplit, MT * 16, N, M, dev_y);
  BD_TRY(check_launch());
  HIP_TRY(hipStreamSynchronize(s));
  return BD_OK;
}

extern "C" int bd_k_attention(void* hip_stream, const float* dev_q, const float* dev_k, const float* dev_v,
                              int n_prefix, int M, int n_q, int n_kv, int D, int mode, float* dev_out, int iters,
                              float* avg_ms) {
  if (dev_q == nullptr || dev_k == nullptr || dev_v == nullptr || dev_out == nullptr) return BD_E_ARG;
  if (M < 1 || M > 64 || n_prefix < 0 || n_q < 1 || n_kv < 1 || n_q % n_kv != 0 || (D != 64 && D != 128)) return BD_E_ARG;
  if ((mode != BD_MODE_BIDIR && mode != BD_MODE_CAUSAL) || iters < 1) return BD_E_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, dev));
  bd_ctx c;                                          // a context shell holding just the attention state
  c.stream = s;
  c.num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  c.cfg.n_q_heads = n_q; c.cfg.n_kv_heads = n_kv; c.D = D; c.G = n_q / n_kv; c.QD = n_q * D;
  const int T = n_prefix + M, MT = ceil_div(M, 16), Mp = MT * 16;
  c.max_kb = ceil_div(T, 32);
  c.kv_layer_elems = (size_t)n_kv * c.max_kb * 32 * D;
  c.n = n_prefix;
  TmpBufs t;
  const int JT = attn_jt(&c, MT);
  const int groups = n_kv * (c.G * MT / JT);
  const int mc = attn_max_chunks(&c, MT);
  c.attn_items_max = groups * mc;
  BD_TRY(t.get(&c.Kc, c.kv_layer_elems * 2));
  BD_TRY(t.get(&c.Vc, c.kv_layer_elems * 2));
  BD_TRY(t.get(&c.q, (size_t)Mp * n_q * D * 2));
  BD_TRY(t.get(&c.ap, (size_t)ceil_div(c.QD, 32) * 32 * Mp * 2));
  BD_TRY(t.get(&c.pO, (size_t)c.attn_items_max * JT * (D / 16) * 64 * 16));
  BD_TRY(t.get(&c.pm, (size_t)c.attn_items_max * JT * 16 * 4));
  BD_TRY(t.get(&c.pl, (size_t)c.attn_items_max * JT * 16 * 4));
  BD_TRY(t.get(&c.st, sizeof(DevState)));
  hipLaunchKernelGGL(set_state_kernel, dim3(1), dim3(1), 0, s, c.st, n_prefix, 1);
  hipLaunchKernelGGL(pack_kv_kernel, dim3(1024), dim3(256), 0, s, dev_k, dev_v, T, n_kv, D, c.max_kb, c.Kc, c.Vc);
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(64), dim3(256), 0, s, dev_q, c.q, (size_t)M * n_q * D);
  BD_TRY(check_launch());
  BD_TRY(timed_loop(s, iters, avg_ms, [&]() { return attention(&c, 0, M, mode); }));
  hipLaunchKernelGGL(unpack_x_kernel, dim3(256), dim3(256), 0, s, c.ap, M, c.QD, dev_out, MT);
  BD_TRY(check_launch());
  HIP_TRY(hipStreamSynchronize(s));
  return BD_OK;
}
