// Stand-alone block-causal attention on caller tensors (include/bd_kernels.h), on the attention kernel that the
// large-M path of the forward runs (prefill_attn.h: pf_attn_kernel, eight wavefronts per (head, 16-row tile) item):
// bd_k_attention allocates its working buffers per call; bd_k_attention_static runs the same kernels on a file-scope
// device array and allocates nothing.
#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/bd_kernels.h"
#include "launch.h"
#include "prefill_attn.h"

namespace bd {
namespace {

// Working buffers of one call (device memory beyond the caller's inputs and output): staging of the operands in the
// layouts the kernel reads, and of its packed result.
struct AttnBufs {
  u16* Kc; u16* Vc;          // packed bf16 caches [n_kv][max_kb][32*D]
  u16* q;                    // [Mp][n_q][D] bf16
  u16* ap;                   // packed bf16 output [Mp][n_q*D]
};
struct AttnShape {
  int n_prefix, M, n_q, n_kv, D, mode;
  int T, MT, Mp, max_kb;
  size_t kv_elems, q_elems, ap_elems;
};

int attn_shape(int n_prefix, int M, int n_q, int n_kv, int D, int mode, AttnShape* o) {
  if (M < 1 || M > 64 || n_prefix < 0 || n_q < 1 || n_kv < 1 || n_q % n_kv != 0 || (D != 64 && D != 128)) return BD_E_ARG;
  if (mode != BD_MODE_BIDIR && mode != BD_MODE_CAUSAL) return BD_E_ARG;
  AttnShape s{};
  s.n_prefix = n_prefix; s.M = M; s.n_q = n_q; s.n_kv = n_kv; s.D = D; s.mode = mode;
  s.T = n_prefix + M; s.MT = ceil_div(M, 16); s.Mp = s.MT * 16;
  s.max_kb = ceil_div(s.T, 32);
  s.kv_elems = (size_t)n_kv * s.max_kb * 32 * D;
  s.q_elems = (size_t)s.Mp * n_q * D;
  s.ap_elems = (size_t)ceil_div(n_q * D, 32) * 32 * s.Mp;
  *o = s;
  return BD_OK;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n_words) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}
__global__ void q_to_bf16_kernel(const float* __restrict__ src, u16* __restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = f32_to_bf16_bits(src[i]);
}
// packed bf16 result -> fp32 [M][K]
__global__ void unpack_x_kernel(const u16* __restrict__ xp, int M, int K, float* __restrict__ x, int MT) {
  const size_t total = (size_t)M * K;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int m = (int)(idx / K), k = (int)(idx % K);
    x[idx] = bf16_bits_to_f32(xp[xp_index(m, k, MT)]);
  }
}
// fp32 [T][n_kv][D] keys and values -> packed bf16 caches of one layer
__global__ void pack_kv_kernel(const float* __restrict__ k, const float* __restrict__ v, int T, int n_kv, int D,
                               int max_kb, u16* __restrict__ Kc, u16* __restrict__ Vc) {
  const size_t total = (size_t)T * n_kv * D;
  const size_t kv_head_elems = (size_t)max_kb * 32 * D;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int d = idx % D, h = (idx / D) % n_kv, p = (int)(idx / ((size_t)D * n_kv));
    Kc[h * kv_head_elems + kp_index(p, d, D / 32)] = f32_to_bf16_bits(k[idx]);
    Vc[h * kv_head_elems + vp_index(p, d, D / 16)] = f32_to_bf16_bits(v[idx]);
  }
}

int launch_attention(hipStream_t s, const AttnShape& sh, const AttnBufs& b) {
  PfAttnArgs t{};
  t.q = b.q; t.Kc = b.Kc; t.Vc = b.Vc; t.max_kb = sh.max_kb; t.n0 = sh.n_prefix; t.Mc = sh.Mp; t.n_q = sh.n_q; t.n_kv = sh.n_kv;
  t.scale_log2e = 1.4426950408889634f / std::sqrt((float)sh.D);
  t.out = b.ap; t.MTc = sh.MT; t.mode = sh.mode; t.Mvalid = sh.M; t.st = nullptr; t.skippable = 0; t.pages = nullptr;
  const int items = sh.n_q * sh.MT;
  if (sh.D == 128) hipLaunchKernelGGL((pf_attn_kernel<128, 8>), dim3(items), dim3(512), 0, s, t);
  else hipLaunchKernelGGL((pf_attn_kernel<64, 8>), dim3(items), dim3(512), 0, s, t);
  return check_launch();
}

// Operand conversion into the working buffers (which are clear), `iters` runs of the kernel, output conversion.
// All on stream s; the caller synchronises.
template <typename Repeat>
int attention_enqueue(hipStream_t s, const AttnShape& sh, const AttnBufs& b, const float* dev_q, const float* dev_k,
                      const float* dev_v, float* dev_out, Repeat&& repeat) {
  hipLaunchKernelGGL(pack_kv_kernel, dim3(1024), dim3(256), 0, s, dev_k, dev_v, sh.T, sh.n_kv, sh.D, sh.max_kb, b.Kc, b.Vc);
  hipLaunchKernelGGL(q_to_bf16_kernel, dim3(64), dim3(256), 0, s, dev_q, b.q, (size_t)sh.M * sh.n_q * sh.D);
  BD_TRY(check_launch());
  BD_TRY(repeat([&]() { return launch_attention(s, sh, b); }));
  hipLaunchKernelGGL(unpack_x_kernel, dim3(256), dim3(256), 0, s, b.ap, sh.M, sh.n_q * sh.D, dev_out, sh.MT);
  return check_launch();
}

struct TmpBufs {
  std::vector<void*> p;
  ~TmpBufs() { for (void* q : p) (void)hipFree(q); }
  template <typename T> int get(T** out, size_t bytes) {
    void* q = nullptr;
    HIP_TRY(hipMalloc(&q, bytes));
    HIP_TRY(hipMemset(q, 0, bytes));
    p.push_back(q);
    *out = static_cast<T*>(q);
    return BD_OK;
  }
};

// ---- the working buffers of bd_k_attention_static ------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)BD_K_ATTENTION_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, resolved on first use

int scratch_of_current_device(unsigned char** out) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) { set_last_error("device index %d out of range", dev); return BD_E_ARG; }
  if (g_scratch_ptr[dev] == nullptr) {
    unsigned char* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return BD_OK;
}

}  // namespace
}  // namespace bd

using namespace bd;

extern "C" int bd_k_attention(void* hip_stream, const float* dev_q, const float* dev_k, const float* dev_v,
                              int n_prefix, int M, int n_q, int n_kv, int D, int mode, float* dev_out, int iters,
                              float* avg_ms) {
  if (dev_q == nullptr || dev_k == nullptr || dev_v == nullptr || dev_out == nullptr || iters < 1) return BD_E_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  AttnShape sh;
  BD_TRY(attn_shape(n_prefix, M, n_q, n_kv, D, mode, &sh));
  TmpBufs t;
  AttnBufs b{};
  BD_TRY(t.get(&b.Kc, sh.kv_elems * 2));
  BD_TRY(t.get(&b.Vc, sh.kv_elems * 2));
  BD_TRY(t.get(&b.q, sh.q_elems * 2));
  BD_TRY(t.get(&b.ap, sh.ap_elems * 2));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  HIP_TRY(hipEventCreate(&e0));
  HIP_TRY(hipEventCreate(&e1));
  int rc = attention_enqueue(s, sh, b, dev_q, dev_k, dev_v, dev_out, [&](auto&& body) {
    int r = body();                                    // the first launch also serves as warm-up
    if (r == BD_OK && iters > 1) {
      (void)hipEventRecord(e0, s);
      for (int i = 0; i < iters && r == BD_OK; ++i) r = body();
      (void)hipEventRecord(e1, s);
    }
    return r;
  });
  const hipError_t e = hipStreamSynchronize(s);
  if (rc == BD_OK && e != hipSuccess) {
    set_last_error("kernel failed: %s", hipGetErrorString(e));
    rc = BD_E_HIP;
  }
  if (rc == BD_OK && avg_ms != nullptr) {
    float ms = 0.f;
    if (iters > 1) { (void)hipEventElapsedTime(&ms, e0, e1); ms /= (float)iters; }
    *avg_ms = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}

extern "C" int bd_k_attention_static(void* hip_stream, const float* dev_q, const float* dev_k, const float* dev_v,
                                     int n_prefix, int M, int n_q, int n_kv, int D, int mode, float* dev_out) {
  if (dev_q == nullptr || dev_k == nullptr || dev_v == nullptr || dev_out == nullptr) return BD_E_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  AttnShape sh;
  BD_TRY(attn_shape(n_prefix, M, n_q, n_kv, D, mode, &sh));
  // carve the working buffers out of the static array, each on a 256-byte boundary
  unsigned char* base = nullptr;
  BD_TRY(scratch_of_current_device(&base));
  size_t off = 0;
  auto carve = [&](size_t bytes) { const size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
  const size_t oK = carve(sh.kv_elems * 2), oV = carve(sh.kv_elems * 2), oq = carve(sh.q_elems * 2), oa = carve(sh.ap_elems * 2);
  const size_t clear_end = off;                        // all of it must start at zero (padding rows and keys)
  if (off > kScratchBytes) {
    set_last_error("bd_k_attention_static: this shape needs %zu bytes of working memory, the static buffer holds %zu", off,
                   kScratchBytes);
    return BD_E_CAPACITY;
  }
  AttnBufs b{};
  b.Kc = reinterpret_cast<u16*>(base + oK); b.Vc = reinterpret_cast<u16*>(base + oV);
  b.q = reinterpret_cast<u16*>(base + oq); b.ap = reinterpret_cast<u16*>(base + oa);
  // the array keeps the last call's contents: clear the staging buffers with a fill kernel (no memset node, so the call
  // can be captured into a graph)
  hipLaunchKernelGGL(fill_zero_kernel, dim3(512), dim3(256), 0, s, reinterpret_cast<uint32_t*>(base), clear_end / 4);
  BD_TRY(check_launch());
  return attention_enqueue(s, sh, b, dev_q, dev_k, dev_v, dev_out, [](auto&& body) { return body(); });
}
