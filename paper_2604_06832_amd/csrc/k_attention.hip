// Stand-alone block-causal attention on caller tensors (include/bd_kernels.h): bd_k_attention allocates its working
// buffers per call; bd_k_attention_static runs the same kernels on a file-scope device array and allocates nothing.
#include <algorithm>
#include <cmath>
#include <vector>

#include "../../include/bd_kernels.h"
#include "attention.h"
#include "launch.h"

namespace bd {
namespace {

// Working buffers of one call (device memory beyond the caller's inputs and output).
struct AttnBufs {
  u16* Kc; u16* Vc;          // packed bf16 caches [n_kv][max_kb][32*D]
  u16* q;                    // [Mp][n_q][D] bf16
  u16* ap;                   // packed bf16 output [Mp][n_q*D]
  float* pO; float* pm; float* pl;   // per-item partials
  DevState* st;
};
struct AttnShape {
  int n_prefix, M, n_q, n_kv, D, mode;
  int T, MT, Mp, G, JT, groups, max_chunks, items_max, max_kb;
  size_t kv_elems, q_elems, ap_elems, pO_floats, pml_floats;
};

int attn_shape(int num_cus, int n_prefix, int M, int n_q, int n_kv, int D, int mode, AttnShape* o) {
  if (M < 1 || M > 64 || n_prefix < 0 || n_q < 1 || n_kv < 1 || n_q % n_kv != 0 || (D != 64 && D != 128)) return BD_E_ARG;
  if (mode != BD_MODE_BIDIR && mode != BD_MODE_CAUSAL) return BD_E_ARG;
  AttnShape s{};
  s.n_prefix = n_prefix; s.M = M; s.n_q = n_q; s.n_kv = n_kv; s.D = D; s.mode = mode;
  s.T = n_prefix + M; s.MT = ceil_div(M, 16); s.Mp = s.MT * 16; s.G = n_q / n_kv;
  const int jt_total = s.G * s.MT;
  s.JT = (jt_total % 4 == 0) ? 4 : ((jt_total % 2 == 0) ? 2 : 1);   // column tiles per item
  s.groups = n_kv * (jt_total / s.JT);
  s.max_chunks = std::max(1, std::min((2 * num_cus) / s.groups, 64));
  s.items_max = s.groups * s.max_chunks;
  s.max_kb = ceil_div(s.T, 32);
  s.kv_elems = (size_t)n_kv * s.max_kb * 32 * D;
  s.q_elems = (size_t)s.Mp * n_q * D;
  s.ap_elems = (size_t)ceil_div(n_q * D, 32) * 32 * s.Mp;
  s.pO_floats = (size_t)s.items_max * s.JT * (D / 16) * 64 * 4;
  s.pml_floats = (size_t)s.items_max * s.JT * 16;
  *o = s;
  return BD_OK;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n_words) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}
__global__ void attn_state_kernel(DevState* st, int n) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { st->n = n; st->error = 0; }
}
__global__ void q_to_bf16_kernel(const float* __restrict__ src, u16* __restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = f32_to_bf16_bits(src[i]);
}

template <int D>
int launch_attention_d(hipStream_t s, const AttnArgs& a, int JT, int grid_p, int grid_c) {
#define BD_ATT(jt)                                                                                      \
  if (JT == jt) {                                                                                       \
    hipLaunchKernelGGL((attn_partial_kernel<D, jt>), dim3(grid_p), dim3(kWGThreads), 0, s, a);           \
    BD_TRY(check_launch());                                                                             \
    hipLaunchKernelGGL((attn_combine_kernel<D, jt>), dim3(grid_c), dim3(kWGThreads), 0, s, a);           \
    return check_launch();                                                                              \
  }
  BD_ATT(1) BD_ATT(2) BD_ATT(4)
#undef BD_ATT
  return BD_E_ARG;
}

int launch_attention(hipStream_t s, const AttnShape& sh, const AttnBufs& b) {
  AttnArgs a{};
  a.Q = b.q;
  a.Kc = reinterpret_cast<const bf16x8*>(b.Kc);
  a.Vc = reinterpret_cast<const bf16x8*>(b.Vc);
  a.st = b.st;
  a.M = sh.M; a.MT = sh.MT; a.n_q = sh.n_q; a.n_kv = sh.n_kv; a.mode = sh.mode; a.max_kb = sh.max_kb;
  a.max_chunks = sh.max_chunks;
  a.scale_log2e = 1.4426950408889634f / std::sqrt((float)sh.D);
  a.pO = b.pO; a.pm = b.pm; a.pl = b.pl; a.out = b.ap;
  const int n_kb = ceil_div(sh.T, 32);
  const int chunk_len = std::max(kWavesPerWG, ceil_div(n_kb, a.max_chunks));
  const int n_chunks = ceil_div(n_kb, chunk_len);
  const int grid_p = sh.groups * n_chunks;
  if (grid_p > sh.items_max) return BD_E_ARG;
  if (sh.D == 128) return launch_attention_d<128>(s, a, sh.JT, grid_p, sh.groups);
  return launch_attention_d<64>(s, a, sh.JT, grid_p, sh.groups);
}

// Operand conversion into the working buffers (which are clear), `iters` runs of the two kernels, output conversion.
// All on stream s; the caller synchronises.
template <typename Repeat>
int attention_enqueue(hipStream_t s, const AttnShape& sh, const AttnBufs& b, const float* dev_q, const float* dev_k,
                      const float* dev_v, float* dev_out, Repeat&& repeat) {
  hipLaunchKernelGGL(attn_state_kernel, dim3(1), dim3(1), 0, s, b.st, sh.n_prefix);
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

int num_cus_of_current_device(int* out) {
  int dev = 0, n = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
  *out = n > 0 ? n : 256;
  return BD_OK;
}

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
  int cus = 0;
  BD_TRY(num_cus_of_current_device(&cus));
  AttnShape sh;
  BD_TRY(attn_shape(cus, n_prefix, M, n_q, n_kv, D, mode, &sh));
  TmpBufs t;
  AttnBufs b{};
  BD_TRY(t.get(&b.Kc, sh.kv_elems * 2));
  BD_TRY(t.get(&b.Vc, sh.kv_elems * 2));
  BD_TRY(t.get(&b.q, sh.q_elems * 2));
  BD_TRY(t.get(&b.ap, sh.ap_elems * 2));
  BD_TRY(t.get(&b.pO, sh.pO_floats * 4));
  BD_TRY(t.get(&b.pm, sh.pml_floats * 4));
  BD_TRY(t.get(&b.pl, sh.pml_floats * 4));
  BD_TRY(t.get(&b.st, sizeof(DevState)));
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
  int cus = 0;
  BD_TRY(num_cus_of_current_device(&cus));
  AttnShape sh;
  BD_TRY(attn_shape(cus, n_prefix, M, n_q, n_kv, D, mode, &sh));
  // carve the working buffers out of the static array, each on a 256-byte boundary
  unsigned char* base = nullptr;
  BD_TRY(scratch_of_current_device(&base));
  size_t off = 0;
  auto carve = [&](size_t bytes) { const size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
  const size_t oK = carve(sh.kv_elems * 2), oV = carve(sh.kv_elems * 2), oq = carve(sh.q_elems * 2), oa = carve(sh.ap_elems * 2);
  const size_t clear_end = off;                        // everything up to here must start at zero (padding rows and keys)
  const size_t oO = carve(sh.pO_floats * 4), om = carve(sh.pml_floats * 4), ol = carve(sh.pml_floats * 4), os = carve(sizeof(DevState));
  if (off > kScratchBytes) {
    set_last_error("bd_k_attention_static: this shape needs %zu bytes of working memory, the static buffer holds %zu", off,
                   kScratchBytes);
    return BD_E_CAPACITY;
  }
  AttnBufs b{};
  b.Kc = reinterpret_cast<u16*>(base + oK); b.Vc = reinterpret_cast<u16*>(base + oV);
  b.q = reinterpret_cast<u16*>(base + oq); b.ap = reinterpret_cast<u16*>(base + oa);
  b.pO = reinterpret_cast<float*>(base + oO); b.pm = reinterpret_cast<float*>(base + om); b.pl = reinterpret_cast<float*>(base + ol);
  b.st = reinterpret_cast<DevState*>(base + os);
  // the array keeps the last call's contents: clear the operand buffers with a fill kernel (no memset node, so the call
  // can be captured into a graph); the partials are fully written by the first kernel before the second reads them
  hipLaunchKernelGGL(fill_zero_kernel, dim3(512), dim3(256), 0, s, reinterpret_cast<uint32_t*>(base), clear_end / 4);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(base + os), sizeof(DevState) / 4);
  BD_TRY(check_launch());
  return attention_enqueue(s, sh, b, dev_q, dev_k, dev_v, dev_out, [](auto&& body) { return body(); });
}
