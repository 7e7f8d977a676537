// Translation unit of the streaming forward kernel (stream_fwd.h): its instantiations and their launchers.
#include "launch.h"
#include "stream_fwd.h"

namespace bd {

// Writes the XCD id of every workgroup of a launch shaped like the forward kernel's (host-side check of the
// workgroup -> XCD rule before a plan relies on it).
__global__ __launch_bounds__(kFwdThreads, 1) void xcc_probe_kernel(unsigned* out) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  if (threadIdx.x == 0) { lds[0] = 1; out[blockIdx.x] = xcc_id(); }
}

int launch_xcc_probe(hipStream_t s, int nwg, unsigned* dev_out) {
  static bool attr_set = false;
  constexpr int lds = stream_lds_bytes<2>();
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&xcc_probe_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  hipLaunchKernelGGL(xcc_probe_kernel, dim3(nwg), dim3(kFwdThreads), lds, s, dev_out);
  return check_launch();
}

namespace {
template <int MT, int D, bool FP8, bool QUAD>
int launch_inst(hipStream_t s, const MegaArgs& a) {
  static bool attr_set = false;
  constexpr int lds = stream_lds_bytes<MT>();
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_fwd_kernel<MT, D, FP8, QUAD>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((stream_fwd_kernel<MT, D, FP8, QUAD>), dim3(a.P.nwg), dim3(kFwdThreads), lds, s, a);
  return check_launch();
}

template <int MT, int D>
int launch_d(hipStream_t s, bool fp8, bool quad, const MegaArgs& a) {
  if (quad) return fp8 ? launch_inst<MT, D, true, true>(s, a) : launch_inst<MT, D, false, true>(s, a);   // quadratic mask (Alg. 2)
  return fp8 ? launch_inst<MT, D, true, false>(s, a) : launch_inst<MT, D, false, false>(s, a);
}
}  // namespace

int launch_stream_fwd(hipStream_t s, int MT, int D, bool fp8, bool quad, const MegaArgs& a) {
  if (MT == 1) return D == 128 ? launch_d<1, 128>(s, fp8, quad, a) : launch_d<1, 64>(s, fp8, quad, a);
  if (MT == 2) return D == 128 ? launch_d<2, 128>(s, fp8, quad, a) : launch_d<2, 64>(s, fp8, quad, a);
  return BD_E_ARG;
}

}  // namespace bd
