// Translation unit of the register-ring forward kernel and the LM head kernel (mega.h).
#include "launch.h"
#include "mega.h"

namespace bd {
namespace {

// Dynamic LDS the forward kernel needs: GEMM staging, or the attention phase's buffers if larger.
template <int MT>
constexpr int mega_lds_total() { return mega_lds_bytes<MT>() > 56 * 1024 ? mega_lds_bytes<MT>() : 56 * 1024; }

template <int MT, int D, bool QUAD>
int launch_mega_inst(hipStream_t s, const MegaArgs& a) {
  static bool attr_set = false;
  constexpr int lds = mega_lds_total<MT>();
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&mega_kernel<MT, D, 2, QUAD>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((mega_kernel<MT, D, 2, QUAD>), dim3(a.P.nwg), dim3(kWGThreads), lds, s, a);
  return check_launch();
}

template <int MT>
int launch_mega_mt(hipStream_t s, int D, bool quad, const MegaArgs& a) {
  if (quad) return D == 128 ? launch_mega_inst<MT, 128, true>(s, a) : launch_mega_inst<MT, 64, true>(s, a);
  return D == 128 ? launch_mega_inst<MT, 128, false>(s, a) : launch_mega_inst<MT, 64, false>(s, a);
}

template <int MT>
int launch_lm_inst(hipStream_t s, const MegaArgs& a) {
  static bool attr_set = false;
  constexpr int lds = mega_lds_total<MT>();
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&lm_kernel<MT>), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((lm_kernel<MT>), dim3(a.P.nwg), dim3(kWGThreads), lds, s, a);
  return check_launch();
}
}  // namespace

int launch_mega_fwd(hipStream_t s, int MT, int D, bool quad, const MegaArgs& a) {
  switch (MT) {
    case 1: return launch_mega_mt<1>(s, D, quad, a);
    case 2: return launch_mega_mt<2>(s, D, quad, a);
    case 3: return launch_mega_mt<3>(s, D, quad, a);
    case 4: return launch_mega_mt<4>(s, D, quad, a);
    default: return BD_E_ARG;
  }
}

int launch_lm_head(hipStream_t s, int MT, const MegaArgs& a) {
  switch (MT) {
    case 1: return launch_lm_inst<1>(s, a);
    case 2: return launch_lm_inst<2>(s, a);
    case 3: return launch_lm_inst<3>(s, a);
    case 4: return launch_lm_inst<4>(s, a);
    default: return BD_E_ARG;
  }
}

}  // namespace bd
