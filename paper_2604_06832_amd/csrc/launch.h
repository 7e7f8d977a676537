// Launch interface between the host translation unit (bd_lib.hip) and the translation units that hold the kernels
// (k_stream.hip, k_mega.hip, k_prefill.hip, k_attention.hip): plain functions, so that the kernel files compile in
// parallel and none of them sees the context structure.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/bd.h"
#include "plan.h"
#include "prefill_args.h"

namespace bd {

// Records the message bd_last_error() returns (bd_lib.hip).
void set_last_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

#define HIP_TRY(expr)                                                                                    \
  do {                                                                                                   \
    hipError_t e__ = (expr);                                                                             \
    if (e__ != hipSuccess) {                                                                             \
      bd::set_last_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), __FILE__, __LINE__);     \
      return BD_E_HIP;                                                                                   \
    }                                                                                                    \
  } while (0)

#define BD_TRY(expr)                \
  do {                              \
    int rc__ = (expr);              \
    if (rc__ != BD_OK) return rc__; \
  } while (0)

inline int check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_last_error("kernel launch failed: %s", hipGetErrorString(e));
    return BD_E_HIP;
  }
  return BD_OK;
}

// k_stream.hip: the forward kernel with decoupled weight streaming, forwards of up to 32 rows (MT = 1, 2).
int launch_stream_fwd(hipStream_t s, int MT, int D, bool fp8, bool quad, const MegaArgs& a);
// Writes the XCD id of every workgroup of a launch shaped like the streaming forward kernel's to dev_out[nwg].
int launch_xcc_probe(hipStream_t s, int nwg, unsigned* dev_out);

// k_mega.hip: the register-ring forward kernel (MT = 1..4) and the LM head kernel.
int launch_mega_fwd(hipStream_t s, int MT, int D, bool quad, const MegaArgs& a);
int launch_lm_head(hipStream_t s, int MT, const MegaArgs& a);

// k_prefill.hip: one chunk of prompt rows through all layers with the large-M kernels.
int launch_prefill_chunk(hipStream_t s, const PfChunk& c);

}  // namespace bd
