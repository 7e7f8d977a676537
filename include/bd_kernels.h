/*
 * bd_kernels.h - kernel-level entry points of the block-denoising library.
 *
 * These expose block-causal attention on caller-provided tensors (the attention kernel that forwards of more than
 * 32 rows and the prompt pass run), per-kernel-class timing of a context, the in-kernel phase trace and the time of
 * the weight stream alone, so that tests can check one operation against the oracle and the benchmark can price
 * one kernel against its roofline.  The entry points themselves are not on the decode path.  Return codes as in
 * bd.h.
 */
#ifndef BD_KERNELS_H_
#define BD_KERNELS_H_

#include <stdint.h>

#include "bd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Block-causal grouped-query attention (Sec. 3.3 mask rules; Alg. 1 draft / verify masks) on explicit
 * operands: dev_q fp32 [M, n_q, D] (already rotated), dev_k / dev_v fp32 [n_prefix + M, n_kv, D] (prefix
 * keys first, then the block's own); all rounded to bf16 inside.  dev_out fp32 [M, n_q*D].
 * mode BD_MODE_BIDIR / BD_MODE_CAUSAL.  M <= 64, D in {64, 128}.  Allocates its working buffers per call
 * and synchronises the stream.  iters > 1 repeats the kernels and *avg_ms (host, may be NULL) receives the
 * mean time of one run. */
int bd_k_attention(void* hip_stream, const float* dev_q, const float* dev_k, const float* dev_v, int n_prefix, int M,
                   int n_q, int n_kv, int D, int mode, float* dev_out, int iters, float* avg_ms);

/* The same operation for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, layouts and result as bd_k_attention with
 * iters = 1, but every working buffer (packed K/V, bf16 Q, packed bf16 result) lives in one static device
 * array of BD_K_ATTENTION_STATIC_BYTES bytes that each GPU the library runs on holds until the process
 * ends.  The call allocates and frees nothing, records no memset node, only enqueues on hip_stream and
 * does not synchronise.  A shape whose working buffers exceed the array returns BD_E_CAPACITY (the text
 * from bd_last_error() names both sizes); bad arguments return BD_E_ARG as for bd_k_attention.  All calls
 * on one GPU share the array: calls that overlap in time on one GPU race, even on different streams. */
#define BD_K_ATTENTION_STATIC_BYTES (32u << 20)
int bd_k_attention_static(void* hip_stream, const float* dev_q, const float* dev_k, const float* dev_v, int n_prefix,
                          int M, int n_q, int n_kv, int D, int mode, float* dev_out);

/* Per-kernel-class timing of a context's forwards: enable brackets every launch with HIP events on
 * the context's stream (and drops earlier samples); read sums the elapsed time of one class. */
int bd_k_profile(bd_ctx* ctx, int enable);
int bd_k_profile_read(bd_ctx* ctx, int kclass, double* total_ms, int* launches);
int bd_k_class_count(void);
const char* bd_k_class_name(int kclass);
/* Algorithmic HBM bytes one launch of that class moves at the current cache length (weights of the
 * GEMM, or the layer's cached K/V for the attention); 0 for classes that stream nothing. */
int64_t bd_k_class_bytes(const bd_ctx* ctx, int kclass);

/* Phase trace of the forward kernel: with enable != 0 every workgroup stores a 100 MHz timestamp at each
 * phase boundary of the next forwards (start; then per layer: QKV done, barrier, attention done, barrier,
 * O done, barrier, gate/up done, barrier, down done, barrier; then LM head done, barrier).  read copies
 * the last forward's [n_wg][per_wg] table to host memory (capacity in entries). */
/* Measurement: time of reading the decoder layers' weight stream of one forward with no consumer, hand-over or barrier
 * (each wavefront its own contiguous share, as the streaming kernel's producers read it): mean of `repeats` launches
 * in milliseconds to *host_ms, the bytes read per launch to *host_bytes.  Synchronises the stream. */
int bd_k_stream_floor(bd_ctx* ctx, int repeats, double* host_ms, int64_t* host_bytes);

/* Test hook: raises the context's device-side error flag, as a forward kernel does when one of its bounded waits
 * gives up.  Every later forward kernel then returns at once (no kernel waits for anything), bd_status and the calls
 * that read a result back (bd_speculative_step, bd_quad_step) return BD_E_HIP, and the context stays unusable. */
int bd_k_raise_device_error(bd_ctx* ctx);

int bd_k_trace(bd_ctx* ctx, int enable);
int bd_k_trace_read(bd_ctx* ctx, unsigned long long* host_out, int capacity, int* n_wg, int* per_wg);

#ifdef __cplusplus
}
#endif
#endif /* BD_KERNELS_H_ */
