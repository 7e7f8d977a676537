/*
 * bd.h - C ABI of the block-denoising decode library for MI355X (gfx950).
 *
 * The calls follow the paper's statement of block-diffusion decoding (Sec. 3.4 "Inference" and
 * Alg. 1 of the appendix "Details of Speculative Decoding"): a causal prefill builds the KV cache;
 * each block is seeded by one autoregressive prediction and then denoised step by step, every step
 * being one decoder forward over the B block positions with the whole cached prefix visible and
 * bidirectional attention inside the block, followed by a confidence-threshold unmask; a finished
 * block is committed to the cache by a causal forward.
 *
 * Conventions
 *   - Every function returns 0 (BD_OK) or a negative BD_E_* code; nothing aborts or throws.  A call
 *     refused for its arguments or its place in the call order (BD_E_ARG, BD_E_STATE, BD_E_CAPACITY,
 *     BD_E_DTYPE) writes no output argument and leaves the context as it was.  After BD_E_HIP (a launch
 *     or runtime call failed, or a bounded wait inside a kernel timed out) the cache and the carry are
 *     undefined: prefill again, or destroy the context if bd_status() reports the time-out.
 *   - "dev" pointers are device memory owned by the caller (for instance PyTorch tensors); "host"
 *     pointers are ordinary host memory.  The library never frees or keeps caller pointers beyond
 *     the call, except that work enqueued on the stream reads/writes dev buffers asynchronously:
 *     they must stay alive until the stream has run the call.
 *   - All GPU work is enqueued on the hipStream_t given to bd_create (NULL = the default stream).
 *     Calls return without synchronising unless stated.  A context is not thread-safe and belongs
 *     to one stream and one device (the device current at bd_create).
 *   - Token ids are int32.  The mask token id is fixed at creation (default vocab-1).
 *   - The library owns the device copies of the weights (repacked into MFMA operand order), the KV
 *     cache, the carry (prediction for the next uncached position) and all scratch memory.
 */
#ifndef BD_H_
#define BD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bd_ctx bd_ctx;

enum {
  BD_OK = 0,
  BD_E_ARG = -1,       /* null pointer, bad shape, B < 1 or B > max_block, unknown name ...      */
  BD_E_STATE = -2,     /* call out of order: weights missing, decode before prefill ...           */
  BD_E_CAPACITY = -3,  /* cache_len + B would exceed max_seq                                      */
  BD_E_DTYPE = -4,     /* unsupported storage type for this tensor                                */
  BD_E_HIP = -5        /* a HIP runtime call failed; bd_last_error() holds the text               */
};

enum { BD_F32 = 0, BD_BF16 = 1, BD_FP8_E4M3 = 2 };

/* In-block attention mode of a forward (Alg. 1: draft mask / verify mask). */
enum { BD_MODE_BIDIR = 0, BD_MODE_CAUSAL = 1 };

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rope_theta;      /* rotary base, 1e6 in every configuration                                  */
  float rms_eps;         /* RMSNorm epsilon, 1e-6                                                     */
  int32_t max_seq;       /* KV-cache capacity in positions (committed context + one block)           */
  int32_t max_block;     /* largest B of any call (<= 64; <= 32 with BD_FP8_E4M3 weights unless max_seq > 128) */
  int32_t mask_token_id; /* id embedded at masked positions; negative = vocab-1                       */
  int32_t weight_dtype;  /* device storage of the seven decoder linears: BD_BF16 or BD_FP8_E4M3       */
  int32_t flags;         /* 0, or BD_FLAG_* bits: alternative code paths, kept for the tests that compare them */
} bd_config;

/* bd_config.flags (0 is the product path; results are the same to rounding, see each flag): */
enum {
  BD_FLAG_CHIP_WIDE_HANDOVER = 1,  /* gate/up -> down hand-over through the chip-wide barrier instead of per XCD (bit-identical) */
  BD_FLAG_REGISTER_RING = 2,       /* forwards of <= 32 rows on the register-ring kernel instead of the streaming one (bf16)      */
  BD_FLAG_PREFILL_DECODE = 4,      /* no large-M kernels: prompts in chunks of max_block rows through the decode kernels, forwards */
                                   /* of 33..64 rows on the register-ring kernel (the only path when max_seq <= 128)              */
  BD_FLAG_PREFILL_STAGED = 8,      /* large-M GEMMs stage their operands through registers instead of loading straight into LDS  */
  BD_FLAG_ATTENTION_KEY_SPLIT = 16,/* attention of forwards of <= 32 rows by the chip-wide key split instead of per XCD           */
  BD_FLAG_MEASURE_NO_WEIGHTS = 32  /* MEASUREMENT ONLY, RESULTS ARE WRONG: the streaming kernel requests no weights, so a forward  */
                                   /* takes what its hand-overs, barriers and arithmetic cost without the stream                  */
};

/* Shape limits: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads; hidden, ffn, vocab and the
 * projection widths multiples of 16; hidden a multiple of 32. */
int bd_create(const bd_config* cfg, void* hip_stream, bd_ctx** out);
void bd_destroy(bd_ctx* ctx);

/* Upload one tensor.  name is one of "embed", "lm_head", "final_norm", "l<i>.attn_norm", "l<i>.wq",
 * "l<i>.wk", "l<i>.wv", "l<i>.wo", "l<i>.ffn_norm", "l<i>.w_gate", "l<i>.w_up", "l<i>.w_down".
 * host_ptr holds the row-major [out_features, in_features] matrix (or the gain vector) in `dtype`:
 * BD_F32 (rounded to bf16 on device), BD_BF16 (raw bits) or, for the seven linears of a
 * BD_FP8_E4M3 context, BD_FP8_E4M3 codes (OCP e4m3fn) with host_scales = one fp32 per output row
 * (the "W8A8 (FP8)" weights of the paper's "System integration" paragraph, here widened to bf16 in
 * registers and multiplied with bf16 activations: at B <= 32 the step is bound by weight bytes, not by
 * matrix throughput; embedding table and LM head stay bf16; other dtypes are refused for these seven).
 * Gain vectors are BD_F32 and must be loaded before the matrices they feed (attn_norm before wq/wk/wv,
 * ffn_norm before w_gate/w_up, final_norm before lm_head: the gain is folded into those matrices' columns;
 * BD_E_STATE otherwise).  The call copies synchronously; the caller keeps ownership of host_ptr. */
int bd_load_weight(bd_ctx* ctx, const char* name, const void* host_ptr, size_t bytes, int dtype,
                   const float* host_scales);

/* Alg. 1 prefill: causal forward over the prompt = n_embed continuous embeddings (dev fp32
 * [n_embed, hidden], may be NULL when n_embed is 0) followed by n_ids token ids (dev int32).  Resets
 * the cache, fills it with the prompt's K/V, sets the carry from the last prompt row.  A prompt of at
 * least 129 rows goes through large-M kernels in chunks of up to 1024 rows and only the final norm + LM
 * head of its last row through the decode path; shorter prompts are processed by the decode kernels in
 * chunks of at most max_block rows. */
int bd_prefill(bd_ctx* ctx, const float* dev_embeds, int n_embed, const int32_t* dev_ids, int n_ids);

/* One denoising step on the current block (Sec. 3.4; Alg. 1 draft step; "Decoding threshold").
 *   dev_block_tokens [B] in/out, dev_mask [B] in/out (1 = still masked).
 *   If mask[0] is set, position 0 first takes the carry's argmax (the autoregressive seed); this is
 *   not counted against fixed_k.  If B > 1, one forward then runs over the block (mask id embedded at
 *   masked positions, bidirectional in-block attention, cache untouched); the candidate and
 *   confidence of position i >= 1 come from row i-1.  Revealed are the masked positions with
 *   confidence > threshold, or the single most confident one if none clears it (ties: lowest
 *   position); with fixed_k > 0 instead exactly min(fixed_k, remaining) most confident positions.
 *   dev_n_unmasked (may be NULL): int32, number of positions revealed by this call (seed included).
 *   dev_conf_out (may be NULL): fp32 [B], confidence of the candidate for every position (position 0:
 *   the carry's). */
int bd_denoise_step(bd_ctx* ctx, int32_t* dev_block_tokens, uint8_t* dev_mask, int B, float threshold,
                    int fixed_k, int32_t* dev_n_unmasked, float* dev_conf_out);

/* Commit a fully decoded block: causal forward over its B tokens, K/V of every layer appended to
 * the cache, carry = prediction of the last row, cache_len += B.  The caller guarantees that no
 * token equals the mask id (not checked: it would need a device synchronisation). */
int bd_commit_block(bd_ctx* ctx, const int32_t* dev_block_tokens, int B);

/* Alg. 1 verify + accept on B drafted ids: causal forward; dev_ar_pred[j] (may be NULL) = argmax of
 * row j; *dev_n_accept (may be NULL) = length of the longest prefix of the draft in which draft[0]
 * equals the carry's argmax and draft[j+1] equals ar_pred[j].  commit != 0 appends all B positions
 * and moves the carry as bd_commit_block does (follow with bd_crop to drop rejected positions). */
int bd_verify_block(bd_ctx* ctx, const int32_t* dev_draft, int B, int commit, int32_t* dev_ar_pred,
                    int32_t* dev_n_accept);

/* A whole block with no host decision and no synchronisation in between (Sec. 3.4 block-by-block decoding with
 * confidence-aware parallel unmasking): seed from the carry, denoising steps until nothing is masked, commit.
 * The library enqueues as many steps as any block can need (B-1 under the threshold rule, ceil((B-1)/fixed_k)
 * under the fixed schedule); a flag on the device tells the kernels of the steps after the last useful one to do
 * nothing, so a block that completes early costs only their launches.
 * dev_tokens_out: device int32[B], the block's tokens.  dev_steps_out: device int32 (may be NULL), the number of
 * denoising forwards that really ran.  Errors as bd_denoise_step, plus BD_E_STATE without a valid carry. */
int bd_decode_block(bd_ctx* ctx, int B, float threshold, int fixed_k, int32_t* dev_tokens_out, int32_t* dev_steps_out);

/* One iteration of the linear self-speculative loop (appendix "Details of Speculative Decoding", Alg. 1), with no
 * host decision in between: the block [x_n, MASK, ...] (x_n = the carry's argmax, i.e. the token predicted for
 * position cache_len) is drafted in one bidirectional forward without cache update (row i-1 fills position i);
 * the draft is verified by one causal forward that writes K/V of all B positions; with a_j = argmax of causal
 * row j, k = 1 + the number of leading drafts d_1.. equal to a_0..; the k emitted tokens are a_0..a_{k-1}; the
 * cache keeps d_0..d_{k-1} (cache_len += k) and a_{k-1} becomes the carry.  B = 1 is one step of ordinary
 * autoregressive decoding.
 * dev_tokens_out: device int32[B]; entries [0, k) are the emitted tokens (all B predictions are written).
 * host_n_accepted: host int32, receives k (1 <= k <= B).  The call synchronises the stream to read k.
 * Errors: BD_E_STATE before prefill or without a valid carry (after bd_crop), BD_E_CAPACITY if
 * cache_len + B > max_seq, BD_E_ARG for NULL pointers or B outside [1, max_block]. */
int bd_speculative_step(bd_ctx* ctx, int B, int32_t* dev_tokens_out, int32_t* host_n_accepted);

/* Quadratic speculative decoding (appendix "Details of Speculative Decoding", Alg. 2): B <= max_block and either
 * B*(B+1) <= max_block rows (decode kernels) or, on a context with max_seq > 128 (large-M kernels, quadratic mask and
 * per-row positions there), B <= 32 (the block of the paper's model: 1056 rows) and B*(B+1) < max_seq; BD_E_ARG
 * otherwise.  (A BD_FP8_E4M3 context without the large-M kernels, max_seq <= 128, takes at most 32 rows.)
 * bd_quad_draft: step 1, the first block's draft: B mask tokens after the context, one bidirectional forward without
 *   cache update; dev_draft_out[0] = the carry's argmax, dev_draft_out[i] = argmax of the row before position i.
 * bd_quad_step: one iteration: a single forward over the B groups [draft[i], MASK x B] (group i at positions
 *   cache_len+i .. cache_len+i+B; a group's first token sees the prefix and the first tokens of the groups up to its
 *   own, every other token the prefix and its own group).  With P[i][j] = argmax of group i, entry j: k = 1 + the
 *   number of leading drafts draft[1..] equal to P[0][0], P[1][0], ..; draft[0..k-1] are the accepted tokens (draft[0]
 *   is exact by construction); their keys and values go to cache positions cache_len .. cache_len+k-1, cache_len += k,
 *   P[k-1][0] becomes the carry, and dev_next_draft[0..B-1] = P[k-1][0..B-1] is the draft of the next iteration.
 *   *host_n_accepted = k; the call synchronises the stream to read it.  dev_draft and dev_next_draft may not alias.
 *   The forward uses cache positions cache_len .. cache_len+B*(B+1)-1 as scratch: BD_E_CAPACITY if they do not fit. */
int bd_quad_draft(bd_ctx* ctx, int B, int32_t* dev_draft_out);
int bd_quad_step(bd_ctx* ctx, int B, const int32_t* dev_draft, int32_t* dev_next_draft, int32_t* host_n_accepted);

/* Alg. 1 Crop: forget cache positions >= new_len (0 <= new_len <= cache_len).  The carry becomes
 * undefined: the next block must bring its own first token (mask[0] = 0). */
int bd_crop(bd_ctx* ctx, int new_len);

/* Committed context length, or a negative error. */
/* Paged cache.  The cache of a context is a pool of max_seq/32 (rounded up) pages of 32 positions, each holding the keys
 * and values of those positions for every layer and kv head; block i of the sequence (positions 32 i .. 32 i + 31) lives
 * in whatever page the page list assigns to it, and every kernel follows that list.  Pages are taken from a free list
 * when a call first touches a block (prefill, any forward: the new rows' keys and values land at cache_len ..) and go
 * back to it when the context is cut (bd_crop, the crop inside a speculative or quadratic step, the reset of
 * bd_prefill), last block first.  Results do not depend on which pages hold which blocks.
 * bd_kv_page_order: the order in which free pages are handed out (host int32[n_pages], a permutation of 0 .. n_pages-1,
 *   n_pages = ceil(max_seq / 32)); default ascending.  BD_E_STATE while any page is in use (call it before bd_prefill or
 *   after bd_crop(ctx, 0)), BD_E_ARG for anything that is not such a permutation.
 * bd_kv_pages: returns the number of blocks in use and writes the page of block i to host_out[i] for i < capacity. */
int bd_kv_page_order(bd_ctx* ctx, const int32_t* host_order, int n_pages);
int bd_kv_pages(const bd_ctx* ctx, int32_t* host_out, int capacity);

int bd_cache_len(const bd_ctx* ctx);

/* Synchronise the stream and report the device-side state: BD_E_HIP if a grid barrier of the forward
 * kernel ever timed out (bounded wait), after which the context must be destroyed. */
int bd_status(bd_ctx* ctx);

/* ---- inspection, used by the parity tests -------------------------------------------------------- */

/* enable != 0: every later forward also stores its fp32 logits (costs vocab*B*4 bytes of writes). */
int bd_debug_logits(bd_ctx* ctx, int enable);
/* Copy the logits of the last forward: dev_out fp32 [rows, vocab], rows <= that forward's B. */
int bd_read_logits(bd_ctx* ctx, float* dev_out, int rows);
/* Unpack cache positions [pos0, pos0+count) of one layer to fp32 [count, n_kv_heads, head_dim]
 * (post-rotary K, and V).  Positions up to cache_len + last B are readable. */
int bd_read_kv(bd_ctx* ctx, int layer, int pos0, int count, float* dev_k_out, float* dev_v_out);
/* The carry: argmax id and its softmax probability (each may be NULL). */
int bd_read_carry(bd_ctx* ctx, int32_t* dev_cand, float* dev_conf);
/* Candidate id and confidence of every row of the last forward (row i predicts position i+1). */
int bd_read_rows(bd_ctx* ctx, int32_t* dev_cand, float* dev_conf, int rows);

/* Algorithmic HBM bytes of one forward at the current cache length: every weight matrix once plus
 * the cached K/V of all layers (what the roofline fraction is priced on). */
int64_t bd_forward_bytes(const bd_ctx* ctx);

const char* bd_strerror(int code);
/* Text of the last BD_E_HIP failure of this process (static storage). */
const char* bd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BD_H_ */
