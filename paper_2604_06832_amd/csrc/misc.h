// Small kernels around the forward: cache read-back for the tests and the per-step decision kernels (seed, unmask,
// commit, verify-accept, quadratic accept).  Compiled into the host translation unit only.
#pragma once
#include "common.h"

namespace bd {

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned floor_u32x4;

// Measurement only: every wavefront reads the weight stream of one forward's layers exactly as the producers of the
// streaming forward kernel lay it out (wavefront w of workgroup b: its own contiguous range, 1 KiB per load, sixteen
// loads in flight), with no consumer, no hand-over and no barrier: the time the bytes alone take on this chip.
__global__ __launch_bounds__(256) void stream_floor_kernel(const floor_u32x4* __restrict__ wstream, long long wave_stride_units,
                                                            const unsigned* __restrict__ frags, unsigned* __restrict__ out) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int sw = blockIdx.x * 4 + wave;
  const floor_u32x4* src = wstream + (size_t)sw * wave_stride_units + lane;
  const unsigned total = frags[sw];
  unsigned acc = 0;
  unsigned f = 0;
  for (; f + 16 <= total; f += 16) {
    floor_u32x4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = __builtin_nontemporal_load(src + (size_t)(f + j) * 64);
#pragma unroll
    for (int j = 0; j < 16; ++j) acc ^= v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
  }
  for (; f < total; ++f) {
    const floor_u32x4 v = __builtin_nontemporal_load(src + (size_t)f * 64);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (acc == 0x9E3779B9u) out[sw] = acc;          // (keeps the loads alive; practically never taken)
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, u16* __restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = f32_to_bf16_bits(src[i]);
}

// Unpack cache positions [pos0, pos0+count) of one layer to fp32 [count][n_kv][D].
// rot_pairs: the K cache holds each head's dims in rotary-pair order (dim i at 2i, dim i + D/2 at 2i + 1).
__global__ void read_kv_kernel(const u16* __restrict__ Kc, const u16* __restrict__ Vc, int n_kv, int D, int max_kb,
                               int pos0, int count, float* __restrict__ k_out, float* __restrict__ v_out,
                               int rot_pairs, const int* __restrict__ pages) {
  const size_t total = (size_t)count * n_kv * D;
  const size_t kv_head_elems = (size_t)max_kb * 32 * D;
  for (size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x; idx < total;
       idx += (size_t)gridDim.x * blockDim.x) {
    const int d = idx % D, h = (idx / D) % n_kv, p = (int)(idx / ((size_t)D * n_kv));
    const int dk = rot_pairs ? (d < D / 2 ? 2 * d : 2 * (d - D / 2) + 1) : d;
    const int key = paged_key(pages, pos0 + p);
    if (k_out) k_out[idx] = bf16_bits_to_f32(Kc[h * kv_head_elems + kp_index(key, dk, D / 32)]);
    if (v_out) v_out[idx] = bf16_bits_to_f32(Vc[h * kv_head_elems + vp_index(key, d, D / 16)]);
  }
}


// ---- per-step decisions -------------------------------------------------------------------------------------

// Seed (Sec. 3.4, causal context decoding): a block whose position 0 is still masked takes the
// carry's argmax there before the forward.
__global__ void seed_kernel(int* tokens, uint8_t* mask, DevState* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->seeded = 0;
    if (mask[0]) {
      tokens[0] = st->carry_cand;
      mask[0] = 0;
      st->seeded = 1;
    }
  }
}

struct FinishArgs {
  int B;
  DevState* st;
  const int* row_cand;      // [B] argmax id of every row of the forward (row i predicts position i+1)
  const float* row_conf;    // [B] its softmax probability
  // denoise
  int* tokens;
  uint8_t* mask;
  float threshold;
  int fixed_k;
  int* n_unmasked;
  float* conf_out;
  // commit / verify
  const int* draft;
  int commit;
  int* ar_pred;
  int* n_accept;
  int skippable;            // bd_decode_block: do nothing once the block is complete, else count the step and set the flag
};

// Confidence-threshold parallel unmask (Sec. 3.4; "Decoding threshold").  Row i-1 predicts block
// position i.  Launched with one wavefront.
__global__ __launch_bounds__(64) void finish_denoise_kernel(FinishArgs a) {
  __shared__ int s_cand[64];
  __shared__ float s_conf[64];
  __shared__ uint8_t s_mask[64];
  if (a.skippable && a.st->skip) return;
  if ((int)threadIdx.x < a.B) {
    s_cand[threadIdx.x] = a.row_cand[threadIdx.x];
    s_conf[threadIdx.x] = a.row_conf[threadIdx.x];
    s_mask[threadIdx.x] = a.mask[threadIdx.x];
    if (a.conf_out) a.conf_out[threadIdx.x] = threadIdx.x == 0 ? a.st->carry_conf : a.row_conf[threadIdx.x - 1];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int revealed = a.st->seeded;
    int remaining = 0;
    for (int i = 1; i < a.B; ++i) remaining += s_mask[i] ? 1 : 0;
    if (remaining > 0) {
      if (a.fixed_k > 0) {
        const int k = min(a.fixed_k, remaining);
        for (int t = 0; t < k; ++t) {                    // k passes of "most confident still masked"
          // (a confidence that is not a number ranks below every number: the first masked position is the fallback)
          int best = -1;
          float bc = -1.f;
          for (int i = 1; i < a.B; ++i)
            if (s_mask[i] && (best < 0 || s_conf[i - 1] > bc)) { bc = s_conf[i - 1] == s_conf[i - 1] ? s_conf[i - 1] : -1.f; best = i; }
          a.tokens[best] = s_cand[best - 1];
          a.mask[best] = 0;
          s_mask[best] = 0;
          ++revealed;
        }
      } else {
        int best = -1, cnt = 0;
        float bc = -1.f;
        for (int i = 1; i < a.B; ++i) {
          if (!s_mask[i]) continue;
          const float c = s_conf[i - 1];
          if (best < 0 || c > bc) { bc = c == c ? c : -1.f; best = i; }
          if (c > a.threshold) {
            a.tokens[i] = s_cand[i - 1];
            a.mask[i] = 0;
            s_mask[i] = 0;
            ++cnt;
          }
        }
        if (cnt == 0) {
          a.tokens[best] = s_cand[best - 1];
          a.mask[best] = 0;
          s_mask[best] = 0;
          cnt = 1;
        }
        revealed += cnt;
      }
    }
    if (a.n_unmasked) *a.n_unmasked = revealed;
    if (a.skippable) {
      int left = 0;
      for (int i = 1; i < a.B; ++i) left += s_mask[i] ? 1 : 0;
      a.st->steps += 1;
      a.st->skip = left == 0;
    }
  }
}

// B == 1 (or nothing to denoise): only report the seed.
__global__ void finish_seed_only_kernel(DevState* st, int* n_unmasked, float* conf_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (n_unmasked) *n_unmasked = st->seeded;
    if (conf_out) conf_out[0] = st->carry_conf;
  }
}

// Causal pass: row j's argmax is the autoregressive prediction a_j (Alg. 1 verify step).  Accept
// length = longest prefix of the draft with draft[0] == carry's argmax and draft[j+1] == a_j.
// With commit, the carry moves to the last row and the context length grows by B.
__global__ __launch_bounds__(64) void finish_causal_kernel(FinishArgs a) {
  __shared__ int s_cand[64];
  __shared__ float s_conf[64];
  if ((int)threadIdx.x < a.B) {
    s_cand[threadIdx.x] = a.row_cand[threadIdx.x];
    s_conf[threadIdx.x] = a.row_conf[threadIdx.x];
    if (a.ar_pred) a.ar_pred[threadIdx.x] = a.row_cand[threadIdx.x];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (a.n_accept && a.commit != 2) {
      int k = 0;
      while (k < a.B && a.draft[k] == (k == 0 ? a.st->carry_cand : s_cand[k - 1])) ++k;
      *a.n_accept = k;
    }
    if (a.commit == 1) {
      a.st->carry_cand = s_cand[a.B - 1];
      a.st->carry_conf = s_conf[a.B - 1];
      a.st->n += a.B;
    } else if (a.commit == 2) {
      // Alg. 1 accept + crop in place: draft[0] is the already accepted first token; k = 1 + the number of leading
      // drafts draft[1..] that equal the predictions a_0..; the emitted tokens are a_0..a_{k-1}; the cache keeps the
      // positions of draft[0..k-1] (the rows beyond were written but the length does not cover them), and a_{k-1}
      // becomes the prediction for the new position n.
      int k = 1;
      while (k < a.B && s_cand[k - 1] == a.draft[k]) ++k;
      *a.n_accept = k;
      a.st->carry_cand = s_cand[k - 1];
      a.st->carry_conf = s_conf[k - 1];
      a.st->n += k;
    }
  }
}

// ---- Alg. 2 (quadratic speculative decoding) ------------------------------------------------------------------
// Rows of the quadratic forward: group i = [draft[i], MASK x B].
__global__ void quad_assemble_kernel(const int* draft, int B, int mask_id, int* ids) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  const int W = B + 1;
  if (r < B * W) ids[r] = (r % W == 0) ? draft[r / W] : mask_id;
}
// Draft 0 of Alg. 2's first block is the carry's prediction (the hidden state of the last context row).
__global__ void quad_first_kernel(int* draft, const DevState* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) draft[0] = st->carry_cand;
}
// Accept: P[i][j] = argmax of group i, entry j (predicts position n+i+j+1).  k = 1 + leading drafts d_1.. that equal
// P[0][0], P[1][0], ..; the next draft block is P[k-1][0..B-1]; the prediction of group k-1's first row becomes the
// carry and the context grows by k (the keys and values of the accepted first rows are moved into place afterwards).
__global__ __launch_bounds__(64) void finish_quad_kernel(FinishArgs a, int* next_draft) {
  const int W = a.B + 1;
  if (threadIdx.x == 0) {
    int k = 1;
    while (k < a.B && a.row_cand[(k - 1) * W] == a.draft[k]) ++k;
    *a.n_accept = k;
    for (int j = 0; j < a.B; ++j) next_draft[j] = a.row_cand[(k - 1) * W + j];
    a.st->carry_cand = a.row_cand[(k - 1) * W];
    a.st->carry_conf = a.row_conf[(k - 1) * W];
    a.st->n += k;
  }
}
// The quadratic forward left the keys and values of row r at cache position n0 + r; the accepted tokens are the
// first rows of groups 0..k-1, i.e. rows i*(B+1), and belong at positions n0 + i.  (Destinations 1..k-1 < B+1 never
// coincide with a source, so all moves are independent.)  One workgroup per (layer, kv head).
__global__ void quad_compact_kv_kernel(u16* Kc, u16* Vc, size_t kv_layer_elems, int n_kv, int D, int max_kb, const DevState* st,
                                       const int* k_ptr, int B, const int* pages) {
  const int layer = blockIdx.x / n_kv, h = blockIdx.x % n_kv;
  const int k = *k_ptr;
  const int n0 = st->n - k;                       // the accept kernel has already advanced the length
  u16* kc = Kc + (size_t)layer * kv_layer_elems + (size_t)h * max_kb * 32 * D;
  u16* vc = Vc + (size_t)layer * kv_layer_elems + (size_t)h * max_kb * 32 * D;
  for (int t = threadIdx.x; t < (k - 1) * D; t += blockDim.x) {
    const int i = 1 + t / D, d = t % D;
    const int dst = paged_key(pages, n0 + i), src = paged_key(pages, n0 + i * (B + 1));
    kc[kp_index(dst, d, D / 32)] = kc[kp_index(src, d, D / 32)];
    vc[vp_index(dst, d, D / 16)] = vc[vp_index(src, d, D / 16)];
  }
}

// Entries [kb0, kb0 + count) of the page table (count <= 16: the values travel as kernel arguments, so the update is
// an ordinary launch in stream order, with no host buffer that would have to stay alive).
struct PageVals { int v[16]; };
__global__ void iota_kernel(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}
__global__ void set_pages_kernel(int* pages, int kb0, int count, PageVals vals) {
  if ((int)threadIdx.x < count) pages[kb0 + threadIdx.x] = vals.v[threadIdx.x];
}

// All positions of a block masked (the state before the draft pass of Alg. 1).
__global__ void fill_masked_kernel(int* tokens, uint8_t* mask, int B, int mask_id, DevState* st, int first_revealed = 0) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) { tokens[i] = mask_id; mask[i] = (i == 0 && first_revealed) ? 0 : 1; }
  if (i == 0) { st->skip = 0; st->steps = 0; }
}
__global__ void raise_error_kernel(DevState* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) st->error = 1;
}
__global__ void read_steps_kernel(const DevState* st, int* out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *out = st->steps;
}

// Commit without an LM-head pass (prompt chunks before the last one).
__global__ void advance_kernel(DevState* st, int B) {
  if (threadIdx.x == 0 && blockIdx.x == 0) st->n += B;
}

__global__ void set_state_kernel(DevState* st, int n, int clear_carry) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->n = n;
    st->seeded = 0;
    if (clear_carry) { st->carry_cand = -1; st->carry_conf = 0.f; }
  }
}

}  // namespace bd
