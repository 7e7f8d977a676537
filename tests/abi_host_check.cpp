// Host-side checks of the C ABI for a build of the library whose host code carries AddressSanitizer and
// UndefinedBehaviorSanitizer (tests/test_abi_sanitized.py builds and runs it): every entry point is called the way
// tests/test_abi_cpu.py calls it -- bad shapes, null pointers, error strings, creation with and without a device --
// so that the argument checks, the error paths and the set-up/tear-down code run under the sanitizers.
#include <cstdio>
#include <cstring>

#include "../include/bd.h"
#include "../include/bd_kernels.h"

static int failures = 0;
#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static bd_config tiny() {
  bd_config c;
  std::memset(&c, 0, sizeof c);
  c.n_layers = 2; c.hidden = 256; c.n_q_heads = 4; c.n_kv_heads = 2; c.head_dim = 64; c.ffn = 688; c.vocab = 1024;
  c.rope_theta = 1.0e6f; c.rms_eps = 1.0e-6f; c.max_seq = 256; c.max_block = 32; c.mask_token_id = -1;
  c.weight_dtype = BD_BF16; c.flags = 0;
  return c;
}

int main() {
  CHECK(std::strcmp(bd_strerror(0), "ok") == 0);
  for (int code = -5; code < 0; ++code) CHECK(std::strcmp(bd_strerror(code), "ok") != 0 && std::strcmp(bd_strerror(code), "unknown error") != 0);
  CHECK(std::strcmp(bd_strerror(-99), "unknown error") == 0);

  bd_ctx* h = nullptr;
  bd_config c = tiny();
  CHECK(bd_create(nullptr, nullptr, &h) == BD_E_ARG);
  CHECK(bd_create(&c, nullptr, nullptr) == BD_E_ARG);
  {
    bd_config b = tiny(); b.head_dim = 48; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG && h == nullptr);
    b = tiny(); b.n_q_heads = 3; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.hidden = 250; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.max_block = 0; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.max_block = 65; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.max_seq = 8; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.vocab = 1000; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.ffn = 100; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.mask_token_id = 1024; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.n_layers = 0; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.rope_theta = 0.f; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.flags = 1 << 20; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
    b = tiny(); b.weight_dtype = BD_F32; CHECK(bd_create(&b, nullptr, &h) == BD_E_DTYPE);
    b = tiny(); b.weight_dtype = BD_FP8_E4M3; b.max_seq = 128; b.max_block = 64; CHECK(bd_create(&b, nullptr, &h) == BD_E_ARG);
  }
  CHECK(bd_prefill(nullptr, nullptr, 0, nullptr, 0) == BD_E_ARG);
  CHECK(bd_denoise_step(nullptr, nullptr, nullptr, 4, 0.9f, 0, nullptr, nullptr) == BD_E_ARG);
  CHECK(bd_commit_block(nullptr, nullptr, 4) == BD_E_ARG);
  CHECK(bd_verify_block(nullptr, nullptr, 4, 1, nullptr, nullptr) == BD_E_ARG);
  CHECK(bd_decode_block(nullptr, 4, 0.9f, 0, nullptr, nullptr) == BD_E_ARG);
  int32_t k = 0;
  CHECK(bd_speculative_step(nullptr, 4, nullptr, &k) == BD_E_ARG);
  CHECK(bd_quad_draft(nullptr, 4, nullptr) == BD_E_ARG);
  CHECK(bd_quad_step(nullptr, 4, nullptr, nullptr, &k) == BD_E_ARG);
  CHECK(bd_crop(nullptr, 0) == BD_E_ARG);
  CHECK(bd_cache_len(nullptr) == BD_E_ARG);
  CHECK(bd_status(nullptr) == BD_E_ARG);
  CHECK(bd_load_weight(nullptr, "embed", nullptr, 0, 0, nullptr) == BD_E_ARG);
  CHECK(bd_k_attention(nullptr, nullptr, nullptr, nullptr, 0, 4, 4, 2, 64, 0, nullptr, 1, nullptr) == BD_E_ARG);
  CHECK(bd_k_attention_static(nullptr, nullptr, nullptr, nullptr, 0, 4, 4, 2, 64, 0, nullptr) == BD_E_ARG);
  double ms = 0;
  CHECK(bd_k_stream_floor(nullptr, 1, &ms, nullptr) == BD_E_ARG);
  CHECK(bd_k_profile(nullptr, 1) == BD_E_ARG);
  CHECK(bd_k_trace(nullptr, 1) == BD_E_ARG);
  CHECK(bd_k_class_count() > 0 && bd_k_class_name(0) != nullptr && bd_k_class_name(99) == nullptr);
  CHECK(bd_kv_page_order(nullptr, nullptr, 0) == BD_E_ARG);
  CHECK(bd_kv_pages(nullptr, nullptr, 0) == BD_E_ARG);
  bd_destroy(nullptr);

  // creation proper: with a device the whole set-up and tear-down run (allocations, plan, packing tables); without one
  // the call has to fail cleanly and leave a message
  const int rc = bd_create(&c, nullptr, &h);
  if (rc == BD_OK) {
    CHECK(h != nullptr);
    CHECK(bd_cache_len(h) == 0);
    CHECK(bd_status(h) == BD_OK);
    CHECK(bd_crop(h, 0) == BD_E_STATE);                       // nothing prefilled yet
    {
      int32_t order[8] = {7, 6, 5, 4, 3, 2, 1, 0}, dup[8] = {0, 0, 1, 2, 3, 4, 5, 6}, out[8];
      CHECK(bd_kv_page_order(h, order, 8) == BD_OK);          // max_seq 256 = 8 pages
      CHECK(bd_kv_page_order(h, order, 7) == BD_E_ARG);
      CHECK(bd_kv_page_order(h, dup, 8) == BD_E_ARG);
      CHECK(bd_kv_pages(h, out, 8) == 0);                     // nothing in use before the first prefill
    }
    CHECK(bd_prefill(h, nullptr, 0, nullptr, 0) == BD_E_ARG);
    float one[256];
    for (float& v : one) v = 1.f;
    CHECK(bd_load_weight(h, "no.such.tensor", one, sizeof one, BD_F32, nullptr) == BD_E_ARG);
    CHECK(bd_load_weight(h, "l0.attn_norm", one, sizeof one, BD_F32, nullptr) == BD_OK);
    CHECK(bd_load_weight(h, "l0.attn_norm", one, sizeof one - 4, BD_F32, nullptr) == BD_E_ARG);
    bd_destroy(h);
    std::printf("device present: create / load / destroy ran\n");
  } else {
    CHECK(rc == BD_E_HIP);
    CHECK(bd_last_error() != nullptr && std::strlen(bd_last_error()) > 0);
    std::printf("no device: create failed cleanly (%s)\n", bd_last_error());
  }
  if (failures == 0) std::printf("ALL OK\n");
  return failures == 0 ? 0 : 1;
}
