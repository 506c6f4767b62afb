// Host-side paths of the C-ABI under AddressSanitizer and UndefinedBehaviorSanitizer: argument validation, the
// workspace layout, context creation and destruction, calls out of order, the table look-ups.  Nothing here reaches
// a kernel launch: every call either fails its checks on the host or only builds host state, so the program runs
// with or without a GPU.  Built and run by tests/test_host_sanitizers.py; exit status 0 = every call answered as
// expected and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "adore.h"

static int failures = 0;
#define EXPECT(cond)                                                          \
  do {                                                                        \
    if (!(cond)) {                                                            \
      std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond);                 \
      ++failures;                                                             \
    }                                                                         \
  } while (0)

static adore_config tiny() {
  adore_config c;
  std::memset(&c, 0, sizeof c);
  c.layers = 1; c.batch = 1; c.heads = 4; c.head_dim = 64; c.hidden = 256; c.cache_slots = 64; c.rebuild_budget = 8;
  c.max_positions = 384; c.ctrl_hidden = 64; c.dtype = ADORE_F32; c.pos_scale = 1.0f / 384; c.score_mode = ADORE_SCORE_STATIC;
  c.rope_base = 0.f;
  return c;
}

int main() {
  EXPECT(adore_abi_version() == ADORE_ABI_VERSION);
  // a pointer that is never dereferenced on the host: the library only stores it
  std::vector<unsigned char> backing(4096);
  void *fake = reinterpret_cast<void *>((reinterpret_cast<uintptr_t>(backing.data()) + 255) / 256 * 256);
  float *ffake = static_cast<float *>(fake);
  adore_weights wt;
  {
    void **p = reinterpret_cast<void **>(&wt);
    for (size_t i = 0; i < sizeof wt / sizeof(void *); ++i) p[i] = fake;
  }
  adore_config c = tiny();
  const size_t n = adore_workspace_bytes(&c);
  EXPECT(n > 0 && n % 256 == 0);
  EXPECT(adore_workspace_bytes(nullptr) == 0);
  adore_ctx *h = nullptr;
  EXPECT(adore_create(nullptr, &wt, fake, n, nullptr, &h) == ADORE_E_INVALID);
  EXPECT(adore_create(&c, nullptr, fake, n, nullptr, &h) == ADORE_E_INVALID);
  EXPECT(adore_create(&c, &wt, nullptr, n, nullptr, &h) == ADORE_E_INVALID);
  EXPECT(adore_create(&c, &wt, fake, n - 1, nullptr, &h) == ADORE_E_WORKSPACE);
  EXPECT(adore_create(&c, &wt, static_cast<char *>(fake) + 16, n, nullptr, &h) == ADORE_E_WORKSPACE);
  // every integer field at values around its limits: the layout arithmetic must not overflow or divide by zero
  const int32_t probes[] = {-2147483647 - 1, -1, 0, 1, 2, 7, 63, 64, 65, 1023, 1024, 1025, 65535, 65536, 2147483647};
  for (size_t field = 0; field < 10; ++field) {
    for (int32_t v : probes) {
      adore_config x = tiny();
      reinterpret_cast<int32_t *>(&x)[field] = v;
      const size_t bytes = adore_workspace_bytes(&x);
      adore_ctx *hx = nullptr;
      const int rc = adore_create(&x, &wt, fake, bytes ? bytes : 256, nullptr, &hx);
      EXPECT(rc == ADORE_OK || rc == ADORE_E_INVALID || rc == ADORE_E_UNSUPPORTED || rc == ADORE_E_WORKSPACE);
      if (rc == ADORE_OK) {
        EXPECT(bytes > 0);
        EXPECT(adore_destroy(hx) == ADORE_OK);
      }
    }
  }
  for (int mode = -1; mode <= 3; ++mode) {
    for (float base : {0.f, 10000.f, -1.f}) {
      adore_config x = tiny();
      x.score_mode = mode;
      x.rope_base = base;
      const size_t bytes = adore_workspace_bytes(&x);
      adore_ctx *hx = nullptr;
      const int rc = adore_create(&x, &wt, fake, bytes ? bytes : 256, nullptr, &hx);
      if (rc == ADORE_OK) EXPECT(adore_destroy(hx) == ADORE_OK);
    }
  }
  // one context, calls out of order and with null arguments
  EXPECT(adore_create(&c, &wt, fake, n, nullptr, &h) == ADORE_OK);
  EXPECT(adore_attend(h, 0, fake, fake, fake, ffake) == ADORE_E_STATE);
  { const int rc = adore_attend(h, 5, fake, fake, fake, ffake); EXPECT(rc == ADORE_E_INVALID || rc == ADORE_E_STATE); }
  EXPECT(adore_schedule(h, fake, nullptr, nullptr, nullptr, nullptr) == ADORE_E_STATE);
  EXPECT(adore_rebuild(h, 0, fake) == ADORE_E_STATE);
  EXPECT(adore_decode_step(h, fake, fake, fake, fake, fake, nullptr, ffake, nullptr) == ADORE_E_STATE);
  EXPECT(adore_init_cache(h, fake, fake, fake, fake, nullptr, 0) == ADORE_E_INVALID);
  EXPECT(adore_init_cache(h, fake, fake, fake, fake, nullptr, c.max_positions) == ADORE_E_INVALID);
  EXPECT(adore_init_cache(h, nullptr, fake, fake, fake, nullptr, 4) == ADORE_E_INVALID);
  EXPECT(adore_set_state(h, nullptr, nullptr, nullptr, nullptr, nullptr, 5) == ADORE_E_INVALID);
  EXPECT(adore_set_state(h, static_cast<const int32_t *>(fake), nullptr, nullptr, nullptr, nullptr, 0) == ADORE_E_INVALID);
  EXPECT(adore_set_input_order(nullptr, 0) == ADORE_E_INVALID);
  EXPECT(adore_set_input_order(h, 0) == ADORE_OK);
  EXPECT(adore_set_input_order(h, 1) == ADORE_OK);
  EXPECT(adore_set_timing(h, 1) == ADORE_OK);
  EXPECT(adore_set_timing(h, 0) == ADORE_OK);
  adore_forward_weights fw = {fake, fake};
  EXPECT(adore_forward_step(h, nullptr, fake, nullptr, fake, nullptr, nullptr, nullptr, nullptr) == ADORE_E_INVALID);
  EXPECT(adore_forward_step(h, &fw, fake, nullptr, fake, nullptr, nullptr, nullptr, nullptr) == ADORE_E_STATE);
  int32_t damaged = 7;
  EXPECT(adore_check_guards(h, &damaged) == ADORE_OK && damaged == -1);
  EXPECT(adore_check_guards(h, nullptr) == ADORE_E_INVALID);
  int32_t step = 0;
  EXPECT(adore_get_state(h, nullptr, nullptr, nullptr, nullptr, nullptr, &step) == ADORE_E_STATE);
  EXPECT(adore_destroy(h) == ADORE_OK);
  EXPECT(adore_destroy(nullptr) == ADORE_E_INVALID);
  // the debug layout
  setenv("ADORE_GUARD_WORDS", "1", 1);
  const size_t guarded = adore_workspace_bytes(&c);
  EXPECT(guarded > n && (guarded - n) % 256 == 0);
  EXPECT(adore_create(&c, &wt, fake, n, nullptr, &h) == ADORE_E_WORKSPACE);
  EXPECT(adore_create(&c, &wt, fake, guarded, nullptr, &h) == ADORE_OK);
  EXPECT(adore_destroy(h) == ADORE_OK);
  unsetenv("ADORE_GUARD_WORDS");
  // tables
  for (int code : {0, -1, -2, -3, -4, -5, -99, 12345}) EXPECT(adore_strerror(code) != nullptr && std::strlen(adore_strerror(code)) > 0);
  for (int i = -3; i < ADORE_N_KERNELS + 3; ++i) EXPECT(adore_kernel_name(i) != nullptr);
  // top-K attention: sizes and argument checks
  EXPECT(adore_topk_attention_workspace_bytes(0, 8, 64) == 0);
  EXPECT(adore_topk_attention_workspace_bytes(3, 100, 128) == size_t(3) * 128 * 128 * 2);
  for (int32_t rows : {1, 7, 512, 65535, 65536, 2147483647})
    for (int32_t seq : {1, 31, 32, 33, 2048, 2049, 32768, 32769, 2147483647})
      (void)adore_topk_attention_workspace_bytes(rows, seq, 128);
  const size_t tn = adore_topk_attention_workspace_bytes(2, 64, 64);
  EXPECT(adore_topk_attention(nullptr, fake, fake, fake, fake, tn, 2, 64, 64, 4, nullptr) == ADORE_E_INVALID);
  EXPECT(adore_topk_attention(fake, fake, fake, fake, fake, tn, 2, 64, 64, 0, nullptr) == ADORE_E_INVALID);
  EXPECT(adore_topk_attention(fake, fake, fake, fake, fake, tn, 2, 64, 96, 4, nullptr) == ADORE_E_UNSUPPORTED);
  EXPECT(adore_topk_attention(fake, fake, fake, fake, fake, tn - 1, 2, 64, 64, 4, nullptr) == ADORE_E_WORKSPACE);
  EXPECT(adore_topk_attention_static(fake, fake, fake, nullptr, 2, 64, 64, 4, nullptr) == ADORE_E_INVALID);
  EXPECT(adore_topk_attention_static(fake, fake, fake, fake, 2, 4096, 64, 4, nullptr) == ADORE_E_WORKSPACE);
  EXPECT(adore_topk_attention_static(fake, fake, fake, fake, 60000, 2048, 128, 4, nullptr) == ADORE_E_WORKSPACE);
  if (failures) {
    std::fprintf(stderr, "%d unexpected answers\n", failures);
    return 1;
  }
  std::puts("host checks ok");
  return 0;
}
