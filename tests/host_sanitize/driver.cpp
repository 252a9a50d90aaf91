// Host-side sanitizer driver: the library's plan and argument-check code (everything that runs
// before the first launch) compiled for the host with AddressSanitizer and
// UndefinedBehaviorSanitizer, driven through the C ABI.  No GPU call is reached: every case below
// either is a pure host query or fails a host-side check.  Any sanitizer report aborts the program.
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "oapl.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::printf("FAILED line %d: %s\n", __LINE__, #cond);                \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

int main() {
  void* one = (void*)(uintptr_t)256;   // aligned, never dereferenced: the checks fail first
  long n_plans = 0;

  // workspace queries over the whole legal range of sizes, and just outside it
  const int64_t Ts[] = {0, 1, 63, 64, 383, 384, 385, 12288, 12289, 61440, 140897, 896842, 1 << 20,
                        (int64_t)65535 * 64, (int64_t)65535 * 64 + 1, (int64_t)65535 * 256, (int64_t)65535 * 256 + 1};
  const int32_t ds[] = {8, 64, 72, 320, 2048, 4096, 5120, 1 << 21, (1 << 21) + 8};
  const int32_t Vs[] = {1, 8, 264, 1544, 151936, 1 << 21, (1 << 21) + 1};
  for (int64_t T : Ts)
    for (int32_t d : ds)
      for (int32_t V : Vs)
        for (int dtype = 0; dtype < 2; ++dtype)
          for (int bwd = 0; bwd < 2; ++bwd) {
            const size_t a = oapl_workspace_bytes(T, d, V, 64, 8, dtype, bwd);
            const bool legal = d <= (1 << 21) && V <= (1 << 21) &&
                               (dtype == OAPL_BF16 ? T <= (int64_t)65535 * 256 : T <= (int64_t)65535 * 64);
            CHECK((a > 0) == legal);
            for (int64_t cap : {(int64_t)0, (int64_t)1, (int64_t)384, (int64_t)5000, (int64_t)12288, (int64_t)1 << 40})
              for (int64_t len : {(int64_t)0, (int64_t)4096, (int64_t)32768, (int64_t)1 << 40}) {
                int64_t rows = -1;
                int32_t bufs = -1;
                const size_t b = oapl_workspace_bytes_for(T, d, V, 64, 8, dtype, bwd, cap, len, &rows, &bufs);
                CHECK((b > 0) == legal);
                if (legal) CHECK(rows >= 1 && bufs >= 1 && b % 256 == 0);
                ++n_plans;
              }
          }
  CHECK(oapl_workspace_bytes(256, 64, 1024, 1 << 20, 1 << 13, 0, 0) == 0);   // n_seq * n_groups above 2^32
  CHECK(oapl_workspace_bytes_for(256, 64, 1024, 8, 2, 0, 1, 0, 0, nullptr, nullptr) > 0);

  // every host-side error of the loss entry points; nothing is launched
  auto loss = [&](int64_t T, int32_t d, int32_t V, int32_t dtype, float beta, void* dH, float* dW, void* ws,
                  size_t ws_bytes, uint32_t flags) {
    float* f = (float*)one;
    return oapl_loss_fwd_bwd_two_beta(one, one, (const int32_t*)one, f, (const int64_t*)one, f, (const int32_t*)one, T,
                                      d, V, 64, 8, dtype, beta, beta, 1.0f, flags, f, nullptr, nullptr, nullptr, dH, dW,
                                      ws, ws_bytes, nullptr);
  };
  float* fone = (float*)one;
  CHECK(loss(1000, 64, 1024, 7, 1.f, one, fone, one, 1 << 20, 0) == OAPL_ERR_DTYPE);
  CHECK(loss(1000, 0, 1024, 0, 1.f, one, fone, one, 1 << 20, 0) == OAPL_ERR_SHAPE);
  CHECK(loss(1000, 64, 1024, 0, 1.f, one, nullptr, one, 1 << 20, 0) == OAPL_ERR_NULL);
  CHECK(loss(1000, 64, 1024, 0, 0.f, one, fone, one, 1 << 20, 0) == OAPL_ERR_BETA);
  CHECK(loss(1000, 64, 1024, 0, 1.f, one, fone, one, 1 << 20, 8) == OAPL_ERR_SHAPE);
  CHECK(loss(1000, 64, 1024, 0, 1.f, one, fone, nullptr, 1 << 20, 0) == OAPL_ERR_WORKSPACE);
  CHECK(loss(1000, 64, 1024, 0, 1.f, one, fone, (void*)(uintptr_t)260, 1 << 30, 0) == OAPL_ERR_WORKSPACE);
  // the budget search: a workspace a little short of the smallest plan makes it try every panel size and fail
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int64_t T : {(int64_t)1000, (int64_t)140897, (int64_t)1 << 20}) {
      if (dtype == OAPL_F32 && T > (int64_t)65535 * 64) continue;
      const int32_t d = dtype ? 4096 : 64, V = dtype ? 151936 : 1024;
      const size_t least = oapl_workspace_bytes_for(T, d, V, 64, 8, dtype, 1, 1, 0, nullptr, nullptr);
      CHECK(least > 256);
      CHECK(loss(T, d, V, dtype, 1.f, one, fone, one, least - 256, 0) == OAPL_ERR_WORKSPACE);
      CHECK(loss(T, d, V, dtype, 1.f, one, fone, one, 0, 0) == OAPL_ERR_WORKSPACE);
    }
  // forward-only entry points
  CHECK(oapl_logprob_fwd(one, one, (const int32_t*)one, 4, 8, 8, 0, fone, nullptr, nullptr, one, 16, nullptr) ==
        OAPL_ERR_WORKSPACE);
  CHECK(oapl_sample_tokens(one, one, 4, 8, 8, 0, 0.0f, 1, (int32_t*)one, nullptr, one, 1 << 20, nullptr) == OAPL_ERR_BETA);
  CHECK(oapl_grpo_loss_fwd_bwd(one, one, (const int32_t*)one, fone, fone, (const int64_t*)one, fone,
                               (const int32_t*)one, 4, 8, 8, 2, 1, 0, 1.5f, 1e-6f, 1.f, 0, fone, nullptr, nullptr, one,
                               fone, one, 1 << 24, nullptr) == OAPL_ERR_BETA);
  // the entry point that allocates nothing: sizes beyond its scratch are refused on the host
  CHECK(oapl_loss_fwd_bwd_noalloc(one, one, (const int32_t*)one, fone, (const int64_t*)one, fone, (const int32_t*)one,
                                  1000, 4096, 151936, 64, 8, 1, 1.f, 1.f, fone, nullptr, nullptr, nullptr, one, fone,
                                  nullptr) == OAPL_ERR_SCRATCH_LIMIT);
  for (int s = -1; s < 13; ++s) CHECK(oapl_status_string(s) != nullptr);
  std::printf("host sanitizer driver: %ld plans, all checks passed\n", n_plans);
  return 0;
}
