// Host-only exercise of libmona's boundary for a sanitizer build (AddressSanitizer + UndefinedBehaviorSanitizer
// on the host code; no GPU needed): every entry point that can run without a device -- the arena layout over
// random lists of matrices, and the argument checks of the others -- is called many times.
// Build and run: tests/host/run_sanitizers.sh
#include "../../include/mona.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

int main() {
  std::mt19937 rng(12345);
  auto dim = [&](int hi) { return 1 + (int)(rng() % hi); };
  for (int round = 0; round < 300; ++round) {
    const int count = 1 + (int)(rng() % 40);
    std::vector<mona_matrix> mats(count);
    for (auto& q : mats) {
      std::memset(&q, 0, sizeof q);
      const int kind = rng() % 4;
      q.m = kind == 0 ? dim(64) : kind == 1 ? dim(700) : 128 * dim(40);
      q.n = kind == 0 ? dim(64) : kind == 1 ? dim(700) : 128 * dim(40);
      q.w_dtype = rng() % 2;
      q.g_dtype = rng() % 2;
    }
    for (int variant = 0; variant < 12; ++variant) {
      mona_options o;
      std::memset(&o, 0, sizeof o);
      o.ns_precision = variant & 1;
      o.state_dtype = (variant >> 1) & 1;
      o.accel_form = variant % 3;
      o.ns_schedule = variant % 3;
      o.overlap = (variant >> 2) & 1;
      o.max_streams = variant % 5;
      size_t bytes = 0;
      EXPECT(mona_state_size(mats.data(), count, &o, &bytes) == MONA_OK);
      size_t least = 0;
      for (auto& q : mats) least += (size_t)q.m * q.n * 4;      // at least M itself
      EXPECT(bytes >= least);
    }
  }
  // argument checks
  size_t bytes = 0;
  mona_matrix one;
  std::memset(&one, 0, sizeof one);
  one.m = 8; one.n = 8;
  EXPECT(mona_state_size(nullptr, 1, nullptr, &bytes) == MONA_EINVAL);
  EXPECT(mona_state_size(&one, 0, nullptr, &bytes) == MONA_EINVAL);
  EXPECT(mona_state_size(&one, 1, nullptr, nullptr) == MONA_EINVAL);
  one.m = 0;
  EXPECT(mona_state_size(&one, 1, nullptr, &bytes) == MONA_EINVAL);
  one.m = 1 << 30; one.n = 4;
  EXPECT(mona_state_size(&one, 1, nullptr, &bytes) == MONA_EINVAL);
  one.m = 8; one.n = 8; one.w_dtype = 7;
  EXPECT(mona_state_size(&one, 1, nullptr, &bytes) == MONA_EINVAL);
  one.w_dtype = 0;
  mona_options bad;
  std::memset(&bad, 0, sizeof bad);
  bad.ns_schedule = 9;
  EXPECT(mona_state_size(&one, 1, &bad, &bytes) == MONA_EINVAL);
  EXPECT(std::strlen(mona_last_error()) > 0);
  mona_state* st = nullptr;
  EXPECT(mona_init_state(&one, 1, nullptr, nullptr, 0, nullptr, &st) == MONA_EINVAL && st == nullptr);
  mona_hparams hp;
  std::memset(&hp, 0, sizeof hp);
  EXPECT(mona_step(nullptr, &one, 1, &hp, nullptr) == MONA_EINVAL);
  EXPECT(mona_step_streaming(nullptr, &one, nullptr, 1, &hp, nullptr) == MONA_EINVAL);
  EXPECT(mona_step_noalloc(&one, nullptr, nullptr, nullptr, nullptr, &hp, 0, nullptr) == MONA_EINVAL);
  EXPECT(mona_free_state(nullptr) == MONA_OK);
  mona_view v;
  EXPECT(mona_state_view(nullptr, 0, 0, &v) == MONA_EINVAL);
  EXPECT(mona_set_profiling(nullptr, 1) == MONA_EINVAL);
  mona_vector vec;
  std::memset(&vec, 0, sizeof vec);
  vec.n = 1000;
  EXPECT(mona_adamw_state_size(&vec, 1, &bytes) == MONA_OK && bytes >= 8000);
  vec.n = 0;
  EXPECT(mona_adamw_state_size(&vec, 1, &bytes) == MONA_EINVAL);
  std::printf("%s (%d failures)\n", failures ? "FAILED" : "ok", failures);
  return failures ? 1 : 0;
}
