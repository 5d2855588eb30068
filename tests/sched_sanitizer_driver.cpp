// Exercises every hat_sched_* entry point, valid and invalid arguments, under
// AddressSanitizer + UndefinedBehaviorSanitizer (host code only).  Exit status 0 = the
// calls returned what the header promises and the sanitizers saw nothing.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <vector>

#include "hat_sched.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main() {
  hat_sched_t* s = nullptr;
  const int32_t bad1[] = {4, 4}, bad2[] = {8, 4};
  CHECK(hat_sched_create(nullptr, 2, 0.8, &s) == -1 && s == nullptr);
  CHECK(hat_sched_create(bad1, 2, 0.8, &s) == -1 && hat_sched_create(bad2, 2, 0.8, &s) == -1);
  CHECK(hat_sched_create(bad1, 0, 0.8, &s) == -1 && hat_sched_create(bad1, 1, 1.5, &s) == -1);
  CHECK(hat_sched_observe(nullptr, 1, 1) == -1 && hat_sched_chunk_size(nullptr, 1, 1, 1, 1, 2) == -1);
  hat_sched_destroy(nullptr);

  uint64_t state = 12345;
  auto rnd = [&]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (double)(state >> 11) / 9007199254740992.0; };
  for (int round = 0; round < 50; ++round) {
    const int nk = 1 + (int)(rnd() * 12);
    std::vector<int32_t> knots(nk);
    int32_t x = 1 + (int)(rnd() * 64);
    for (int i = 0; i < nk; ++i) { knots[i] = x; x += 1 + (int)(rnd() * 1500); }
    CHECK(hat_sched_create(knots.data(), nk, rnd(), &s) == 0 && s != nullptr);
    CHECK(hat_sched_mu(s) == 0.0 && hat_sched_predict(s, 100.0) == 0.0);
    CHECK(hat_sched_observe(s, -1.0, 1.0) == -1 && hat_sched_observe(s, 1.0, std::nan("")) == -1);
    CHECK(hat_sched_observe(s, std::numeric_limits<double>::infinity(), 1.0) == -1);
    for (int t = 0; t < 200; ++t) {
      const double mu = rnd() * 1.5 * knots.back(), eta = 0.5 + 0.004 * mu * (0.5 + rnd());
      CHECK(hat_sched_observe(s, mu, eta) == 0);
      CHECK(std::isfinite(hat_sched_predict(s, rnd() * 3.0 * knots.back())));
      const int32_t lo = 1 + (int)(rnd() * 32), hi = lo + (int)(rnd() * 4096);
      const int32_t c = hat_sched_chunk_size(s, 8192.0, 1e3 + rnd() * 1e7, 1 + (int)(rnd() * 8), lo, hi);
      CHECK(c >= lo && c <= hi);
      CHECK(hat_sched_parallel_draft_steps(s, 1 + rnd() * 7, 8192.0, 1e3 + rnd() * 1e7, 1e3 + rnd() * 1e7, 0.1 + rnd() * 50) >= 0);
    }
    CHECK(hat_sched_chunk_size(s, 0.0, 1.0, 1, 1, 2) == -1 && hat_sched_chunk_size(s, 1.0, 1.0, 0, 1, 2) == -1);
    CHECK(hat_sched_chunk_size(s, 1.0, 1.0, 1, 0, 2) == -1 && hat_sched_chunk_size(s, 1.0, 1.0, 1, 3, 2) == -1);
    CHECK(hat_sched_parallel_draft_steps(s, 1, 1, 1, 1, 0.0) == -1);
    hat_sched_destroy(s);
    s = nullptr;
  }
  std::puts("sched sanitizer driver: ok");
  return 0;
}
