// Exercises the host-only entry points of libbaklava under AddressSanitizer / UBSan.
// Built and run by tests/test_host_sanitizers.py; exits 0 when every call behaved.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>

#include "baklava.h"

static int fails = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("FAILED: %s (line %d)\n", #cond, __LINE__); ++fails; } } while (0)

int main() {
  std::mt19937_64 rng(12345);
  std::lognormal_distribution<double> ln(0.0, 1.5);
  for (int rep = 0; rep < 300; ++rep) {
    const int m = 1 + (int)(rng() % 300);
    std::vector<double> imp(m);
    for (double& v : imp) v = ln(rng);
    const int lo = (int)(rng() % 200), hi = lo + (int)(rng() % 140000);
    const int64_t B = (int64_t)m * lo + (int64_t)(rng() % ((uint64_t)m * (hi - lo) + 1));
    std::vector<int32_t> b(m, -1);
    const int st = baklava_alloc_proportional(imp.data(), m, B, lo, hi, b.data());
    CHECK(st == BAKLAVA_OK);
    int64_t sum = 0;
    for (int i = 0; i < m; ++i) { sum += b[i]; CHECK(b[i] >= lo && b[i] <= hi); }
    CHECK(sum == B);
    for (int i = 0; i < m; ++i)
      for (int j = 0; j < m; j += 17)
        if (imp[i] < imp[j]) CHECK(b[i] <= b[j]);

    std::vector<int32_t> size(m), out(m);
    for (int32_t& s : size) s = (int32_t)(rng() % 50000);
    std::vector<double> u(m);
    for (double& v : u) v = (double)(rng() % 1000) / 1000.0;
    CHECK(baklava_alloc_threshold(u.data(), m, size.data(), 0.5, 0.3, out.data()) == BAKLAVA_OK);
    int64_t s0 = 0, s1 = 0;
    for (int i = 0; i < m; ++i) { s0 += size[i]; s1 += out[i]; }
    CHECK(s0 == s1);
    CHECK(baklava_alloc_threshold(u.data(), m, size.data(), 0.5, 0.3, size.data()) == BAKLAVA_OK);  // aliasing allowed
  }
  // extreme weights: tiny importances next to a huge one, and a single head
  {
    std::vector<double> imp = {1e-300, 1.0, 1e300, 5e-324};
    std::vector<int32_t> b(4);
    CHECK(baklava_alloc_proportional(imp.data(), 4, 1000, 1, 2000000000, b.data()) == BAKLAVA_OK);
    CHECK((int64_t)b[0] + b[1] + b[2] + b[3] == 1000);
    double one = 3.0;
    int32_t bo = 0;
    CHECK(baklava_alloc_proportional(&one, 1, 77, 0, 100, &bo) == BAKLAVA_OK && bo == 77);
    CHECK(baklava_alloc_proportional(&one, 1, 2147483647LL, 0, 2147483647, &bo) == BAKLAVA_OK && bo == 2147483647);
  }
  // error paths
  {
    double imp[2] = {1.0, NAN};
    int32_t b[2];
    CHECK(baklava_alloc_proportional(imp, 2, 10, 0, 10, b) == BAKLAVA_EINVAL);
    CHECK(baklava_alloc_proportional(nullptr, 2, 10, 0, 10, b) == BAKLAVA_EINVAL);
    double ok[2] = {1.0, 2.0};
    CHECK(baklava_alloc_proportional(ok, 2, 100, 0, 10, b) == BAKLAVA_EINFEASIBLE);
    CHECK(baklava_alloc_proportional(ok, 0, 0, 0, 10, b) == BAKLAVA_EINVAL);
  }
  // layout
  {
    std::vector<int32_t> bud = {5, 9, 1, 2};
    std::vector<int64_t> off(8);
    std::vector<int32_t> cap(8);
    int64_t total = 0;
    CHECK(baklava_layout(bud.data(), 2, 2, 2, 3, off.data(), cap.data(), &total) == BAKLAVA_OK);
    CHECK(total == 2 * (5 + 9 + 1 + 2) + 8 * 3);
    CHECK(off[7] + cap[7] == total);
    bud[0] = 2147483647;
    CHECK(baklava_layout(bud.data(), 2, 2, 2, 3, off.data(), cap.data(), &total) == BAKLAVA_EINVAL);
    CHECK(baklava_layout(bud.data(), 0, 2, 2, 3, off.data(), cap.data(), &total) == BAKLAVA_EINVAL);
  }
  CHECK(baklava_strerror(BAKLAVA_OK) != nullptr && baklava_strerror(12345) != nullptr);
  std::printf("%s (%d failures)\n", fails ? "FAILED" : "ok", fails);
  return fails ? 1 : 0;
}
