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
    // a NaN importance would make the ordering of the receivers undefined: refused, like a NaN threshold
    const double keep = u[m / 2];
    u[m / 2] = std::nan("");
    CHECK(baklava_alloc_threshold(u.data(), m, size.data(), 0.5, 0.3, out.data()) == BAKLAVA_EINVAL);
    u[m / 2] = keep;
    CHECK(baklava_alloc_threshold(u.data(), m, size.data(), std::nan(""), 0.3, out.data()) == BAKLAVA_EINVAL);
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
  // split-K planner: random capacities (zero, tiny, beyond the longest run), every target / launch kind
  for (int rep = 0; rep < 200; ++rep) {
    const int L = 1 + (int)(rng() % 4), cpl = 1 + (int)(rng() % 9);
    const int n = L * cpl;
    std::vector<int32_t> cap(n);
    std::vector<int64_t> off(n);
    int64_t total = 0;
    for (int c = 0; c < n; ++c) {
      const uint64_t r = rng() % 100;
      cap[c] = r < 5 ? 0 : r < 60 ? (int32_t)(rng() % 700) : r < 98 ? (int32_t)(rng() % 200000) : (int32_t)((1 << 22) + rng() % 5000);
      off[c] = total;
      total += cap[c];
    }
    const int chunk = 256 + 64 * (int)(rng() % 30);
    const int target = (rng() % 3 == 0) ? 0 : 1 + (int)(rng() % 600);
    const int whole = (int)(rng() % 2);
    int64_t n_items = -1;
    CHECK(baklava_plan_schedule(off.data(), cap.data(), L, cpl, chunk, target, whole, 0, nullptr, &n_items) == BAKLAVA_OK);
    CHECK(n_items >= n);
    std::vector<baklava_work_item> items((size_t)n_items);
    int64_t n2 = -1;
    CHECK(baklava_plan_schedule(off.data(), cap.data(), L, cpl, chunk, target, whole, n_items, items.data(), &n2) == BAKLAVA_OK);
    CHECK(n2 == n_items);
    std::vector<int64_t> rows(n, 0);
    std::vector<char> slot_seen((size_t)n_items, 0);
    for (const baklava_work_item& it : items) {
      CHECK(it.cache >= 0 && it.cache < n && it.count >= 0 && it.count <= (1 << 22));
      CHECK(it.start % 64 == 0 && it.start + (int64_t)it.count <= cap[it.cache] && it.row0 == off[it.cache] + it.start);
      CHECK(it.slot >= 0 && it.slot < n_items && !slot_seen[it.slot]);
      slot_seen[it.slot] = 1;
      rows[it.cache] += it.count;
    }
    for (int c = 0; c < n; ++c) CHECK(rows[c] == cap[c]);
    if (n_items > 1) {
      CHECK(baklava_plan_schedule(off.data(), cap.data(), L, cpl, chunk, target, whole, n_items - 1, items.data(), &n2) == BAKLAVA_ECAPACITY);
      CHECK(n2 == n_items);
    }
  }
  {
    int64_t off1 = 0, n_items = 0;
    int32_t cap1 = 1000;
    CHECK(baklava_plan_schedule(&off1, &cap1, 1, 1, 100, 0, 0, 0, nullptr, &n_items) == BAKLAVA_EINVAL);   // chunk below 256
    CHECK(baklava_plan_schedule(&off1, &cap1, 1, 1, 300, 0, 0, 0, nullptr, &n_items) == BAKLAVA_EINVAL);   // not a multiple of 64
    CHECK(baklava_plan_schedule(nullptr, &cap1, 1, 1, 256, 0, 0, 0, nullptr, &n_items) == BAKLAVA_EINVAL);
    cap1 = -5;
    CHECK(baklava_plan_schedule(&off1, &cap1, 1, 1, 256, 0, 0, 0, nullptr, &n_items) == BAKLAVA_EINVAL);
  }
  // importances from similarities, and the two-level allocation
  for (int rep = 0; rep < 200; ++rep) {
    const int L = 1 + (int)(rng() % 6), Hkv = 1 + (int)(rng() % 8), G = 1 + (int)(rng() % 8);
    std::vector<double> sim((size_t)L * Hkv * G), imp((size_t)L * Hkv), limp(L);
    for (double& v : sim) v = (double)(rng() % 2001) / 1000.0 - 1.0;
    CHECK(baklava_kv_importance(sim.data(), L, Hkv * G, Hkv, imp.data()) == BAKLAVA_OK);
    for (double v : imp) CHECK(v >= 0.0 && v <= 1.0);
    for (double& v : limp) v = 0.001 + (double)(rng() % 1000) / 1000.0;
    for (double& v : imp) v += 1e-6;                              // strictly positive for the allocator
    const int lo = 1 + (int)(rng() % 50), hi = lo + 1 + (int)(rng() % 5000);
    const int64_t m = (int64_t)L * Hkv;
    const int64_t B = m * lo + (int64_t)(rng() % (uint64_t)(m * (hi - lo) + 1));
    std::vector<int32_t> bud((size_t)m, -1);
    CHECK(baklava_alloc_two_level(limp.data(), imp.data(), L, Hkv, B, lo, hi, 0.5, 0.25, bud.data()) == BAKLAVA_OK);
    int64_t sum = 0;
    for (int32_t b : bud) { CHECK(b >= 0); sum += b; }
    CHECK(sum == B);
    CHECK(baklava_alloc_two_level(limp.data(), imp.data(), L, Hkv, m * lo - 1, lo, hi, 0.5, 0.25, bud.data()) == BAKLAVA_EINFEASIBLE);
  }
  CHECK(baklava_kv_importance(nullptr, 1, 4, 2, nullptr) == BAKLAVA_EINVAL);
  {
    double s4[4] = {0.1, 0.2, 0.3, 0.4}, o2[2];
    CHECK(baklava_kv_importance(s4, 1, 4, 3, o2) == BAKLAVA_EINVAL);   // 4 heads do not split over 3 KV heads
  }
  CHECK(baklava_strerror(BAKLAVA_OK) != nullptr && baklava_strerror(12345) != nullptr);
  std::printf("%s (%d failures)\n", fails ? "FAILED" : "ok", fails);
  return fails ? 1 : 0;
}
