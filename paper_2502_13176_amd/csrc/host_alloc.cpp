// Host-only part of libbaklava: budget allocation and arena layout.
// No GPU call is made from this file.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <vector>

#include "baklava.h"

namespace {

typedef unsigned __int128 u128;
constexpr int kFracBits = 40;
constexpr uint64_t kOne = uint64_t(1) << kFracBits;

inline int64_t clip64(u128 x, int64_t lo, int64_t hi) {
  if (x < (u128)lo) return lo;
  if (x > (u128)hi) return hi;
  return (int64_t)x;
}

}  // namespace

extern "C" const char* baklava_strerror(int status) {
  switch (status) {
    case BAKLAVA_OK: return "ok";
    case BAKLAVA_EINVAL: return "invalid argument";
    case BAKLAVA_EINFEASIBLE: return "budget constraints cannot be met";
    case BAKLAVA_ECAPACITY: return "capacity exceeded";
    case BAKLAVA_EHIP: return "HIP runtime call failed";
    case BAKLAVA_ESTATE: return "call order violated";
    case BAKLAVA_ENOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

// Proportional budgets with an exact sum: the allocator the benchmark workloads ask for (the paper
// itself only states the principle that more important caches get more memory, and gives
// Algorithm 2).  Fixed-point weights make every rounding an integer decision.
extern "C" int baklava_alloc_proportional(const double* importance, int32_t m, int64_t global_budget,
                                          int32_t lo, int32_t hi, int32_t* budget_out) {
  if (!importance || !budget_out || m <= 0 || lo < 0 || hi < lo || global_budget < 0) return BAKLAVA_EINVAL;
  double top = 0.0;
  for (int32_t i = 0; i < m; ++i) {
    const double v = importance[i];
    if (!std::isfinite(v) || !(v > 0.0)) return BAKLAVA_EINVAL;
    top = std::max(top, v);
  }
  if ((int64_t)m * lo > global_budget || (int64_t)m * hi < global_budget) return BAKLAVA_EINFEASIBLE;

  std::vector<uint64_t> w(m);
  uint64_t wmin = kOne;
  for (int32_t i = 0; i < m; ++i) {
    const double scaled = std::floor((importance[i] / top) * (double)kOne);
    w[i] = scaled < 1.0 ? 1 : (uint64_t)scaled;
    wmin = std::min(wmin, w[i]);
  }
  auto filled = [&](u128 lam) -> int64_t {
    int64_t s = 0;
    for (int32_t i = 0; i < m; ++i) s += clip64((lam * w[i]) >> kFracBits, lo, hi);
    return s;
  };
  // Above lam_top every head is clipped to hi.
  const u128 lam_top = (((u128)hi << kFracBits) / wmin) + 1;
  u128 lam;
  if (filled(lam_top) <= global_budget) {
    lam = lam_top;
  } else {
    u128 a = 0, z = lam_top;  // filled(a) <= B < filled(z)
    while (z - a > 1) {
      const u128 mid = a + (z - a) / 2;
      if (filled(mid) <= global_budget) a = mid; else z = mid;
    }
    lam = a;
  }
  struct Cand { uint64_t frac, w; int32_t i; };
  std::vector<Cand> elig;
  int64_t sum = 0;
  for (int32_t i = 0; i < m; ++i) {
    const u128 prod = lam * w[i];
    const u128 x = prod >> kFracBits;
    const int64_t b = clip64(x, lo, hi);
    budget_out[i] = (int32_t)b;
    sum += b;
    if (x >= (u128)lo && x < (u128)hi) elig.push_back({(uint64_t)(prod & (kOne - 1)), w[i], i});
  }
  int64_t left = global_budget - sum;
  if (left < 0 || left > (int64_t)elig.size()) return BAKLAVA_EINFEASIBLE;  // cannot happen
  std::sort(elig.begin(), elig.end(), [](const Cand& p, const Cand& q) {
    if (p.frac != q.frac) return p.frac > q.frac;
    if (p.w != q.w) return p.w > q.w;
    return p.i < q.i;
  });
  for (int64_t r = 0; r < left; ++r) budget_out[elig[r].i] += 1;
  return BAKLAVA_OK;
}

// Algorithm 2: shrink the caches below the importance threshold, hand what they free to the
// most important of the others.
extern "C" int baklava_alloc_threshold(const double* importance, int32_t m, const int32_t* size_in,
                                       double t, double r, int32_t* budget_out) {
  if (!importance || !size_in || !budget_out || m <= 0) return BAKLAVA_EINVAL;
  if (!(r >= 0.0 && r <= 1.0) || !std::isfinite(t)) return BAKLAVA_EINVAL;
  std::vector<int64_t> size(m);
  std::vector<int32_t> low, high;
  for (int32_t i = 0; i < m; ++i) {
    // the algorithm orders importances and compares them with t: a NaN has no place in either
    if (size_in[i] < 0 || !std::isfinite(importance[i])) return BAKLAVA_EINVAL;
    size[i] = size_in[i];
    (importance[i] < t ? low : high).push_back(i);
  }
  const int64_t n = (int64_t)low.size();
  if (n != 0 && n != m) {
    int64_t freed = 0;
    for (int32_t i : low) {
      const int64_t d = (int64_t)std::floor(r * (double)size[i]);
      size[i] -= d;
      freed += d;
    }
    const int64_t k = std::min<int64_t>(n, m - n);
    std::stable_sort(high.begin(), high.end(),
                     [&](int32_t a, int32_t b) { return importance[a] > importance[b]; });
    const int64_t base = freed / k, rem = freed % k;
    for (int64_t rank = 0; rank < k; ++rank) size[high[rank]] += base + (rank < rem ? 1 : 0);
  }
  for (int32_t i = 0; i < m; ++i) {
    if (size[i] > INT32_MAX) return BAKLAVA_EINVAL;
    budget_out[i] = (int32_t)size[i];
  }
  return BAKLAVA_OK;
}

extern "C" int baklava_layout(const int32_t* budget, int32_t L, int32_t Hkv, int32_t batch,
                              int32_t slack, int64_t* off_out, int32_t* cap_out,
                              int64_t* total_tokens_out) {
  if (!budget || !off_out || !cap_out || !total_tokens_out) return BAKLAVA_EINVAL;
  if (L <= 0 || Hkv <= 0 || batch <= 0 || slack < 0) return BAKLAVA_EINVAL;
  int64_t total = 0;
  for (int32_t l = 0; l < L; ++l)
    for (int32_t b = 0; b < batch; ++b)
      for (int32_t h = 0; h < Hkv; ++h) {
        const int64_t bud = budget[(int64_t)l * Hkv + h];
        if (bud < 0 || bud + slack > INT32_MAX) return BAKLAVA_EINVAL;
        const int64_t c = ((int64_t)l * batch + b) * Hkv + h;
        off_out[c] = total;
        cap_out[c] = (int32_t)(bud + slack);
        total += bud + slack;
      }
  *total_tokens_out = total;
  return BAKLAVA_OK;
}

// Algorithm 1, step 2: group mean of the head similarities, affine map to [0, 1], complement.
extern "C" int baklava_kv_importance(const double* similarity_host, int32_t L, int32_t Hq, int32_t Hkv,
                                     double* importance_out) {
  if (!similarity_host || !importance_out || L <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) return BAKLAVA_EINVAL;
  const int32_t G = Hq / Hkv;
  // a rounding slack on the range check: means of fp32 cosines can exceed 1 by an ulp
  for (int64_t i = 0; i < (int64_t)L * Hq; ++i)
    if (!std::isfinite(similarity_host[i]) || std::fabs(similarity_host[i]) > 1.0 + 1e-6) return BAKLAVA_EINVAL;
  for (int32_t l = 0; l < L; ++l)
    for (int32_t h = 0; h < Hkv; ++h) {
      double acc = 0.0;
      for (int32_t g = 0; g < G; ++g) acc += similarity_host[(int64_t)l * Hq + (int64_t)h * G + g];
      importance_out[(int64_t)l * Hkv + h] = 1.0 - (acc / G + 1.0) / 2.0;
    }
  return BAKLAVA_OK;
}

// Layer pools by the proportional rule, then an equal split and Algorithm 2 inside each layer.
extern "C" int baklava_alloc_two_level(const double* layer_importance, const double* head_importance, int32_t L,
                                       int32_t Hkv, int64_t global_budget, int32_t lo, int32_t hi, double t,
                                       double r, int32_t* budget_out) {
  if (!layer_importance || !head_importance || !budget_out || L <= 0 || Hkv <= 0) return BAKLAVA_EINVAL;
  if (lo < 0 || hi < lo || (int64_t)Hkv * hi > INT32_MAX) return BAKLAVA_EINVAL;
  std::vector<int32_t> pools(L);
  int st = baklava_alloc_proportional(layer_importance, L, global_budget, Hkv * lo, Hkv * hi, pools.data());
  if (st != BAKLAVA_OK) return st;
  std::vector<int32_t> size(Hkv), order(Hkv);
  for (int32_t l = 0; l < L; ++l) {
    const double* imp = head_importance + (int64_t)l * Hkv;
    const int32_t base = pools[l] / Hkv, rem = pools[l] % Hkv;
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return imp[a] > imp[b]; });
    std::fill(size.begin(), size.end(), base);
    for (int32_t i = 0; i < rem; ++i) size[order[i]] += 1;
    st = baklava_alloc_threshold(imp, Hkv, size.data(), t, r, budget_out + (int64_t)l * Hkv);
    if (st != BAKLAVA_OK) return st;
  }
  return BAKLAVA_OK;
}

// Split-K schedule: runs of equal length over each cache's capacity, in launch order.
extern "C" int baklava_plan_schedule(const int64_t* off_host, const int32_t* cap_host, int32_t L,
                                     int32_t caches_per_layer, int32_t chunk, int32_t target_items,
                                     int32_t whole_model, int64_t max_items, baklava_work_item* items_out,
                                     int64_t* n_items_out) {
  if (!off_host || !cap_host || !n_items_out || L <= 0 || caches_per_layer <= 0) return BAKLAVA_EINVAL;
  if (chunk < 256 || chunk % 64 || chunk > (1 << 22) || max_items < 0 || target_items < 0) return BAKLAVA_EINVAL;
  if (whole_model != 0 && whole_model != 1) return BAKLAVA_EINVAL;
  const int64_t n_caches = (int64_t)L * caches_per_layer;
  for (int64_t c = 0; c < n_caches; ++c)
    if (cap_host[c] < 0 || off_host[c] < 0) return BAKLAVA_EINVAL;
  auto runs = [&](int64_t c, int64_t run) { return std::max<int64_t>(1, ((int64_t)cap_host[c] + run - 1) / run); };
  auto round64 = [](int64_t x) { return (x + 63) / 64 * 64; };
  // run length of every cache: `chunk`, or what the item target of its launch unit (a layer, or
  // the whole model) asks for
  const int64_t n_units = whole_model ? 1 : L;
  const int64_t unit_caches = whole_model ? n_caches : caches_per_layer;
  std::vector<int64_t> cache_run(n_caches, chunk);
  if (target_items > 0) {
    for (int64_t u = 0; u < n_units; ++u) {
      const int64_t c0 = u * unit_caches, c1 = c0 + unit_caches;
      auto items_at = [&](int64_t run) {
        int64_t n = 0;
        for (int64_t c = c0; c < c1; ++c) n += runs(c, run);
        return n;
      };
      // a unit never has fewer items than caches
      const int64_t target = std::max<int64_t>(target_items, unit_caches);
      if (items_at(chunk) <= target) continue;
      // the shortest run length, in steps of 64 rows, that meets the target (items_at is non-increasing)
      int64_t lo = chunk / 64, hi = (int64_t(1) << 31) / 64;
      while (hi - lo > 1) {
        const int64_t mid = (lo + hi) / 2;
        if (items_at(mid * 64) > target) lo = mid; else hi = mid;
      }
      // a work item never spans more than 2^22 rows (the kernels address its rows with 32-bit byte offsets)
      const int64_t unit_run = std::min<int64_t>(hi * 64, int64_t(1) << 22);
      // inside a cache the runs are then made equal: no run grows, the count stays
      for (int64_t c = c0; c < c1; ++c) {
        const int64_t n = runs(c, unit_run);
        cache_run[c] = std::max<int64_t>(chunk, round64(((int64_t)cap_host[c] + n - 1) / n));
      }
    }
  }
  std::vector<int64_t> first_slot(n_caches + 1, 0);
  for (int64_t c = 0; c < n_caches; ++c) first_slot[c + 1] = first_slot[c] + runs(c, cache_run[c]);
  const int64_t n_items = first_slot[n_caches];
  *n_items_out = n_items;
  if (n_items > INT32_MAX) return BAKLAVA_EINVAL;
  if (!items_out) return BAKLAVA_OK;
  if (n_items > max_items) return BAKLAVA_ECAPACITY;
  // cache order: longest capacity first (stable), inside each layer or over the whole model
  std::vector<int32_t> order(n_caches);
  std::iota(order.begin(), order.end(), 0);
  auto longer = [&](int32_t a, int32_t b) { return cap_host[a] > cap_host[b]; };
  if (whole_model) {
    std::stable_sort(order.begin(), order.end(), longer);
  } else {
    for (int32_t l = 0; l < L; ++l)
      std::stable_sort(order.begin() + (int64_t)l * caches_per_layer,
                       order.begin() + (int64_t)(l + 1) * caches_per_layer, longer);
  }
  int64_t k = 0;
  for (int32_t c : order) {
    const int32_t cap = cap_host[c];
    const int64_t run = cache_run[c];
    const int32_t nsplit = (int32_t)(first_slot[c + 1] - first_slot[c]);
    for (int32_t s = 0; s < nsplit; ++s) {
      baklava_work_item& it = items_out[k++];
      it.cache = c;
      it.start = (int32_t)(s * run);
      it.count = (int32_t)std::max<int64_t>(0, std::min<int64_t>(run, cap - s * run));
      it.slot = (int32_t)(first_slot[c] + s);
      it.nsplit = nsplit;
      it.reserved = 0;
      it.row0 = off_host[c] + it.start;
    }
  }
  return BAKLAVA_OK;
}
