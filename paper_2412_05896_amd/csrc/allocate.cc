// Host-side adaptive allocation of per-layer KV-cache sizes.
//
// The paper's Alg. 1 grows an allocation list one token at a time, always
// taking the waiting token with the largest normalised contribution
// Sort(w_l)[-(n_l+1)] / Sum(w_l) (the marginal gain of Eq. 21).  Because each
// layer's contributions are non-increasing, the tokens taken after N steps are
// exactly the N largest contributions over all layers, equal values ordered by
// (layer, rank).  The total-size problem (Eq. 17) is therefore solved here by
// selecting a threshold over all contributions instead of iterating; the
// target-R_avg problem (Eq. 18) needs the running sum in the order of the
// picks and is solved by a heap merge of the per-layer sorted lists.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <functional>
#include <limits>
#include <queue>
#include <utility>
#include <vector>

#include "xkv.h"

namespace {

struct Layer {
  std::vector<float> asc;  // values sorted ascending
  double sum = 0.0;        // their sum, added in that order
  int64_t lo = 0, hi = 0;  // floor and cap on the budget
  // Contribution of the token of descending rank r (0 = largest).
  double p(int64_t r) const {
    if (sum == 0.0) return 0.0;
    return static_cast<double>(asc[asc.size() - 1 - static_cast<size_t>(r)]) / sum;
  }
  // Number of ranks in [from, hi) whose contribution satisfies pred; pred is
  // true on a prefix because contributions do not increase with rank.
  template <typename Pred>
  int64_t prefix(int64_t from, Pred pred) const {
    int64_t a = from, b = hi;
    while (a < b) {
      const int64_t mid = a + (b - a) / 2;
      if (pred(p(mid))) a = mid + 1; else b = mid;
    }
    return a - from;
  }
};

}  // namespace

extern "C" xkv_status xkv_allocate_budgets(int32_t n_layers, const float* const* w,
                                           const int64_t* len, int32_t mode, int64_t total_size,
                                           double target_ravg, const int64_t* min_budget,
                                           const int64_t* max_budget, int64_t* budgets_out,
                                           double* ravg_out) {
  if (n_layers <= 0 || w == nullptr || len == nullptr || budgets_out == nullptr)
    return XKV_ERR_INVALID_ARG;
  if (mode != XKV_ALLOC_TOTAL_SIZE && mode != XKV_ALLOC_TARGET_RAVG) return XKV_ERR_INVALID_ARG;
  if (mode == XKV_ALLOC_TARGET_RAVG && !(target_ravg >= 0.0 && target_ravg <= 1.0))
    return XKV_ERR_INVALID_ARG;
  for (int32_t l = 0; l < n_layers; ++l) {
    if (len[l] < 0 || (len[l] > 0 && w[l] == nullptr)) return XKV_ERR_INVALID_ARG;
    for (int64_t j = 0; j < len[l]; ++j) {
      const float x = w[l][j];
      if (!(x >= 0.0f) || std::isinf(x)) return XKV_ERR_INVALID_ARG;
    }
  }

  std::vector<Layer> layers(static_cast<size_t>(n_layers));
  int64_t sum_lo = 0, sum_hi = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    Layer& y = layers[l];
    y.lo = min_budget ? min_budget[l] : 0;
    y.hi = max_budget ? std::min<int64_t>(max_budget[l], len[l]) : len[l];
    if (y.lo < 0 || y.lo > y.hi) return XKV_ERR_INFEASIBLE;
    sum_lo += y.lo;
    sum_hi += y.hi;
  }
  if (mode == XKV_ALLOC_TOTAL_SIZE && (total_size < sum_lo || total_size > sum_hi))
    return XKV_ERR_INFEASIBLE;

  for (int32_t l = 0; l < n_layers; ++l) {
    Layer& y = layers[l];
    y.asc.assign(w[l], w[l] + len[l]);
    std::sort(y.asc.begin(), y.asc.end());
    double s = 0.0;
    for (float x : y.asc) s += static_cast<double>(x);
    y.sum = s;
  }

  std::vector<int64_t> n(static_cast<size_t>(n_layers));
  for (int32_t l = 0; l < n_layers; ++l) n[l] = layers[l].lo;

  if (mode == XKV_ALLOC_TOTAL_SIZE) {
    const int64_t need = total_size - sum_lo;
    if (need > 0) {
      // Threshold = the need-th largest contribution among all candidates.
      std::vector<double> all;
      all.reserve(static_cast<size_t>(sum_hi - sum_lo));
      for (const Layer& y : layers)
        for (int64_t r = y.lo; r < y.hi; ++r) all.push_back(y.p(r));
      std::nth_element(all.begin(), all.begin() + (need - 1), all.end(), std::greater<double>());
      const double tau = all[static_cast<size_t>(need - 1)];
      int64_t taken = 0;
      for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t gt = layers[l].prefix(layers[l].lo, [tau](double x) { return x > tau; });
        n[l] += gt;
        taken += gt;
      }
      // Contributions equal to the threshold: lower layers first.
      int64_t left = need - taken;
      for (int32_t l = 0; l < n_layers && left > 0; ++l) {
        const int64_t eq = layers[l].prefix(n[l], [tau](double x) { return x >= tau; });
        const int64_t take = std::min(eq, left);
        n[l] += take;
        left -= take;
      }
    }
  } else {
    // Importance already held by the floors, then picks in greedy order.
    double r_total = 0.0;
    for (int32_t l = 0; l < n_layers; ++l)
      for (int64_t r = 0; r < layers[l].lo; ++r) r_total += layers[l].p(r);
    using Item = std::pair<double, int32_t>;  // (contribution, layer)
    auto worse = [](const Item& a, const Item& b) {
      return a.first < b.first || (a.first == b.first && a.second > b.second);
    };
    std::priority_queue<Item, std::vector<Item>, decltype(worse)> heap(worse);
    for (int32_t l = 0; l < n_layers; ++l)
      if (n[l] < layers[l].hi) heap.push({layers[l].p(n[l]), l});
    while (r_total / n_layers < target_ravg && !heap.empty()) {
      const Item top = heap.top();
      heap.pop();
      r_total += top.first;
      const int32_t l = top.second;
      n[l] += 1;
      if (n[l] < layers[l].hi) heap.push({layers[l].p(n[l]), l});
    }
  }

  double ravg = 0.0;
  for (int32_t l = 0; l < n_layers; ++l) {
    double r = 0.0;
    for (int64_t k = 0; k < n[l]; ++k) r += layers[l].p(k);
    ravg += r;
    budgets_out[l] = n[l];
  }
  if (ravg_out) *ravg_out = ravg / n_layers;
  return XKV_OK;
}

// Sampling-based overhead reduction (Sec. 4.3): the allocation lists recorded
// on sampled tasks are averaged into the list for the next task.  All
// arithmetic is exact: with column sums c_l and grand total C the target of
// layer l is x_l = N c_l / C, compared through the integers N c_l - n_l C.
extern "C" xkv_status xkv_average_allocations(int32_t n_samples, int32_t n_layers,
                                              const int64_t* lists, int64_t total_size,
                                              const int64_t* min_budget, const int64_t* max_budget,
                                              int64_t* budgets_out) {
  if (n_samples <= 0 || n_layers <= 0 || lists == nullptr || budgets_out == nullptr || total_size < 0)
    return XKV_ERR_INVALID_ARG;
  typedef __int128 wide;
  std::vector<wide> col(static_cast<size_t>(n_layers), 0);
  wide tot = 0;
  for (int32_t s = 0; s < n_samples; ++s)
    for (int32_t l = 0; l < n_layers; ++l) {
      const int64_t v = lists[static_cast<int64_t>(s) * n_layers + l];
      if (v < 0) return XKV_ERR_INVALID_ARG;
      col[l] += v;
      tot += v;
    }
  if (tot == 0) return XKV_ERR_INVALID_ARG;
  std::vector<int64_t> lo(n_layers), hi(n_layers);
  wide sum_lo = 0, sum_hi = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    lo[l] = min_budget ? min_budget[l] : 0;
    hi[l] = max_budget ? max_budget[l] : std::numeric_limits<int64_t>::max();
    if (lo[l] < 0 || lo[l] > hi[l]) return XKV_ERR_INFEASIBLE;
    sum_lo += lo[l];
    sum_hi += hi[l];
  }
  if (total_size < sum_lo || total_size > sum_hi) return XKV_ERR_INFEASIBLE;

  const wide N = total_size;
  std::vector<int64_t> n(n_layers);
  std::vector<wide> rem(n_layers);               // N c_l mod C: the fractional part times C
  wide given = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    n[l] = static_cast<int64_t>(N * col[l] / tot);
    rem[l] = N * col[l] % tot;
    given += n[l];
  }
  std::vector<int32_t> order(n_layers);
  for (int32_t l = 0; l < n_layers; ++l) order[l] = l;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return rem[a] > rem[b]; });
  for (int64_t i = 0; i < static_cast<int64_t>(N - given); ++i) n[order[static_cast<size_t>(i)]] += 1;

  wide have = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    n[l] = std::max(lo[l], std::min(hi[l], n[l]));
    have += n[l];
  }
  // deficit of layer l times C: N c_l - n_l C (how far it is below its target)
  auto deficit = [&](int32_t l) { return N * col[l] - static_cast<wide>(n[l]) * tot; };
  while (have != N) {
    int32_t pick = -1;
    for (int32_t l = 0; l < n_layers; ++l) {
      if (have < N) {
        if (n[l] >= hi[l]) continue;
        if (pick < 0 || deficit(l) > deficit(pick)) pick = l;
      } else {
        if (n[l] <= lo[l]) continue;
        if (pick < 0 || deficit(l) < deficit(pick)) pick = l;
      }
    }
    if (pick < 0) return XKV_ERR_INFEASIBLE;     // cannot happen after the checks above
    if (have < N) { n[pick] += 1; have += 1; } else { n[pick] -= 1; have -= 1; }
  }
  for (int32_t l = 0; l < n_layers; ++l) budgets_out[l] = n[l];
  return XKV_OK;
}
