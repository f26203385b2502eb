// Host-side trajectory placement (paper Sec. 5.2): presorted dynamic programming over the
// trajectories in descending length order (Eq. 3), the interference factor F(s) tabulated from a
// profile of the decode step time per batch size, bundling of the short tail, and the simulator
// of a group that decodes concurrently.  Plain C++; no device work.
#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

#include "heddle.h"

namespace {

// Cost of one worker's group: longest trajectory x base per-token time x interference of the
// group's size; the product order is part of the contract (results are compared bit for bit).
inline double group_cost(double first_len, double T, const double* F, int64_t size) { return (first_len * T) * F[size]; }

struct Profile {
  int32_t n;
  const double* bs;
  const double* ts;
  // step time at batch size s: linear between the profiled points, flat below the first,
  // last slope continued above the last
  double at(double s) const {
    if (s <= bs[0] || n == 1) return ts[0];
    for (int32_t i = 0; i + 1 < n; ++i)
      if (s <= bs[i + 1]) return ts[i] + (ts[i + 1] - ts[i]) * ((s - bs[i]) / (bs[i + 1] - bs[i]));
    return ts[n - 1] + (ts[n - 1] - ts[n - 2]) * ((s - bs[n - 1]) / (bs[n - 1] - bs[n - 2]));
  }
  bool valid() const {
    if (n < 1 || bs == nullptr || ts == nullptr) return false;
    for (int32_t i = 0; i + 1 < n; ++i)
      if (!(bs[i] < bs[i + 1])) return false;
    return true;
  }
};

}  // namespace

extern "C" {

int heddle_placement_dp(int32_t n, const double* len_desc, const int32_t* count, int32_t m, const double* F,
                        int32_t F_len, double T, int32_t mode, int32_t* sizes_out, double* makespan_out) {
  if (n < 0 || m < 1 || sizes_out == nullptr || makespan_out == nullptr || (mode != 0 && mode != 1))
    return HEDDLE_E_INVAL;
  if (n > 0 && (len_desc == nullptr || F == nullptr)) return HEDDLE_E_INVAL;
  std::fill(sizes_out, sizes_out + m, 0);
  *makespan_out = 0.0;
  if (n == 0) return HEDDLE_OK;
  for (int32_t i = 0; i + 1 < n; ++i)
    if (len_desc[i] < len_desc[i + 1]) return HEDDLE_E_INVAL;

  std::vector<int64_t> cum(static_cast<size_t>(n) + 1, 0);        // members among the first i elements
  for (int32_t i = 0; i < n; ++i) {
    const int64_t c = count ? count[i] : 1;
    if (c < 1) return HEDDLE_E_INVAL;
    cum[i + 1] = cum[i] + c;
  }
  if (cum[n] >= F_len) return HEDDLE_E_INVAL;                     // F must reach the largest possible group

  // The crossing search below needs F non-decreasing over the sizes that can occur.
  bool monotone = true;
  for (int64_t s = 1; s < cum[n] && monotone; ++s) monotone = F[s] <= F[s + 1];
  const bool scan = mode == 1 || !monotone;

  const int32_t J = std::min(m, n);
  const size_t stride = static_cast<size_t>(n) + 1;
  std::vector<double> dp(stride * (J + 1), std::numeric_limits<double>::infinity());   // dp[j * stride + i]
  std::vector<int32_t> arg(stride * (J + 1), -1);
  dp[0] = 0.0;
  for (int32_t i = 1; i <= n; ++i) {
    dp[stride + i] = group_cost(len_desc[0], T, F, cum[i]);
    arg[stride + i] = 0;
  }
  for (int32_t j = 2; j <= J; ++j) {
    const double* prev = &dp[stride * (j - 1)];
    for (int32_t i = j; i <= n; ++i) {
      auto tail = [&](int32_t k) { return group_cost(len_desc[k], T, F, cum[i] - cum[k]); };
      double best = std::numeric_limits<double>::infinity();
      int32_t best_k = -1;
      if (scan) {                                   // Eq. 3 as written: every split position
        for (int32_t k = j - 1; k < i; ++k) {
          const double v = std::max(prev[k], tail(k));
          if (v < best) best = v, best_k = k;
        }
      } else {
        // prev[k] does not decrease with k and tail(k) does not increase: the minimum of their
        // maximum sits where they cross.  first = smallest k with prev[k] >= tail(k).
        int32_t lo = j - 1, hi = i;                 // answer in [lo, hi]; hi = i means "never"
        while (lo < hi) {
          const int32_t mid = lo + (hi - lo) / 2;
          if (prev[mid] >= tail(mid)) hi = mid; else lo = mid + 1;
        }
        const int32_t first = lo;
        if (first < i) best = prev[first], best_k = first;
        if (first > j - 1) {
          const double before = tail(first - 1);    // left of the crossing the maximum is tail(k)
          if (before <= best) {
            // smallest k whose tail(k) already equals this value (ties go to the smallest k)
            int32_t a = j - 1, b = first - 1;
            while (a < b) {
              const int32_t mid = a + (b - a) / 2;
              if (tail(mid) <= before) b = mid; else a = mid + 1;
            }
            best = before, best_k = a;
          }
        }
      }
      dp[stride * j + i] = best;
      arg[stride * j + i] = best_k;
    }
  }
  *makespan_out = dp[stride * J + n];
  int32_t i = n;
  for (int32_t j = J; j >= 1; --j) {
    const int32_t k = arg[stride * j + i];
    sizes_out[j - 1] = i - k;
    i = k;
  }
  return HEDDLE_OK;
}

int heddle_placement_aggregate(int32_t n, const double* len_desc, double threshold, int32_t bundle,
                               int32_t* first_out, int32_t* count_out, int32_t* n_elems_out) {
  if (n < 0 || n_elems_out == nullptr || (n > 0 && (!len_desc || !first_out || !count_out))) return HEDDLE_E_INVAL;
  int32_t e = 0;
  for (int32_t i = 0; i < n;) {
    const int32_t c = (len_desc[i] >= threshold || bundle <= 1) ? 1 : std::min(bundle, n - i);
    first_out[e] = i;
    count_out[e] = c;
    ++e;
    i += c;
  }
  *n_elems_out = e;
  return HEDDLE_OK;
}

int heddle_interference_table(int32_t n_prof, const double* batch_sizes, const double* step_time, int32_t n,
                              double* F_out) {
  const Profile p{n_prof, batch_sizes, step_time};
  if (!p.valid() || n < 0 || F_out == nullptr) return HEDDLE_E_INVAL;
  const double t1 = p.at(1.0);
  if (!(t1 > 0.0)) return HEDDLE_E_INVAL;
  F_out[0] = 0.0;
  for (int32_t s = 1; s <= n; ++s) F_out[s] = std::max(p.at(static_cast<double>(s)) / t1, F_out[s - 1]);
  return HEDDLE_OK;
}

int heddle_simulate_group(int32_t n, const int32_t* lengths, int32_t n_prof, const double* batch_sizes,
                          const double* step_time, double* time_out) {
  const Profile p{n_prof, batch_sizes, step_time};
  if (!p.valid() || n < 0 || time_out == nullptr || (n > 0 && lengths == nullptr)) return HEDDLE_E_INVAL;
  for (int32_t i = 0; i < n; ++i)
    if (lengths[i] < 0) return HEDDLE_E_INVAL;
  std::vector<int32_t> L(lengths, lengths + n);
  std::sort(L.begin(), L.end(), [](int32_t a, int32_t b) { return a > b; });
  double total = 0.0;
  int64_t done = 0;
  for (int32_t active = n; active >= 1; --active) {       // the shortest one still running ends the phase
    const int64_t upto = L[active - 1];
    total += static_cast<double>(upto - done) * p.at(static_cast<double>(active));
    done = upto;
  }
  *time_out = total;
  return HEDDLE_OK;
}

}  // extern "C"
