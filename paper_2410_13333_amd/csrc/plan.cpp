// Lower level of the parallelization planner (Sec. 4.2, Eq. 1-3), Theorem 2 and the theoretic optimum of Sec. 7.2.
// Host code only; the C ABI is declared in include/mls_plan.h.
//
// Eq. 2 and Eq. 3 have the same shape: minimise max_j r_j * k_j over non-negative integers k_j with sum k_j = S and
// optional upper bounds.  The optimal value is one of the products r_j * k (k = 0..S); a value v is feasible iff
// sum_j min(cap_j, max{k : r_j * k <= v}) >= S, which is monotone in v, so the smallest feasible candidate is found
// by bisection over the sorted candidates.  All comparisons are between products r_j * k computed the same way, so
// no rounding of a quotient can misplace a candidate.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "../../include/mls.h"
#include "../../include/mls_plan.h"
#include "kernels.h"

namespace {

// largest k in [0, hi] with r * k <= v
int64_t count_within(double r, double v, int64_t hi) {
  if (hi <= 0) return 0;
  double q = std::floor(v / r);
  int64_t k = q >= double(hi) ? hi : (q <= 0 ? 0 : int64_t(q));
  while (k < hi && r * double(k + 1) <= v) k++;
  while (k > 0 && r * double(k) > v) k--;
  return k;
}

// the shared min-max split; returns false if the bounds cannot hold S
bool minmax_split(const double* r, const int64_t* cap, int n, int64_t S, int64_t* k, double* value) {
  std::vector<int64_t> hi(n);
  int64_t room = 0;
  for (int j = 0; j < n; j++) {
    hi[j] = (cap && cap[j] >= 0) ? std::min(cap[j], S) : S;
    room += hi[j];
  }
  if (room < S) return false;
  auto feasible = [&](double v) {
    int64_t got = 0;
    for (int j = 0; j < n && got < S; j++) got += count_within(r[j], v, hi[j]);
    return got >= S;
  };
  // bisection over the candidates r_j * c, one stage at a time: for each stage the smallest count c whose product
  // is feasible (binary search, the products of one stage are sorted); the optimum is the smallest of those
  double best = std::numeric_limits<double>::infinity();
  for (int j = 0; j < n; j++) {
    if (!feasible(r[j] * double(hi[j]))) continue;
    int64_t lo = 0, up = hi[j];
    while (lo < up) {
      const int64_t mid = lo + (up - lo) / 2;
      if (feasible(r[j] * double(mid))) up = mid; else lo = mid + 1;
    }
    best = std::min(best, r[j] * double(lo));
  }
  // Among the splits that reach the optimum, take the one with the smallest SUM of loads (the warm-up and
  // cool-down term of the pipeline time model, Sec. 4.2): fill the fastest stages up to what fits under the
  // optimum first (ties: the earlier stage first).
  std::vector<int> order(n);
  for (int j = 0; j < n; j++) order[j] = j;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return r[a] < r[b]; });
  int64_t left = S;
  for (int j = 0; j < n; j++) k[j] = 0;
  for (int j : order) {
    k[j] = std::min(left, count_within(r[j], best, hi[j]));
    left -= k[j];
  }
  double v = 0;
  for (int j = 0; j < n; j++) v = std::max(v, r[j] * double(k[j]));
  if (value) *value = v;
  return true;
}

bool rates_ok(const double* r, int n) {
  for (int j = 0; j < n; j++)
    if (!(r[j] > 0) || !std::isfinite(r[j])) return false;
  return true;
}

}  // namespace

extern "C" {

int mls_plan_layers(const double* y, const int64_t* cap, int32_t n, int64_t L, int64_t* l, double* o) {
  if (!y || !l) return mls::set_error(MLS_E_NULL, "mls_plan_layers: null argument");
  if (n < 1 || L < 0 || !rates_ok(y, n)) return mls::set_error(MLS_E_CONFIG, "mls_plan_layers: need n >= 1, L >= 0 and finite rates > 0");
  std::vector<int64_t> out(n);
  double v = 0;
  if (!minmax_split(y, cap, n, L, out.data(), &v)) return mls::set_error(MLS_E_RANGE, "mls_plan_layers: the stage capacities cannot hold L layers");
  std::copy(out.begin(), out.end(), l);
  if (o) *o = v;
  return MLS_OK;
}

int mls_plan_microbatches(const double* o, int32_t dp, int64_t n_mb, int64_t* m, double* t) {
  if (!o || !m) return mls::set_error(MLS_E_NULL, "mls_plan_microbatches: null argument");
  if (dp < 1 || n_mb < 0 || !rates_ok(o, dp)) return mls::set_error(MLS_E_CONFIG, "mls_plan_microbatches: need dp >= 1, n_mb >= 0 and finite bottlenecks > 0");
  std::vector<int64_t> out(dp);
  double v = 0;
  minmax_split(o, nullptr, dp, n_mb, out.data(), &v);
  std::copy(out.begin(), out.end(), m);
  if (t) *t = v;
  return MLS_OK;
}

int mls_plan_lower_level(const double* y, const int64_t* cap, const int32_t* pp, int32_t dp, int64_t L, int64_t n_mb,
                         double tau, int64_t* l, int64_t* m, double* step_time) {
  if (!y || !pp || !l || !m) return mls::set_error(MLS_E_NULL, "mls_plan_lower_level: null argument");
  if (dp < 1 || L < 1 || n_mb < 0 || !(tau > 0)) return mls::set_error(MLS_E_CONFIG, "mls_plan_lower_level: need dp >= 1, L >= 1, n_mb >= 0, tau > 0");
  int64_t stages = 0;
  for (int i = 0; i < dp; i++) {
    if (pp[i] < 1) return mls::set_error(MLS_E_CONFIG, "mls_plan_lower_level: every pipeline needs at least one stage");
    stages += pp[i];
  }
  if (!rates_ok(y, int(stages))) return mls::set_error(MLS_E_CONFIG, "mls_plan_lower_level: rates must be finite and > 0");
  std::vector<int64_t> lo(stages), mo(dp);
  std::vector<double> o(dp);
  int64_t at = 0;
  for (int i = 0; i < dp; i++) {  // Eq. 2, once per pipeline
    if (!minmax_split(y + at, cap ? cap + at : nullptr, pp[i], L, lo.data() + at, &o[i]))
      return mls::set_error(MLS_E_RANGE, "mls_plan_lower_level: a pipeline's stage capacities cannot hold L layers");
    at += pp[i];
  }
  double t = 0;
  minmax_split(o.data(), nullptr, dp, n_mb, mo.data(), &t);  // Eq. 3 (L >= 1, so every o[i] > 0)
  std::copy(lo.begin(), lo.end(), l);
  std::copy(mo.begin(), mo.end(), m);
  if (step_time) *step_time = t * tau;
  return MLS_OK;
}

int64_t mls_plan_layer_cap(double a_f, double a_fb, double s, double nu, int32_t pp, int32_t j, double capacity,
                           double reserve) {
  if (pp < 1 || j < 1 || j > pp || !(a_f >= 0) || !(a_fb >= 0) || !(s >= 0) || !(nu >= 0)) return -1;
  const double mu = a_f * double(pp - j) + a_fb + s;
  if (!(mu > 0) || !std::isfinite(mu)) return -1;
  const double room = capacity - reserve - nu;
  if (!(room > 0)) return 0;
  return int64_t(std::floor(room / mu));
}

int mls_plan_split_groups(const double* x, int32_t n, const int32_t* sizes, const double* rho, int32_t k,
                          int32_t* group_of, double* inv_sum) {
  if (!x || !sizes || !rho || !group_of) return mls::set_error(MLS_E_NULL, "mls_plan_split_groups: null argument");
  if (n < 1 || k < 1 || k > 8 || !rates_ok(x, n) || !rates_ok(rho, k))
    return mls::set_error(MLS_E_CONFIG, "mls_plan_split_groups: need n >= 1, 1 <= k <= 8 and finite rates > 0");
  int64_t total = 0;
  for (int g = 0; g < k; g++) {
    if (sizes[g] < 1) return mls::set_error(MLS_E_CONFIG, "mls_plan_split_groups: group sizes must be positive");
    total += sizes[g];
  }
  if (total != n) return mls::set_error(MLS_E_CONFIG, "mls_plan_split_groups: the group sizes must add up to n");
  // GPUs in descending order of their rates (stable: equal rates keep their index order)
  std::vector<int> by_rate(n);
  for (int i = 0; i < n; i++) by_rate[i] = i;
  std::stable_sort(by_rate.begin(), by_rate.end(), [&](int a, int b) { return x[a] > x[b]; });
  std::vector<int> order(k), best_order;
  for (int g = 0; g < k; g++) order[g] = g;
  double best = -1.0;
  do {  // order[p] = the group that takes the p-th run of the sorted list
    double sum = 0.0;
    int at = 0;
    for (int p = 0; p < k; p++) {
      const int g = order[p];
      sum += 1.0 / (rho[g] * x[by_rate[at]]);  // the run's first GPU has its largest rate
      at += sizes[g];
    }
    if (sum > best) {
      best = sum;
      best_order = order;
    }
  } while (std::next_permutation(order.begin(), order.end()));
  int at = 0;
  for (int p = 0; p < k; p++) {
    const int g = best_order[p];
    for (int i = 0; i < sizes[g]; i++) group_of[by_rate[at + i]] = g;
    at += sizes[g];
  }
  if (inv_sum) *inv_sum = best;
  return MLS_OK;
}

double mls_grouping_time_ratio(const double* y1, int32_t n1, const double* y2, int32_t n2) {
  if (!y1 || !y2 || n1 < 1 || n2 < 1 || !rates_ok(y1, n1) || !rates_ok(y2, n2)) return std::nan("");
  double s1 = 0, s2 = 0;
  for (int i = 0; i < n1; i++) s1 += 1.0 / y1[i];
  for (int i = 0; i < n2; i++) s2 += 1.0 / y2[i];
  return s2 / s1;
}

double mls_theoretic_slowdown(int64_t N, const double* x, int32_t n) {
  if (N < 1 || n < 0 || n > N || (n > 0 && (!x || !rates_ok(x, n)))) return std::nan("");
  double s = double(N - n);
  for (int i = 0; i < n; i++) s += 1.0 / x[i];
  return double(N) / s;
}

}  // extern "C"
