// Host-side batch-size controller: the proportional rule of Eq. 4 / Eq. 5 with the
// stability measures of "Control stability" (bounds, dead-band; the EWMA state is
// kept by the caller).  Compiled with floating-point contraction off so that every
// operation rounds once, in the order written.
#include <cmath>
#include <cstdint>
#include <vector>

#include "dynb_internal.h"

namespace {

// Integers in {floor(q_k), floor(q_k)+1} that sum to `total`; the units left over after
// flooring go to the largest fractional parts, lowest index first among equals.
void hamilton_round(const std::vector<double>& q, int64_t total, std::vector<int64_t>& f) {
  const int K = (int)q.size();
  f.resize(K);
  std::vector<double> frac(K);
  int64_t sum = 0;
  for (int k = 0; k < K; ++k) {
    double fl = std::floor(q[k]);
    f[k] = (int64_t)fl;
    frac[k] = q[k] - fl;
    sum += f[k];
  }
  int64_t rem = total - sum;
  std::vector<char> used(K, 0);
  while (rem > 0) {
    int pick = -1;
    for (int k = 0; k < K; ++k)
      if (!used[k] && (pick < 0 || frac[k] > frac[pick])) pick = k;
    if (pick < 0) {  // every worker already got one: go round again
      used.assign(K, 0);
      continue;
    }
    f[pick] += 1;
    used[pick] = 1;
    --rem;
  }
  while (rem < 0) {  // unreachable when sum(q) ~ total; mirrors the rule above
    int pick = -1;
    for (int k = 0; k < K; ++k)
      if (f[k] > 0 && (pick < 0 || frac[k] < frac[pick])) pick = k;
    f[pick] -= 1;
    frac[pick] = 2.0;
    ++rem;
  }
}

// Clamp to [lo, hi], then restore the sum one sample at a time: surplus is taken from the
// largest entry, a deficit is given to the smallest entry (lowest index among equals).
void restore_bounds(std::vector<int64_t>& c, int64_t total, int64_t lo, int64_t hi) {
  const int K = (int)c.size();
  int64_t sum = 0;
  for (int k = 0; k < K; ++k) {
    if (c[k] < lo) c[k] = lo;
    if (c[k] > hi) c[k] = hi;
    sum += c[k];
  }
  while (sum > total) {
    int pick = -1;
    for (int k = 0; k < K; ++k)
      if (c[k] > lo && (pick < 0 || c[k] > c[pick])) pick = k;
    c[pick] -= 1;
    --sum;
  }
  while (sum < total) {
    int pick = -1;
    for (int k = 0; k < K; ++k)
      if (c[k] < hi && (pick < 0 || c[k] < c[pick])) pick = k;
    c[pick] += 1;
    ++sum;
  }
}

}  // namespace

extern "C" int dynb_controller_step(const double* t, const int32_t* b, int32_t K,
                                    int32_t global_batch, const dynb_gains* gains,
                                    int32_t* b_next) {
  if (!t || !b || !gains || !b_next) return dynb::fail(DYNB_ERR_BADARG, "controller: null pointer");
  if (K < 1 || K > DYNB_MAX_WORKERS) return dynb::fail(DYNB_ERR_BADARG, "controller: K out of range");
  const int64_t G = global_batch;
  int64_t sum_b = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return dynb::fail(DYNB_ERR_BADARG, "controller: negative batch size");
    sum_b += b[k];
    if (!std::isfinite(t[k]) || !(t[k] > 0.0))
      return dynb::fail(DYNB_ERR_BADARG, "controller: iteration time not finite and positive");
  }
  if (sum_b != G) return dynb::fail(DYNB_ERR_BADARG, "controller: sum(b) != global_batch");
  const int64_t lo = gains->b_min, hi = gains->b_max;
  if (lo < 0 || hi < lo || (int64_t)K * lo > G || (int64_t)K * hi < G)
    return dynb::fail(DYNB_ERR_BADARG, "controller: bounds cannot hold the global batch");
  const double kp = gains->kp, band = gains->deadband;
  if (!std::isfinite(kp) || !std::isfinite(band) || band < 0.0)
    return dynb::fail(DYNB_ERR_BADARG, "controller: bad gains");

  // tbar: plain mean in worker order
  double tsum = 0.0;
  for (int k = 0; k < K; ++k) tsum = tsum + t[k];
  const double tbar = tsum / (double)K;

  // Eq. 4 / Eq. 5 with gain kp, then the bounds
  std::vector<double> r(K);
  const double flo = (double)lo, fhi = (double)hi;
  double S = 0.0;
  for (int k = 0; k < K; ++k) {
    const double bk = (double)b[k];
    const double X = bk / t[k];
    const double tau = t[k] - tbar;
    const double delta = -((kp * X) * tau);
    double v = bk + delta;
    if (v < flo) v = flo;
    else if (v > fhi) v = fhi;
    r[k] = v;
  }
  for (int k = 0; k < K; ++k) S = S + r[k];
  if (!(S > 0.0)) {
    for (int k = 0; k < K; ++k) b_next[k] = b[k];
    return DYNB_OK;
  }

  // keep the global batch: rescale, integerise, re-impose the bounds
  std::vector<double> q(K);
  for (int k = 0; k < K; ++k) q[k] = (r[k] * (double)G) / S;
  std::vector<int64_t> cand;
  hamilton_round(q, G, cand);
  restore_bounds(cand, G, lo, hi);

  // dead-band on the integer candidates, relative to the old sizes
  double worst = 0.0;
  for (int k = 0; k < K; ++k) {
    int64_t d = cand[k] - (int64_t)b[k];
    if (d < 0) d = -d;
    if (d == 0) continue;
    const double rel = (b[k] == 0) ? INFINITY : (double)d / (double)b[k];
    if (rel > worst) worst = rel;
  }
  const bool resize = worst > band;
  for (int k = 0; k < K; ++k) b_next[k] = resize ? (int32_t)cand[k] : b[k];
  return DYNB_OK;
}

extern "C" int dynb_ewma_update(double* mu, const double* t, int32_t K, double alpha,
                                int32_t reset) {
  if (!mu || !t) return dynb::fail(DYNB_ERR_BADARG, "ewma: null pointer");
  if (K < 1 || K > DYNB_MAX_WORKERS) return dynb::fail(DYNB_ERR_BADARG, "ewma: K out of range");
  if (!(alpha >= 0.0 && alpha <= 1.0)) return dynb::fail(DYNB_ERR_BADARG, "ewma: alpha not in [0,1]");
  for (int k = 0; k < K; ++k) {
    if (reset) mu[k] = t[k];
    else mu[k] = alpha * t[k] + (1.0 - alpha) * mu[k];
  }
  return DYNB_OK;
}

extern "C" int dynb_static_allocate(const double* X, int32_t K, int32_t b0, int32_t* b_out) {
  if (!X || !b_out) return dynb::fail(DYNB_ERR_BADARG, "static: null pointer");
  if (K < 1 || K > DYNB_MAX_WORKERS || b0 < 0) return dynb::fail(DYNB_ERR_BADARG, "static: bad K or b0");
  double S = 0.0;
  for (int k = 0; k < K; ++k) {
    if (!std::isfinite(X[k]) || !(X[k] > 0.0))
      return dynb::fail(DYNB_ERR_BADARG, "static: throughput not finite and positive");
    S = S + X[k];
  }
  const int64_t G = (int64_t)K * b0;
  std::vector<double> q(K);
  for (int k = 0; k < K; ++k) q[k] = (X[k] * (double)G) / S;
  std::vector<int64_t> f;
  hamilton_round(q, G, f);
  for (int k = 0; k < K; ++k) b_out[k] = (int32_t)f[k];
  return DYNB_OK;
}
