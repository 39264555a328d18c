// Host-side batch-size controller: the proportional rule of Eq. 4 / Eq. 5 with the
// stability measures of "Control stability" (bounds, dead-band), as a stateless step (the
// caller keeps the EWMA) and as an object that keeps the smoothed times, the sizes and the
// upper bounds learnt from observed throughput drops between iterations.  Compiled with
// floating-point contraction off so that every operation rounds once, in the order written.
#include <cmath>
#include <cstdint>
#include <new>
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
void restore_bounds(std::vector<int64_t>& c, int64_t total, int64_t lo, const int64_t* hi) {
  const int K = (int)c.size();
  int64_t sum = 0;
  for (int k = 0; k < K; ++k) {
    if (c[k] < lo) c[k] = lo;
    if (c[k] > hi[k]) c[k] = hi[k];
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
      if (c[k] < hi[k] && (pick < 0 || c[k] < c[pick])) pick = k;
    c[pick] += 1;
    ++sum;
  }
}

// Arguments common to the stateless call and the stateful object.
int check_step_args(const double* t, const int32_t* b, int K, int64_t G, const dynb_gains& gains) {
  if (K < 1 || K > DYNB_MAX_WORKERS) return dynb::fail(DYNB_ERR_BADARG, "controller: K out of range");
  int64_t sum_b = 0;
  for (int k = 0; k < K; ++k) {
    if (b[k] < 0) return dynb::fail(DYNB_ERR_BADARG, "controller: negative batch size");
    sum_b += b[k];
    if (t && (!std::isfinite(t[k]) || !(t[k] > 0.0)))
      return dynb::fail(DYNB_ERR_BADARG, "controller: iteration time not finite and positive");
  }
  if (sum_b != G) return dynb::fail(DYNB_ERR_BADARG, "controller: sum(b) != global_batch");
  const int64_t lo = gains.b_min, hi = gains.b_max;
  if (lo < 0 || hi < lo || (int64_t)K * lo > G || (int64_t)K * hi < G)
    return dynb::fail(DYNB_ERR_BADARG, "controller: bounds cannot hold the global batch");
  if (!std::isfinite(gains.kp) || !std::isfinite(gains.deadband) || gains.deadband < 0.0)
    return dynb::fail(DYNB_ERR_BADARG, "controller: bad gains");
  return DYNB_OK;
}

// Steps 2-4 of the summary in "Control stability" on validated input.  hi[k] is worker k's
// upper bound; `force` takes the candidate sizes whatever the dead-band says.
void step_core(const double* t, const int32_t* b, int K, int64_t G, double kp, double band,
               int64_t lo, const int64_t* hi, bool force, int32_t* b_next) {
  // tbar: plain mean in worker order
  double tsum = 0.0;
  for (int k = 0; k < K; ++k) tsum = tsum + t[k];
  const double tbar = tsum / (double)K;

  // Eq. 4 / Eq. 5 with gain kp, then the bounds
  std::vector<double> r(K);
  const double flo = (double)lo;
  double S = 0.0;
  for (int k = 0; k < K; ++k) {
    const double bk = (double)b[k];
    const double X = bk / t[k];
    const double tau = t[k] - tbar;
    const double delta = -((kp * X) * tau);
    double v = bk + delta;
    const double fhi = (double)hi[k];
    if (v < flo) v = flo;
    else if (v > fhi) v = fhi;
    r[k] = v;
  }
  for (int k = 0; k < K; ++k) S = S + r[k];
  if (!(S > 0.0)) {
    for (int k = 0; k < K; ++k) b_next[k] = b[k];
    return;
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
  const bool resize = force || worst > band;
  for (int k = 0; k < K; ++k) b_next[k] = resize ? (int32_t)cand[k] : b[k];
}

}  // namespace

extern "C" int dynb_controller_step(const double* t, const int32_t* b, int32_t K,
                                    int32_t global_batch, const dynb_gains* gains,
                                    int32_t* b_next) {
  if (!t || !b || !gains || !b_next) return dynb::fail(DYNB_ERR_BADARG, "controller: null pointer");
  if (int rc = check_step_args(t, b, K, global_batch, *gains)) return rc;
  int64_t hi[DYNB_MAX_WORKERS];
  for (int k = 0; k < K; ++k) hi[k] = gains->b_max;
  step_core(t, b, K, global_batch, gains->kp, gains->deadband, gains->b_min, hi, false, b_next);
  return DYNB_OK;
}

// ---- the controller with its state between iterations ("Control stability") ----------------
struct dynb_controller {
  int K;
  int64_t G;
  dynb_controller_config cfg;
  int32_t b[DYNB_MAX_WORKERS];
  double mu[DYNB_MAX_WORKERS];
  int64_t hi[DYNB_MAX_WORKERS];      // learnt upper bounds, start at gains.b_max
  int32_t since;                     // iterations smoothed since the last readjustment
  bool have_prev;                    // a readjustment has happened
  int32_t prev_b[DYNB_MAX_WORKERS];  // the sizes it replaced
  double prev_X[DYNB_MAX_WORKERS];   // and the smoothed throughputs at that moment
  int32_t readjustments;
};

extern "C" int dynb_controller_create(const dynb_controller_config* cfg, const int32_t* b0,
                                      int32_t K, int32_t global_batch, dynb_controller** out) {
  if (!cfg || !b0 || !out) return dynb::fail(DYNB_ERR_BADARG, "controller: null pointer");
  if (int rc = check_step_args(nullptr, b0, K, global_batch, cfg->gains)) return rc;
  const double a = cfg->gains.ewma_alpha;
  if (!(a >= 0.0 && a <= 1.0) || !(cfg->drop_tolerance >= 0.0) || !std::isfinite(cfg->drop_tolerance) ||
      cfg->min_observations < 1)
    return dynb::fail(DYNB_ERR_BADARG, "controller: bad smoothing constant, tolerance or min_observations");
  dynb_controller* c = new (std::nothrow) dynb_controller();
  if (!c) return dynb::fail(DYNB_ERR_STATE, "controller: out of host memory");
  c->K = K;
  c->G = global_batch;
  c->cfg = *cfg;
  for (int k = 0; k < K; ++k) {
    c->b[k] = b0[k];
    c->mu[k] = 0.0;
    c->hi[k] = cfg->gains.b_max;
  }
  c->since = 0;
  c->have_prev = false;
  c->readjustments = 0;
  *out = c;
  return DYNB_OK;
}

extern "C" void dynb_controller_destroy(dynb_controller* c) { delete c; }

extern "C" int dynb_controller_observe(dynb_controller* c, const double* t, int32_t* b_next,
                                       int32_t* resized) {
  if (!c || !t || !b_next) return dynb::fail(DYNB_ERR_BADARG, "controller: null pointer");
  const int K = c->K;
  for (int k = 0; k < K; ++k)
    if (!std::isfinite(t[k]) || !(t[k] > 0.0))
      return dynb::fail(DYNB_ERR_BADARG, "controller: iteration time not finite and positive");

  // 1. smoothed times over the iterations since the last readjustment
  const double a = c->cfg.gains.ewma_alpha;
  for (int k = 0; k < K; ++k)
    c->mu[k] = c->since == 0 ? t[k] : a * t[k] + (1.0 - a) * c->mu[k];
  c->since += 1;

  // 2. a worker that was given more samples and got slower per sample for it keeps the
  //    size it had before as its upper bound
  if (c->cfg.adaptive_b_max && c->have_prev) {
    for (int k = 0; k < K; ++k) {
      if (c->b[k] <= c->prev_b[k] || c->prev_b[k] <= 0) continue;
      const double X_now = (double)c->b[k] / c->mu[k];
      if (!(X_now < c->prev_X[k] * (1.0 - c->cfg.drop_tolerance))) continue;
      int64_t cap = c->prev_b[k];
      if (cap < c->cfg.gains.b_min) cap = c->cfg.gains.b_min;
      int64_t room = cap;
      for (int j = 0; j < K; ++j)
        if (j != k) room += c->hi[j];
      if (cap < c->hi[k] && room >= c->G) c->hi[k] = cap;
    }
  }
  bool force = false;
  for (int k = 0; k < K; ++k) force = force || c->b[k] > c->hi[k];

  bool changed = false;
  if (c->since >= c->cfg.min_observations || force) {
    // 3. proportional rule on the smoothed times, bounds, dead-band
    int32_t cand[DYNB_MAX_WORKERS];
    step_core(c->mu, c->b, K, c->G, c->cfg.gains.kp, c->cfg.gains.deadband, c->cfg.gains.b_min,
              c->hi, force, cand);
    for (int k = 0; k < K; ++k) changed = changed || cand[k] != c->b[k];
    if (changed) {
      // 4. remember what is being replaced; the smoothing restarts
      for (int k = 0; k < K; ++k) {
        c->prev_b[k] = c->b[k];
        c->prev_X[k] = (double)c->b[k] / c->mu[k];
        c->b[k] = cand[k];
      }
      c->have_prev = true;
      c->since = 0;
      c->readjustments += 1;
    }
  }
  for (int k = 0; k < K; ++k) b_next[k] = c->b[k];
  if (resized) *resized = changed ? 1 : 0;
  return DYNB_OK;
}

extern "C" int dynb_controller_read(const dynb_controller* c, int32_t* b, double* mu,
                                    int32_t* b_hi, int32_t* observations,
                                    int32_t* readjustments) {
  if (!c) return dynb::fail(DYNB_ERR_BADARG, "controller: null pointer");
  for (int k = 0; k < c->K; ++k) {
    if (b) b[k] = c->b[k];
    if (mu) mu[k] = c->mu[k];
    if (b_hi) b_hi[k] = (int32_t)c->hi[k];
  }
  if (observations) *observations = c->since;
  if (readjustments) *readjustments = c->readjustments;
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

extern "C" int dynb_estimate_throughput(const dynb_worker_resources* r, int32_t K, double* X_out) {
  if (!r || !X_out) return dynb::fail(DYNB_ERR_BADARG, "estimate_throughput: null pointer");
  if (K < 1 || K > DYNB_MAX_WORKERS) return dynb::fail(DYNB_ERR_BADARG, "estimate_throughput: bad K");
  int with_flops = 0;
  for (int k = 0; k < K; ++k) {
    if (!std::isfinite(r[k].half_precision_flops) || r[k].half_precision_flops < 0.0)
      return dynb::fail(DYNB_ERR_BADARG, "estimate_throughput: FLOPs of worker %d not finite or negative", k);
    if (r[k].half_precision_flops > 0.0) ++with_flops;
  }
  if (with_flops != 0 && with_flops != K)
    return dynb::fail(DYNB_ERR_BADARG,
                      "estimate_throughput: either every worker or no worker states its FLOPs");
  for (int k = 0; k < K; ++k) {
    if (with_flops == 0 && r[k].cpu_cores < 1)
      return dynb::fail(DYNB_ERR_BADARG, "estimate_throughput: worker %d has no CPU cores", k);
    X_out[k] = with_flops ? r[k].half_precision_flops : (double)r[k].cpu_cores;
  }
  return DYNB_OK;
}

extern "C" int dynb_lr_schedule(int64_t step, const int64_t* boundaries, const double* values,
                                int32_t n_values, double* lr) {
  if (!values || !lr || (n_values > 1 && !boundaries))
    return dynb::fail(DYNB_ERR_BADARG, "lr_schedule: null pointer");
  if (n_values < 1) return dynb::fail(DYNB_ERR_BADARG, "lr_schedule: no values");
  for (int i = 1; i + 1 < n_values; ++i)
    if (boundaries[i] < boundaries[i - 1])
      return dynb::fail(DYNB_ERR_BADARG, "lr_schedule: boundaries must not decrease");
  int i = 0;
  while (i < n_values - 1 && step >= boundaries[i]) ++i;
  *lr = values[i];
  return DYNB_OK;
}
