"""CPU checker for the batch-size controller.  TEST INFRASTRUCTURE ONLY (see
oracle/network.py): the product path never imports this.

The controller is a heuristic iteration, so this file follows the paper's
steps in the paper's order and notation (Section "Proportional-Control Based
Dynamic Policy", Eq. 4 and Eq. 5, and the four-step summary that closes the
subsection "Control stability"):

  1. smoothed iteration times mu_k (an EWMA over the iterations since the last
     readjustment; controller_step takes mu as `t`, DynamicBatcher keeps the state);
  2. error tau_k = t_k - tbar, throughput X_k = b_k / t_k,
     Delta(b_k) = -X_k tau_k, b_k' = b_k + Delta(b_k);
  3. bounds b_min <= b_k' <= b_max;
  4. dead-band: all workers are resized if max_k |Delta b_k| / b_k exceeds the
     threshold, otherwise nothing changes.

Where the paper is silent this file takes these readings:
  * tbar is the unweighted arithmetic mean, summed in worker order;
  * a scalar gain kp multiplies Delta (kp = 1 is the paper's rule);
  * the proportional rule does not conserve sum_k b_k, while the paper keeps
    the global batch fixed: after the bounds the real-valued sizes are
    rescaled to the global batch G, turned into integers by the
    largest-remainder method (ties to the lowest worker index), and entries
    that rescaling/rounding pushed outside the bounds are moved back one
    sample at a time (taking from the largest / giving to the smallest entry,
    ties to the lowest index);
  * the dead-band compares the final integer candidates with the old sizes,
    relative to the old size, in absolute value, strictly greater-than;
    a worker that had b_k = 0 and would receive samples always exceeds it.

All arithmetic is IEEE double, one rounding per operation, in exactly the
order written here (Python floats never fuse a multiply with an add).

Pins (tests/test_oracle_controller.py): the closed form b' = b tbar / t of the
paper, the sign rule, the throughput-proportional fixed point on synthetic
speed profiles, a hand-worked two-worker example, brute-force invariants on
all small integer inputs, and the dead-band/noise behaviour.  The rescaling
and integer rounding are this build's reading (parity unpinned by the paper;
pinned by sum(b_next) = G and the bounds).  DynamicBatcher is pinned by the
unrolled closed form of the EWMA, the equal-iteration-time goal state under an
affine time model, a hand-worked throughput-knee example, and the paper's
qualitative timelines (convergence within two readjustments; oscillation
without a dead-band under noisy times).
"""
from __future__ import annotations

import math


class ControllerError(ValueError):
    pass


def proportional_step(t, b, kp=1.0):
    """Eq. 4 and Eq. 5, real-valued: r_k = b_k + kp * (-X_k tau_k)."""
    K = len(b)
    s = 0.0
    for k in range(K):
        s = s + float(t[k])
    tbar = s / float(K)
    r = []
    for k in range(K):
        bk = float(b[k])
        tk = float(t[k])
        X = bk / tk
        tau = tk - tbar
        delta = -((kp * X) * tau)
        r.append(bk + delta)
    return r


def largest_remainder(q, total):
    """Integers f_k >= 0 with sum = total, f_k in {floor(q_k), floor(q_k)+1}."""
    K = len(q)
    f = [int(math.floor(v)) for v in q]
    frac = [q[k] - float(f[k]) for k in range(K)]
    rem = total - sum(f)
    taken = [False] * K
    while rem > 0:
        best = -1
        for k in range(K):
            if not taken[k] and (best < 0 or frac[k] > frac[best]):
                best = k
        if best < 0:                      # more than K left over: start another round
            taken = [False] * K
            continue
        f[best] += 1
        taken[best] = True
        rem -= 1
    while rem < 0:                        # cannot happen for sum(q) ~ total; kept for safety
        best = -1
        for k in range(K):
            if f[k] > 0 and (best < 0 or frac[k] < frac[best]):
                best = k
        f[best] -= 1
        frac[best] = 2.0
        rem += 1
    return f


def enforce_bounds_integer(c, total, b_min, b_max):
    """Move integer sizes back inside [b_min, b_max] while keeping their sum.
    b_max is one bound for all workers or a list with one bound per worker."""
    K = len(c)
    hi = list(b_max) if isinstance(b_max, (list, tuple)) else [b_max] * K
    c = [min(max(c[k], b_min), hi[k]) for k in range(K)]
    s = sum(c)
    while s > total:
        best = -1
        for k in range(K):
            if c[k] > b_min and (best < 0 or c[k] > c[best]):
                best = k
        c[best] -= 1
        s -= 1
    while s < total:
        best = -1
        for k in range(K):
            if c[k] < hi[k] and (best < 0 or c[k] < c[best]):
                best = k
        c[best] += 1
        s += 1
    return c


def controller_step(t, b, global_batch, kp=1.0, deadband=0.05, b_min=1, b_max=None,
                    b_hi=None, force=False, **_unused):
    """One controller invocation: (smoothed) times t[K], sizes b[K] -> new integer sizes.

    b_hi, if given, holds one upper bound per worker (each at most b_max; the learnt bounds
    of DynamicBatcher); force=True takes the candidate sizes whatever the dead-band says."""
    K = len(b)
    G = int(global_batch)
    if b_max is None:
        b_max = G
    if b_hi is not None:
        if len(b_hi) != K or any(int(h) < b_min or int(h) > b_max for h in b_hi) \
                or sum(int(h) for h in b_hi) < G:
            raise ControllerError("per-worker upper bounds cannot hold the global batch")
    if K < 1 or len(t) != K:
        raise ControllerError("K < 1 or length mismatch")
    if any(int(v) < 0 for v in b) or sum(int(v) for v in b) != G:
        raise ControllerError("b must be non-negative and sum to the global batch")
    if any((not math.isfinite(v)) or v <= 0.0 for v in t):
        raise ControllerError("iteration times must be finite and positive")
    if b_min < 0 or b_max < b_min or K * b_min > G or K * b_max < G:
        raise ControllerError("bounds cannot hold the global batch")
    if not (math.isfinite(kp) and math.isfinite(deadband)) or deadband < 0.0:
        raise ControllerError("bad gains")

    r = proportional_step(t, b, kp)                                   # step 2
    his = [int(b_max)] * K if b_hi is None else [int(h) for h in b_hi]
    lo = float(b_min)
    r = [lo if r[k] < lo else (float(his[k]) if r[k] > float(his[k]) else r[k])
         for k in range(K)]                                           # step 3
    S = 0.0
    for v in r:
        S = S + v
    if not (S > 0.0):
        return [int(v) for v in b]
    q = [(v * float(G)) / S for v in r]                               # keep sum_k b_k = G
    cand = largest_remainder(q, G)
    cand = enforce_bounds_integer(cand, G, int(b_min), his)

    worst = 0.0                                                       # step 4
    for k in range(K):
        d = abs(cand[k] - int(b[k]))
        if d == 0:
            continue
        rel = math.inf if int(b[k]) == 0 else float(d) / float(int(b[k]))
        if rel > worst:
            worst = rel
    if worst > deadband or force:
        return cand
    return [int(v) for v in b]


def ewma_update(mu, t, alpha, reset):
    """Step 1: mu_k <- t_k on the first iteration after a readjustment, else
    mu_k <- alpha t_k + (1 - alpha) mu_k."""
    if reset:
        return [float(v) for v in t]
    return [alpha * float(t[k]) + (1.0 - alpha) * float(mu[k]) for k in range(len(t))]


def static_allocation(X, b0):
    """Open-loop sizes proportional to the throughput estimates X_k with the
    global batch K*b0 kept (Section "Static Mini-batch Allocation Policy"; the
    printed formula lacks the factor K that its own invariant sum_k b_k = K b0
    requires).  Integers by the largest-remainder method."""
    K = len(X)
    G = K * int(b0)
    S = 0.0
    for v in X:
        S = S + float(v)
    q = [(float(v) * float(G)) / S for v in X]
    return largest_remainder(q, G)


def estimate_throughput(cpu_cores, half_precision_flops):
    """Throughput estimates X_k from the servers' resources (Section "Static Mini-batch
    Allocation Policy", paragraph "Estimating throughput"): the number of CPU cores when the
    workers use only CPUs (no worker states a FLOPs figure), the half-precision FLOPs of each
    server when CPU and GPU servers are mixed (every worker states one).  Only the ratios
    matter to static_allocation()."""
    flops = [float(v) for v in half_precision_flops]
    if all(v == 0.0 for v in flops):
        X = [float(c) for c in cpu_cores]
    elif all(v > 0.0 for v in flops):
        X = flops
    else:
        raise ValueError("either every worker or no worker states its half-precision FLOPs")
    if any(not (v > 0.0) or not math.isfinite(v) for v in X):
        raise ValueError("resources must be positive and finite")
    return X


class DynamicBatcher:
    """The controller with its state between iterations (subsection "Control stability"):
    the smoothed iteration times since the last readjustment, the current sizes, and the
    per-worker upper bounds learnt from the throughput curve.

    observe(t) takes the iteration times of the iteration that just ended and returns the
    sizes for the next one:

      1. mu_k <- EWMA of t_k over the iterations since the last readjustment (the first
         iteration after a readjustment restarts it: mu_k = t_k);
      2. learnt upper bound: a worker whose size was raised at the last readjustment, from
         b_old to its current size, and whose smoothed throughput b_k / mu_k is now below the
         throughput b_old / mu_old it had before, gets b_hi_k = b_old;
      3. Eq. 4 / Eq. 5 on mu, bounds [b_min, b_hi_k], dead-band (controller_step);
      4. after a readjustment the EWMA restarts and the sizes/throughputs it replaced are
         remembered for step 2.

    Readings where the paper is silent:
      * the throughput comparison of step 2 is made on every iteration, on smoothed times,
        with a relative tolerance drop_tolerance (0 = any drop counts); bounds only ever
        shrink; a bound that would leave sum_k b_hi_k below the global batch is not taken;
      * a current size above its (new) upper bound forces the readjustment, dead-band or not;
      * min_observations iterations must have been smoothed since the last readjustment
        before the next one is considered (1 = the paper's every-iteration check).
    """

    def __init__(self, b0, global_batch, kp=1.0, deadband=0.05, ewma_alpha=0.5, b_min=1,
                 b_max=None, drop_tolerance=0.0, min_observations=1, adaptive_b_max=True):
        self.K = len(b0)
        self.G = int(global_batch)
        self.kp, self.deadband, self.alpha = float(kp), float(deadband), float(ewma_alpha)
        self.b_min = int(b_min)
        self.b_max = self.G if b_max is None else int(b_max)
        self.drop_tolerance = float(drop_tolerance)
        self.min_observations = int(min_observations)
        self.adaptive = bool(adaptive_b_max)
        if sum(int(v) for v in b0) != self.G or any(int(v) < 0 for v in b0):
            raise ControllerError("b0 must be non-negative and sum to the global batch")
        if self.min_observations < 1 or not (0.0 <= self.alpha <= 1.0) \
                or not (self.drop_tolerance >= 0.0):
            raise ControllerError("bad controller constants")
        self.b = [int(v) for v in b0]
        self.mu = [0.0] * self.K
        self.b_hi = [self.b_max] * self.K
        self.observations = 0            # iterations smoothed since the last readjustment
        self.prev_b = None               # sizes replaced by the last readjustment
        self.prev_X = None               # smoothed throughputs at that moment
        self.readjustments = 0

    def observe(self, t):
        K = self.K
        if len(t) != K or any((not math.isfinite(v)) or v <= 0.0 for v in t):
            raise ControllerError("iteration times must be finite and positive")
        self.mu = ewma_update(self.mu, t, self.alpha, self.observations == 0)     # step 1
        self.observations += 1

        force = False
        if self.adaptive and self.prev_b is not None:                             # step 2
            for k in range(K):
                if self.b[k] > self.prev_b[k] and self.prev_b[k] > 0:
                    X_now = float(self.b[k]) / self.mu[k]
                    if X_now < self.prev_X[k] * (1.0 - self.drop_tolerance):
                        new_hi = max(self.prev_b[k], self.b_min)
                        if new_hi < self.b_hi[k] and \
                                sum(self.b_hi) - self.b_hi[k] + new_hi >= self.G:
                            self.b_hi[k] = new_hi
        for k in range(K):
            if self.b[k] > self.b_hi[k]:
                force = True

        if self.observations < self.min_observations and not force:
            return list(self.b)
        cand = controller_step(self.mu, self.b, self.G, kp=self.kp, deadband=self.deadband,
                               b_min=self.b_min, b_max=self.b_max, b_hi=self.b_hi,
                               force=force)                                       # step 3
        if cand != self.b:                                                        # step 4
            self.prev_b = list(self.b)
            self.prev_X = [float(self.b[k]) / self.mu[k] for k in range(K)]
            self.b = cand
            self.observations = 0
            self.readjustments += 1
        return list(self.b)
