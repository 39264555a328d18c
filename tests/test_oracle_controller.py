"""Pins for oracle/controller.py against the paper's statements and brute force."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import controller as oc
from paper_2305_12213_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_rows(name):
    rows = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([f.split() for f in line.split(";")])
    return rows


def test_hand_worked_examples():
    for G, kp, db, b, s, want in read_rows("controller_worked_examples.txt"):
        b = [int(v) for v in b]; s = [float(v) for v in s]
        t = synth.iteration_times(b, s)
        got = oc.controller_step(t, b, int(G[0]), kp=float(kp[0]), deadband=float(db[0]),
                                 b_min=1, b_max=int(G[0]))
        assert got == [int(v) for v in want], (b, s, got)


def test_static_allocation_reproduces_the_papers_gpu_cpu_ratio():
    for X, b0, want in read_rows("static_allocation_example.txt"):
        got = oc.static_allocation([float(v) for v in X], int(b0[0]))
        assert got == [int(v) for v in want]
        if len(got) == 2:
            assert abs(got[0] / got[1] - 4.3) < 0.1      # "only 4.3x faster"


def test_throughput_estimates_from_cores_or_half_precision_flops():
    # CPU-only workers: core counts (the paper's three workers with 3, 5 and 12 cores)
    X = oc.estimate_throughput([3, 5, 12], [0, 0, 0])
    assert X == [3.0, 5.0, 12.0]
    assert oc.static_allocation(X, 100) == [45, 75, 180]
    # mixed CPU / GPU servers: half-precision FLOPs, whatever the core counts say; the paper's
    # GPU : CPU FLOPs ratio 0.813 : 0.187 gives its batch-size ratio
    X = oc.estimate_throughput([8, 48], [0.813e14, 0.187e14])
    assert oc.static_allocation(X, 500) == [813, 187]
    with pytest.raises(ValueError):
        oc.estimate_throughput([8, 48], [1e14, 0])          # stated for some workers only
    with pytest.raises(ValueError):
        oc.estimate_throughput([8, 0], [0, 0])


def test_raw_step_equals_closed_form_b_tbar_over_t():
    rng = np.random.default_rng(0)
    for _ in range(200):
        K = int(rng.integers(1, 9))
        b = rng.integers(1, 500, K)
        t = rng.uniform(0.1, 50.0, K)
        r = oc.proportional_step(list(t), list(b), 1.0)
        tbar = t.mean()
        np.testing.assert_allclose(r, b * tbar / t, rtol=1e-12)


def test_sign_rule_slower_than_average_shrinks_faster_grows():
    r = oc.proportional_step([1.0, 2.0, 3.0], [10, 10, 10], 1.0)
    assert r[0] > 10 and abs(r[1] - 10) < 1e-12 and r[2] < 10


def test_gain_scales_the_correction_linearly():
    t, b = [3.0, 5.0, 11.0], [20, 30, 40]
    r1 = oc.proportional_step(t, b, 1.0); rh = oc.proportional_step(t, b, 0.5)
    for k in range(3):
        assert abs((rh[k] - b[k]) - 0.5 * (r1[k] - b[k])) < 1e-12


def proportional_target(G, s):
    q = np.array(s) * G / np.sum(s)
    return q


@pytest.mark.parametrize("G,s", [(64, [1.0, 0.5]), (256, [1, 1, 0.5, 0.25]),
                                 (512, [1, 0.4, 0.2, 0.08]),
                                 (4096, [0.004 ** (k / 15) for k in range(16)]),
                                 (1024, [1, .25, .5, .5, 1, .25, 1, .5])])
def test_fixed_point_is_throughput_proportional_and_reached_in_one_adjustment(G, s):
    K = len(s)
    target = proportional_target(G, s)
    for start in ([G // K] * K, [v + 1 for v in synth.ragged_split(G - K, K, 5)]):
        b = list(start)
        assert sum(b) == G
        t = synth.iteration_times(b, s)
        # "no active bounds": a far-off start can push the raw step past b_max = G
        b1 = oc.controller_step(t, b, G, kp=1.0, deadband=0.0, b_min=1, b_max=10 ** 9)
        assert sum(b1) == G
        assert np.all(np.abs(np.array(b1) - target) < 1.0)        # proportional up to rounding
        # iteration times are now equal up to one sample's worth of work
        b2 = oc.controller_step(synth.iteration_times(b1, s), b1, G, kp=1.0, deadband=0.05,
                                b_min=1, b_max=G)
        big = [k for k in range(K) if b1[k] >= 40]               # small b_k: rounding > 5 %
        assert all(b2[k] == b1[k] for k in big) or b2 == b1
        # the paper: converged "after only two batch adjustments"
        b3 = oc.controller_step(synth.iteration_times(b2, s), b2, G, kp=1.0, deadband=0.05,
                                b_min=1, b_max=G)
        assert np.all(np.abs(np.array(b3) - target) < 1.5)


def test_half_gain_halves_the_distance_each_call():
    s, G = [1.0, 1.0, 0.5, 0.25], 25600
    target = proportional_target(G, s)
    b = [G // 4] * 4
    prev = np.abs(np.array(b) - target).max()
    for _ in range(6):
        b = oc.controller_step(synth.iteration_times(b, s), b, G, kp=0.5, deadband=0.0,
                               b_min=1, b_max=G)
        cur = np.abs(np.array(b) - target).max()
        assert cur < 0.75 * prev + 2
        prev = cur
    assert prev < 0.05 * G / 4


def test_brute_force_invariants_on_all_small_inputs():
    speeds = [[1.0, 0.5, 0.25], [1.0, 1.0, 1.0], [0.3, 1.0, 0.05]]
    for G in range(3, 13):
        for b in itertools.product(range(0, G + 1), repeat=3):
            if sum(b) != G:
                continue
            for s in speeds:
                t = synth.iteration_times(b, s)
                for lo, hi in ((0, G), (1, G), (1, max(G // 2, (G + 2) // 3)), (2, G)):
                    if 3 * lo > G or 3 * hi < G:
                        continue
                    for db in (0.0, 0.05):
                        out = oc.controller_step(t, list(b), G, kp=1.0, deadband=db,
                                                 b_min=lo, b_max=hi)
                        assert sum(out) == G
                        if out != list(b):
                            assert all(lo <= v <= hi for v in out), (b, s, lo, hi, out)


def test_bounds_are_enforced_under_extreme_heterogeneity():
    s = [1.0, 1e-6, 1e-6, 1e-6]
    b = [64] * 4
    out = oc.controller_step(synth.iteration_times(b, s), b, 256, kp=1.0, deadband=0.0,
                             b_min=8, b_max=200)
    assert sum(out) == 256 and min(out) >= 8 and max(out) <= 200
    # r = (4.8e7 -> 200, 48, 48, 48), sum 344, rescaled to 256: (148.84, 35.72, 35.72, 35.72)
    assert out == [149, 36, 36, 35]
    # r = (15, 184.5), sum 199.5, rescaled: (19.25, 236.75) -> (19, 237): above b_max = 200,
    # so 37 samples move to the smallest entry
    out = oc.controller_step([1.0, 2.0], [10, 246], 256, deadband=0.0, b_min=8, b_max=200)
    assert out == [56, 200]


def test_deadband_stops_noise_chasing_and_zero_deadband_does_not():
    s, G = [1.0, 0.4, 0.2, 0.08], 5120
    rng = np.random.default_rng(42)
    for db, expect_quiet in ((0.05, True), (0.0, False)):
        b = [G // 4] * 4
        for _ in range(2):        # b_max = G clips the first raw step: two adjustments converge
            b = oc.controller_step(synth.iteration_times(b, s), b, G, deadband=0.0)
        assert np.all(np.abs(np.array(b) - proportional_target(G, s)) < 1.0)
        changes = 0
        for _ in range(50):
            t = [v * (1.0 + 0.02 * (2 * rng.random() - 1)) for v in synth.iteration_times(b, s)]
            nb = oc.controller_step(t, b, G, kp=1.0, deadband=db, b_min=1, b_max=G)
            changes += nb != b
            b = nb
        assert (changes == 0) if expect_quiet else (changes > 25)


def test_speed_change_mid_run_is_tracked():
    G = 1200
    s = [1.0, 1.0, 1.0]
    b = [400, 400, 400]
    assert oc.controller_step(synth.iteration_times(b, s), b, G) == b
    s = [1.0, 0.25, 1.0]                                   # worker 1 slows down 4x
    b = oc.controller_step(synth.iteration_times(b, s), b, G)
    assert np.all(np.abs(np.array(b) - proportional_target(G, s)) < 1.0)
    s = [1.0, 1e-9, 1.0]                                   # ... and then stalls
    # tbar is dominated by the stalled worker, so b_1' = b_1 tbar / t_1 ~ b_1 / K per call:
    # its share falls geometrically until the lower bound holds it
    seen = [b[1]]
    for _ in range(6):
        b = oc.controller_step(synth.iteration_times(b, s), b, G, b_min=4)
        assert sum(b) == G and b[1] <= seen[-1]
        seen.append(b[1])
    assert b[1] == 4 and b[0] == b[2] == 598


def test_idle_worker_and_errors():
    out = oc.controller_step([1.0, 1.0], [10, 0], 10, deadband=0.0, b_min=0)
    assert out == [10, 0]                                  # zero throughput stays at zero
    out = oc.controller_step([1.0, 1.0], [10, 0], 10, deadband=0.0, b_min=1)
    assert out == [9, 1]
    for bad in (dict(t=[1.0, -1.0], b=[5, 5], G=10), dict(t=[1.0, math.nan], b=[5, 5], G=10),
                dict(t=[1.0, 1.0], b=[5, 4], G=10), dict(t=[1.0, 1.0], b=[11, -1], G=10),
                dict(t=[1.0], b=[5, 5], G=10)):
        with pytest.raises(oc.ControllerError):
            oc.controller_step(bad["t"], bad["b"], bad["G"])
    with pytest.raises(oc.ControllerError):
        oc.controller_step([1.0, 1.0], [5, 5], 10, b_min=6)
    with pytest.raises(oc.ControllerError):
        oc.controller_step([1.0, 1.0], [5, 5], 10, b_max=4)


def test_largest_remainder_properties():
    rng = np.random.default_rng(7)
    for _ in range(300):
        K = int(rng.integers(1, 10)); G = int(rng.integers(K, 500))
        w = rng.random(K) + 1e-3
        q = list(w * G / w.sum())
        f = oc.largest_remainder(q, G)
        assert sum(f) == G
        assert all(math.floor(q[k]) <= f[k] <= math.floor(q[k]) + 1 for k in range(K))
    assert oc.largest_remainder([1.5, 1.5, 1.0], 4) == [2, 1, 1]     # tie -> lowest index


def test_ewma_closed_form():
    mu = oc.ewma_update(None, [4.0, 8.0], 0.5, reset=True)
    assert mu == [4.0, 8.0]
    mu = oc.ewma_update(mu, [8.0, 8.0], 0.25, reset=False)
    assert mu == [5.0, 8.0]
    # constant input is a fixed point; a unit step decays as (1 - alpha)^n
    mu = [0.0]
    for n in range(1, 6):
        mu = oc.ewma_update(mu, [1.0], 0.3, reset=False)
        assert abs(mu[0] - (1 - 0.7 ** n)) < 1e-12


# ---------------------------------------------------------------------------------------------
# DynamicBatcher: the controller with its state (subsection "Control stability")
# ---------------------------------------------------------------------------------------------
def test_ewma_since_last_readjustment_matches_unrolled_sum():
    # mu after n iterations without readjustment = alpha * sum_i (1-alpha)^i t_{n-i} + (1-alpha)^(n-1) t_1
    rng = np.random.default_rng(5)
    alpha = 0.3
    d = oc.DynamicBatcher([40, 40, 40], 120, ewma_alpha=alpha, deadband=10.0)   # never resizes
    ts = rng.uniform(1.0, 2.0, size=(7, 3))
    for n in range(1, 8):
        d.observe(list(ts[n - 1]))
        want = (1 - alpha) ** (n - 1) * ts[0]
        for i in range(1, n):
            want = want + alpha * (1 - alpha) ** (n - 1 - i) * ts[i]
        np.testing.assert_allclose(d.mu, want, rtol=1e-13)
    assert d.readjustments == 0 and d.observations == 7


def test_ewma_restarts_after_a_readjustment():
    d = oc.DynamicBatcher([50, 50], 100, ewma_alpha=0.25)
    d.observe([10.0, 30.0])                      # large error: resizes
    assert d.readjustments == 1 and d.observations == 0
    d.observe([7.0, 9.0])
    assert d.mu == [7.0, 9.0]                    # first iteration after the readjustment: no memory
    d2 = oc.DynamicBatcher([50, 50], 100, ewma_alpha=0.25, deadband=10.0)
    d2.observe([10.0, 30.0]); d2.observe([7.0, 9.0])
    assert d2.mu == [0.25 * 7.0 + 0.75 * 10.0, 0.25 * 9.0 + 0.75 * 30.0]


def test_goal_state_equal_iteration_times_under_affine_time_model():
    # with t_k = c_k + b_k/s_k the goal t_i = t_j has the solution b_k = s_k (T - c_k) with
    # sum_k b_k = G; the controller must settle there (dead-band 0: within rounding)
    s = [1.0, 2.0, 5.0, 8.0]; c = [3.0, 1.0, 2.0, 0.5]; G = 4000
    T = (G + sum(sk * ck for sk, ck in zip(s, c))) / sum(s)
    want = [sk * (T - ck) for sk, ck in zip(s, c)]
    d = oc.DynamicBatcher([G // 4] * 4, G, ewma_alpha=1.0, deadband=0.0)
    b = list(d.b)
    for it in range(40):
        b = d.observe(synth.plant_times(b, s, overhead=c))
    assert sum(b) == G
    assert max(abs(bk - wk) for bk, wk in zip(b, want)) <= 2.0, (b, want)
    t = synth.plant_times(b, s, overhead=c)
    assert (max(t) - min(t)) / min(t) < 5e-3


def test_timeline_converges_within_two_readjustments_with_deadband():
    # Fig. "Batch sizes quickly converge within two adjustments": three workers, equal start,
    # a fixed overhead makes the proportional rule inexact, so the first step lands near the
    # goal and the second finishes; the dead-band then holds the sizes.
    s = [3.0, 9.0, 18.0]; c = [0.4, 0.4, 0.4]; G = 300
    d = oc.DynamicBatcher([100, 100, 100], G, ewma_alpha=0.5, deadband=0.05)
    b = list(d.b); history = []
    for it in range(30):
        b = d.observe(synth.plant_times(b, s, overhead=c))
        history.append(list(b))
    assert 1 <= d.readjustments <= 2
    assert history[2:] == [history[2]] * 28                 # flat after the second iteration
    t = synth.plant_times(b, s, overhead=c)
    assert (max(t) - min(t)) / (sum(t) / 3) < 0.10          # inside the dead-band's resolution


def test_timeline_oscillates_without_deadband_under_noise():
    # Fig. "Oscillations in mini-batch sizes without dead-banding": the same loop chases the
    # noise forever with a zero dead-band and stops after the start-up with the paper's 0.05.
    s = [3.0, 5.0, 12.0]; G = 600
    def run(deadband, alpha):
        # (the learnt upper bounds are off: with zero tolerance they would read the noise as
        # throughput drops and freeze the sizes, which is not what the figure shows)
        d = oc.DynamicBatcher([200, 200, 200], G, ewma_alpha=alpha, deadband=deadband,
                              adaptive_b_max=False)
        b = list(d.b)
        for it in range(200):
            b = d.observe(synth.plant_times(b, s, noise=0.02, seed=77, step=it))
        return d.readjustments
    assert run(0.0, 1.0) > 100
    assert run(0.05, 1.0) <= 3
    assert run(0.05, 0.5) <= 2


def test_dynamic_heterogeneity_is_tracked_and_ewma_spans_only_the_quiet_interval():
    G = 1200
    d = oc.DynamicBatcher([300] * 4, G, ewma_alpha=0.5, deadband=0.05)
    s = [1.0, 1.0, 2.0, 4.0]
    b = list(d.b)
    for it in range(10):
        b = d.observe(synth.plant_times(b, s))
    assert b == [150, 150, 300, 600] and d.readjustments == 1
    s = [1.0, 0.25, 2.0, 4.0]                               # worker 1 loses 3/4 of its speed
    n0 = d.readjustments
    for it in range(20):
        b = d.observe(synth.plant_times(b, s))
    want = [G * v / sum(s) for v in s]
    assert max(abs(bk - wk) / wk for bk, wk in zip(b, want)) < 0.06
    assert 1 <= d.readjustments - n0 <= 6                   # smoothed: a few steps, then quiet
    for it in range(20):
        assert d.observe(synth.plant_times(b, s)) == b


def test_throughput_knee_hand_worked_trace():
    rows = read_rows("throughput_knee_example.txt")
    d = oc.DynamicBatcher([50, 50], 100, ewma_alpha=1.0, deadband=0.05, b_min=1, b_max=100)
    b = list(d.b)
    for it, want_b, want_hi in rows:
        b = d.observe(synth.plant_times(b, [1.0, 3.0], knee=[None, 60], knee_penalty=2.0))
        assert b == [int(v) for v in want_b], (it, b)
        assert d.b_hi == [int(v) for v in want_hi], (it, d.b_hi)


def test_learnt_bound_never_breaks_the_global_batch_and_only_shrinks():
    rng = np.random.default_rng(11)
    for trial in range(30):
        K = int(rng.integers(2, 7)); G = int(rng.integers(K * 20, K * 200))
        s = list(rng.uniform(0.5, 8.0, K))
        knee = [int(v) for v in rng.integers(G // K // 2, G, K)]
        d = oc.DynamicBatcher(synth.ragged_split(G, K, trial), G, ewma_alpha=0.5, b_min=1)
        b = list(d.b); hi_prev = list(d.b_hi)
        for it in range(25):
            b = d.observe(synth.plant_times(b, s, knee=knee, knee_penalty=3.0, noise=0.01,
                                            seed=trial, step=it))
            assert sum(b) == G and all(1 <= b[k] <= d.b_hi[k] for k in range(K))
            assert all(d.b_hi[k] <= hi_prev[k] for k in range(K)) and sum(d.b_hi) >= G
            hi_prev = list(d.b_hi)


def test_min_observations_delays_the_first_readjustment():
    d = oc.DynamicBatcher([50, 50], 100, ewma_alpha=0.5, min_observations=3)
    assert d.observe([10.0, 30.0]) == [50, 50]
    assert d.observe([10.0, 30.0]) == [50, 50]
    assert d.observe([10.0, 30.0]) == [75, 25]


def test_per_worker_bounds_in_the_stateless_step():
    b = oc.controller_step([1.0, 1.0, 4.0], [40, 40, 40], 120, deadband=0.0, b_hi=[45, 120, 120])
    assert sum(b) == 120 and b[0] <= 45 and b[2] < 40
    with pytest.raises(oc.ControllerError):
        oc.controller_step([1.0, 1.0], [50, 50], 100, b_hi=[40, 40])
