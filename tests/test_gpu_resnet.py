"""GPU parity of the ResNet-style layers: batch normalisation over each worker's own rows and
residual additions (the shape of the paper's first workload, Section "Experimental Evaluation"),
against the checker with bfloat16 rounding emulated."""
import numpy as np
import pytest

from oracle import network as on
from paper_2305_12213_amd import binding, synth
from gpu_harness import DeviceRun, relerr, worker_grads_as_lists, worst_pair_relerr, worst_relerr
from relu_ties import resolved_worker_references

pytestmark = pytest.mark.gpu

TOL_EMULATED = 8e-3     # as in test_gpu_parity.py
TOL_BF16 = 2e-2         # the tolerance stated for bfloat16 gradients


def perturbed(spec, seed):
    """He weights, small random biases, batch-norm scale and shift away from 1 and 0."""
    rng = np.random.default_rng(seed)
    out = []
    for W, b in synth.init_params(spec, "he", seed):
        if W.ndim == 1:
            out.append(((1.0 + 0.3 * rng.standard_normal(W.shape)).astype(np.float32),
                        (0.3 * rng.standard_normal(b.shape)).astype(np.float32)))
        else:
            out.append((W, (0.1 * rng.standard_normal(b.shape)).astype(np.float32)))
    return out


def layer_errors(got, ref):
    """Largest error over the (weight, bias) gradient pairs of one worker, max-abs-normalised
    per tensor -- except that a bias gradient is measured on the scale of its layer's weight
    gradient when that is larger: the bias of a layer that feeds a batch normalisation has a
    gradient of exactly zero (the normalisation removes the mean), and what either side computes
    for it is only the sum of the roundings of the stored input gradients."""
    worst = 0.0
    for (gW, gb), (rW, rb) in zip(got, ref):
        sw = np.max(np.abs(rW))
        worst = max(worst, np.max(np.abs(gW - rW)) / sw if sw > 0 else np.max(np.abs(gW)))
        sb = max(np.max(np.abs(rb)), sw)
        worst = max(worst, np.max(np.abs(gb - rb)) / sb if sb > 0 else np.max(np.abs(gb)))
    return worst


def check(spec, params, x, y, b, label, tol=TOL_EMULATED):
    run = DeviceRun(spec, params, max(1, sum(b)), len(b))
    g = run.forward_backward_aggregate(x, y, b).cpu().numpy()
    got = worker_grads_as_lists(spec, g, run.P)
    refs, losses, n_amb, n_flip = resolved_worker_references(spec, params, x, y, b, got, True)
    got_losses = run.losses(len(b))
    for k in range(len(b)):
        e = layer_errors(got[k], refs[k])
        assert e < tol, (label, "worker", k, b[k], e, n_amb, n_flip)
        assert abs(got_losses[k] - losses[k]) <= 4e-3 * max(1.0, abs(losses[k]))
        if b[k] == 0:
            assert np.all(g[k] == 0.0)
    # the aggregate, given the gradients the comparison accepted
    agg = on.weighted_aggregate(refs, b)
    out = synth.unflatten_params(spec, run.out.cpu().numpy()[:run.P])
    assert layer_errors(out, agg) < tol
    return run


@pytest.mark.parametrize("b", [[6, 3], [1, 0, 9, 2], [12]])
def test_residual_block_worker_gradients(b):
    spec = synth.resnet_block_spec(channels=16, image=(8, 8, 3), classes=10)
    params = perturbed(spec, 31)
    x, y = synth.make_batch(spec, "normal", sum(b), 31, 0)
    check(spec, params, x, y, b, "resnet block " + str(b))


def test_two_blocks_odd_sizes_and_channel_padding():
    # channel count that needs padding, an image that is not square, two blocks in a row
    spec = synth.resnet_block_spec(channels=12, image=(7, 5, 3), classes=4, blocks=2)
    params = perturbed(spec, 32)
    b = [4, 7, 2]
    x, y = synth.make_batch(spec, "uniform", sum(b), 32, 0)
    # through four normalisations a stored value that rounded the other way has spread (every
    # value computed from it rounds independently from there on): the tolerance stated for
    # bfloat16 holds, the sharper one of the one-block cases no longer does (measured 9e-3 once
    # the band of admissible ReLU decisions was narrowed to what it has to excuse)
    check(spec, params, x, y, b, "two blocks", tol=TOL_BF16)


def test_batchnorm_on_dense_features_and_plain_residual():
    # the same layers without convolutions: rows are samples
    spec = {"dtype": "bf16", "input": (40,), "classes": 6,
            "layers": [synth.dense(40, 24, relu=True), synth.dense(24, 24, relu=False),
                       synth.batchnorm(24, relu=True), synth.dense(24, 24, relu=False),
                       synth.add(0, relu=False), synth.dense(24, 6, relu=False)]}
    params = perturbed(spec, 33)
    b = [9, 1, 14]      # a worker with one sample: its variance is zero, eps carries the division
    x, y = synth.make_batch(spec, "normal", sum(b), 33, 0)
    check(spec, params, x, y, b, "dense bn")


def test_training_steps_with_momentum_follow_the_checker():
    # a few steps on both sides from the same state (the checker owns the trajectory)
    spec = synth.resnet_block_spec(channels=8, image=(8, 8, 3), classes=5)
    ref_p = perturbed(spec, 34)
    ref_v = on.zeros_like_params(ref_p)
    b = [5, 11]
    run = DeviceRun(spec, ref_p, 16, 2)
    for step in range(3):
        x, y = synth.make_batch(spec, "uniform", 16, 34, step)
        run.set_params(ref_p); run.set_velocity(ref_v)
        g = run.forward_backward_aggregate(x, y, b).cpu().numpy()
        run.update(0.05, 0.9)
        got = worker_grads_as_lists(spec, g, run.P)
        refs, _, _, _ = resolved_worker_references(spec, ref_p, x, y, b, got, True)
        agg = on.weighted_aggregate(refs, b)
        p_given, _ = on.momentum_update(ref_p, ref_v, agg, 0.05, 0.9)
        assert worst_relerr(run.params.cpu().numpy()[:run.P], spec, p_given) < TOL_EMULATED
        assert layer_errors(got[0], refs[0]) < TOL_EMULATED and layer_errors(got[1], refs[1]) < TOL_EMULATED
        _, gk = on.worker_gradients(spec, ref_p, x, y, b, emulate_bf16=True)
        new_p, ref_v = on.momentum_update(ref_p, ref_v, on.weighted_aggregate(gk, b), 0.05, 0.9)
        ref_v = [(W.astype(np.float32).astype(np.float64), bb.astype(np.float32).astype(np.float64))
                 for W, bb in ref_v]
        ref_p = [(W.astype(np.float32), bb.astype(np.float32)) for W, bb in new_p]


def test_layer_descriptions_are_validated():
    def model(layers):
        return binding.Model({"dtype": "bf16", "input": (4, 4, 3), "classes": 2, "layers": layers})
    ok = [synth.conv3x3(3, 4, 1), synth.conv3x3(4, 4, 1, relu=False), synth.batchnorm(4, True),
          synth.add(0, True), synth.gap(), synth.dense(4, 2, False)]
    model(ok)
    for bad in ([synth.conv3x3(3, 4, 1), synth.batchnorm(5, True), synth.gap(), synth.dense(4, 2, False)],
                [synth.conv3x3(3, 4, 1), synth.add(0, True), synth.gap(), synth.dense(4, 2, False)],
                [synth.conv3x3(3, 4, 1), synth.conv3x3(4, 8, 1), synth.conv3x3(8, 8, 1),
                 synth.add(0, True), synth.gap(), synth.dense(8, 2, False)],
                [synth.conv3x3(3, 4, 1), synth.conv3x3(4, 4, 1), synth.conv3x3(4, 4, 1),
                 synth.add(0, True), synth.conv3x3(4, 4, 1), synth.add(0, True), synth.gap(),
                 synth.dense(4, 2, False)]):
        with pytest.raises(binding.DynbError):
            model(bad)
    with pytest.raises(binding.DynbError):      # fp32 models have no such layers
        binding.Model({"dtype": "f32", "input": (8,), "classes": 2,
                       "layers": [synth.dense(8, 4, True), synth.batchnorm(4, False),
                                  synth.dense(4, 2, False)]})


WORKLOAD_SPLIT = [170, 169, 86, 43, 22, 11, 0, 11]      # ragged, one idle worker; sums to 512


def workload_size_case(spec, seed, capsys, label, workers=(4, 5, 7)):
    """One pass at the residual workload's batch (512 samples of 32x32x3, 8 workers) and the
    checker's gradients for the given workers (by default the three small ones), each computed
    alone from its own rows (workers are independent of one another: their own statistics).
    Checks for all workers what holds at any size; returns what the caller compares."""
    b = WORKLOAD_SPLIT
    params = perturbed(spec, seed)
    x, y = synth.make_batch(spec, "uniform", sum(b), seed, 0)
    with capsys.disabled():
        print("\n  residual workload (%s): GPU pass" % label, flush=True)
    run = DeviceRun(spec, params, sum(b), len(b))
    g = run.forward_backward_aggregate(x, y, b).cpu().numpy()
    got = worker_grads_as_lists(spec, g, run.P)
    got_losses = run.losses(len(b))
    off = np.concatenate([[0], np.cumsum(b)])
    small = {}
    for k in workers:
        with capsys.disabled():
            print("  residual workload (%s): checker, worker %d (%d samples)" % (label, k, b[k]),
                  flush=True)
        rows = slice(off[k], off[k + 1])
        losses, refs = on.worker_gradients(spec, params, x[rows], y[rows], [b[k]], emulate_bf16=True)
        assert abs(got_losses[k] - losses[0]) <= 4e-3 * max(1.0, abs(losses[0]))
        small[k] = (got[k], refs[0], params, x[rows], y[rows])
    assert np.all(g[6] == 0.0)
    # the aggregate against the weighted sum of the written gradients (float64 on the host)
    lam = np.asarray(b, dtype=np.float64) / sum(b)
    want = np.tensordot(lam, g[:, :run.P].astype(np.float64), axes=1)
    have = run.out.cpu().numpy()[:run.P].astype(np.float64)
    assert np.max(np.abs(have - want)) <= 1e-5 * np.max(np.abs(want))
    # a bias in front of a normalisation: zero gradient up to the summed roundings of the stored
    # input gradients -- small against the weight gradient (without the normalisation's mean
    # subtraction a bias gradient is as large as, or larger than, the weight gradient)
    kinds = [L["kind"] for L in spec["layers"] if L["kind"] in ("conv3x3", "dense", "bn")]
    for k in range(len(b)):
        for i, kind in enumerate(kinds[:-1]):
            if kind == "conv3x3" and kinds[i + 1] == "bn" and b[k] > 0:
                gW, gb = got[k][i]
                assert np.max(np.abs(gb)) <= 0.25 * np.max(np.abs(gW)), (k, i)
    return small


@pytest.mark.parametrize("depth", ["one normalisation", "one block"])
def test_normalisation_kernels_at_workload_size(depth, capsys):
    """Many row chunks per worker (11 264 ... 174 080 rows), 64 channels.  With one
    normalisation the stored values of the two sides round alike almost everywhere and the
    gradients agree to the sharp tolerance; through one residual block (two normalisations,
    three convolutions behind the first) the first differently rounded values have begun to
    spread, and the stated bfloat16 tolerance is what holds (ties in the ReLUs are not resolved:
    one unit among a worker's >= 11 000 pixels moves a gradient by far less)."""
    if depth == "one block":
        spec = synth.resnet_block_spec(64, (32, 32, 3), 10, 1)
    else:
        spec = {"dtype": "bf16", "input": (32, 32, 3), "classes": 10,
                "layers": [synth.conv3x3(3, 64, 1, relu=False), synth.batchnorm(64, relu=True),
                           synth.gap(), synth.dense(64, 10, relu=False)]}
    # one block: also the largest worker (170 images, 174 080 pixel rows, 170 row chunks per
    # normalisation), alone on the checker's side
    workers = (0, 4, 5, 7) if depth == "one block" else (4, 5, 7)
    for k, (got, ref, _, _, _) in workload_size_case(spec, 77, capsys, depth, workers).items():
        e = layer_errors(got, ref)
        assert e < (TOL_BF16 if depth == "one block" else TOL_EMULATED), (depth, "worker", k, e)


def test_residual_workload_three_blocks(capsys):
    """The residual workload itself (three blocks).  Through six normalisations the bfloat16
    roundings of the two sides no longer stay alike: a stored value that rounds the other way
    changes the values computed from it, which then round independently, and the gradient that
    passes a normalisation is a small difference of large terms -- the rounding noise of the
    checker itself (emulated against exact arithmetic) is 5-10 % of these gradients.  What is
    compared here is therefore that the kernels are no farther from the emulating checker than
    that emulation is from exact arithmetic (or within the ordinary tolerance, where that is
    larger); the sharp comparison of the same kernels at this size is the test above."""
    spec = synth.config(5)["spec"]
    assert sum(WORKLOAD_SPLIT) == synth.config(5)["global_batch"]
    cases = workload_size_case(spec, synth.BASE_SEED + 5, capsys, "three blocks")
    for k, (got, ref, params, xk, yk) in cases.items():
        _, exact = on.worker_gradients(spec, params, xk, yk, [len(yk)], emulate_bf16=False)
        for i, ((gW, gb), (rW, rb), (eW, eb)) in enumerate(zip(got, ref, exact[0])):
            scale = np.max(np.abs(rW))
            noise = np.max(np.abs(eW - rW)) / scale
            err = np.max(np.abs(gW - rW)) / scale
            assert err <= max(TOL_EMULATED, noise), ("worker", k, "tensor", i, err, noise)
            sb = max(np.max(np.abs(rb)), scale)
            assert np.max(np.abs(gb - rb)) / sb <= max(TOL_EMULATED, np.max(np.abs(eb - rb)) / sb, noise)
