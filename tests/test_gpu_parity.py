"""GPU parity: the HIP path (through the C interface) against the CPU checker, element by
element on the same seeded inputs.

Tolerances (max-abs-normalised per tensor, max|got - ref| / max|ref|): fp32 1e-4; bf16 2e-2.
The bf16 reference is the checker with bfloat16 rounding emulated at the points where the kernels
store 16-bit values; against it the kernels differ only by fp32-vs-fp64 accumulation and by a
stored value that rounds the other way now and then (one bfloat16 unit in the last place, 2^-8
relative).  In a worker with a handful of samples one stored value can dominate an output entry,
and two such roundings can chain (an activation and the gradient arriving at it), so the tests
hold the kernels to 2 * 2^-8 = 8e-3, inside the 2e-2 the method is allowed.
ReLU derivative decisions on units inside the rounding band are resolved as tests/relu_ties.py
describes; all other decisions are the checker's.
"""
import numpy as np
import pytest

from oracle import controller as oc
from oracle import network as on
from paper_2305_12213_amd import binding, synth
from gpu_harness import DeviceRun, relerr, worker_grads_as_lists, worst_pair_relerr, worst_relerr
from relu_ties import resolved_worker_references

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TOL_EMULATED = 8e-3


def check_worker_gradients(spec, params, x, y, b, run=None, label=""):
    run = run or DeviceRun(spec, params, max(1, sum(b)), len(b))
    g = run.forward_backward(x, y, b).cpu().numpy()
    bf = spec["dtype"] == "bf16"
    got = worker_grads_as_lists(spec, g, run.P)
    refs, losses, n_amb, n_flip = resolved_worker_references(spec, params, x, y, b, got, bf)
    got_losses = run.losses(len(b))
    tol = TOL_EMULATED if bf else TOL["f32"]
    for k in range(len(b)):
        e = worst_pair_relerr(got[k], refs[k])
        assert e < tol, (label, "worker", k, b[k], e, n_amb, n_flip)
        assert abs(got_losses[k] - losses[k]) <= (4e-3 if bf else 1e-5) * max(1.0, abs(losses[k]))
        assert np.all(g[k, run.P:] == 0.0)
        if b[k] == 0:
            assert np.all(g[k] == 0.0)
    if bf and not any(L.get("relu") for L in spec["layers"]):
        # no 0/1 decisions: the exact float64 computation is a fair reference at 2e-2
        _, exact = on.worker_gradients(spec, params, x, y, b)
        for k in range(len(b)):
            assert worst_pair_relerr(got[k], exact[k]) < TOL["bf16"]
    return run, g, refs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dims,b", [
    ([64, 10], [32, 32]),
    ([64, 10], [1, 63]),
    ([40, 24, 7], [5, 0, 3]),                      # widths that are no multiple of anything
    ([72, 130, 66, 10], [1, 2, 3, 15, 16, 17, 31, 33]),
    ([256, 192, 10], [63, 65, 127, 129]),          # several tiles and ragged tails
    ([200, 300, 5], [255, 257, 1]),
    ([96, 64, 12], [0, 0, 9]),
    ([48, 1100], [3, 5]),                          # more classes than the softmax keeps in registers
    ([48, 1000], [2, 7]),                          # ... and just below that
])
def test_worker_gradients_on_ragged_splits(dtype, dims, b):
    spec = synth.mlp_spec(dims, dtype)
    params = synth.init_params(spec, "he", 17)
    # non-zero biases so that the bias path is exercised
    rng = np.random.default_rng(1)
    params = [(W, (rng.standard_normal(bb.shape) * 0.1).astype(np.float32)) for W, bb in params]
    x, y = synth.make_batch(spec, "normal", sum(b), 99, 0)
    check_worker_gradients(spec, params, x, y, b, label=str((dtype, dims, b)))


def small_cnn():
    return {"dtype": "bf16", "input": (8, 8, 3), "classes": 5,
            "layers": [synth.conv3x3(3, 8, 1), synth.conv3x3(8, 16, 2), synth.conv3x3(16, 24, 2),
                       synth.gap(), synth.dense(24, 5, relu=False)]}


@pytest.mark.parametrize("b", [[4, 3], [1, 0, 6], [9], [2, 2, 2, 2], [17, 1]])
def test_cnn_worker_gradients_on_ragged_splits(b):
    # implicit-GEMM convolutions (stride 1 and 2, channel counts that need padding), pooling,
    # split weight-gradient reductions
    spec = small_cnn()
    params = synth.init_params(spec, "he", 23)
    rng = np.random.default_rng(2)
    params = [(W, (rng.standard_normal(bb.shape) * 0.1).astype(np.float32)) for W, bb in params]
    x, y = synth.make_batch(spec, "uniform", sum(b), 77, 0)
    check_worker_gradients(spec, params, x, y, b, label="cnn " + str(b))


def test_cnn_odd_image_size_and_wide_channels():
    spec = {"dtype": "bf16", "input": (7, 5, 3), "classes": 4,
            "layers": [synth.conv3x3(3, 40, 2), synth.conv3x3(40, 72, 1), synth.gap(),
                       synth.dense(72, 4, relu=False)]}
    params = synth.init_params(spec, "he", 5)
    x, y = synth.make_batch(spec, "normal", 11, 6, 0)
    check_worker_gradients(spec, params, x, y, [5, 6], label="cnn odd")


@pytest.mark.parametrize("channels", [(72, 136, 40), (128, 64, 32)])
def test_cnn_channel_blocks_and_row_chunks(channels):
    # more than 64 input and output channels (several 64-channel blocks, the last one ragged),
    # channel counts that are and are not powers of two, a stride-2 layer, and workers whose
    # pixel rows span several chunks of the weight-gradient reduction with a ragged last chunk
    c1, c2, c3 = channels
    spec = {"dtype": "bf16", "input": (8, 8, 3), "classes": 5,
            "layers": [synth.conv3x3(3, c1, 1), synth.conv3x3(c1, c2, 1), synth.conv3x3(c2, c3, 2),
                       synth.gap(), synth.dense(c3, 5, relu=False)]}
    params = synth.init_params(spec, "he", 51)
    b = [9, 1, 0, 5]
    x, y = synth.make_batch(spec, "normal", sum(b), 52, 0)
    check_worker_gradients(spec, params, x, y, b, label="cnn blocks %s" % (channels,))


@pytest.mark.parametrize("image,channels", [((32, 32, 3), (64, 128, 72)), ((8, 32, 3), (64, 20, 64))])
def test_cnn_on_32_wide_images(image, channels):
    # 32-wide images select the halo-tile convolution kernel for forward and input gradient and
    # the row-staged weight gradient (stride 1; whole 64-channel blocks per tap: 64 and 128
    # channels; output channel counts that fill a block, leave 8, or are no multiple of 8; an
    # image one tile high); the stem (3 channels), layers behind a ragged channel count and the
    # strided layer stay on the gathered-operand kernel
    c1, c2, c3 = channels
    spec = {"dtype": "bf16", "input": image, "classes": 5,
            "layers": [synth.conv3x3(3, c1, 1), synth.conv3x3(c1, c2, 1), synth.conv3x3(c2, c3, 1),
                       synth.conv3x3(c3, 16, 2), synth.gap(), synth.dense(16, 5, relu=False)]}
    params = synth.init_params(spec, "he", 61)
    rng = np.random.default_rng(3)
    params = [(W, (rng.standard_normal(bb.shape) * 0.1).astype(np.float32)) for W, bb in params]
    b = [2, 0, 1]
    x, y = synth.make_batch(spec, "uniform", sum(b), 62, 0)
    check_worker_gradients(spec, params, x, y, b, label="cnn 32 wide %s" % (channels,))


def test_sixty_four_workers():
    # the largest worker count the interface takes, most workers tiny, some idle
    for dtype in ("f32", "bf16"):
        spec = synth.mlp_spec([48, 40, 6], dtype)
        params = synth.init_params(spec, "he", 41)
        b = synth.ragged_split(300, 64, 9)
        assert len(b) == 64 and 0 in b
        x, y = synth.make_batch(spec, "normal", sum(b), 41, 0)
        check_worker_gradients(spec, params, x, y, b, label="K=64 " + dtype)


def test_large_tile_kernels_on_ragged_edges(capsys):
    # sizes that select the 256 x 256 tile kernels for the forward, input-gradient and
    # weight-gradient products (at least 192 tiles of 256 x 256: layer 1 forward 13 x 16, layer 2
    # input gradient 13 x 16, layer 2 weight gradient 14 x 16) while no dimension is a multiple
    # of the tile: 3100 rows, widths 3900 and 3340, a reduction length (600) that ends inside a
    # stage, workers of 1265, 1023, 1, 0, 257 and 554 rows (segment tails inside 16-byte
    # granules, an idle worker)
    spec = synth.mlp_spec([600, 3900, 3340, 24], "bf16")
    params = synth.init_params(spec, "he", 43)
    b = [1265, 1023, 1, 0, 257, 554]
    x, y = synth.make_batch(spec, "normal", sum(b), 43, 0)
    with capsys.disabled():
        print("large ragged tiles: checker at work (about a minute)", flush=True)
    check_worker_gradients(spec, params, x, y, b, label="256-tile ragged")


def test_linear_hidden_layer_with_a_large_input():
    # no ReLU under the second layer: its input gradient reads no mask, so the schedule gives the
    # layer's 17 MB input a sequential read of its own before the weight gradient re-fetches it
    spec = {"dtype": "bf16", "input": (512,), "classes": 24,
            "layers": [synth.dense(512, 4096, relu=False), synth.dense(4096, 24, relu=False)]}
    params = synth.init_params(spec, "he", 47)
    b = [1000, 600, 0, 512]
    x, y = synth.make_batch(spec, "normal", sum(b), 47, 0)
    check_worker_gradients(spec, params, x, y, b, label="linear hidden layer")


def test_same_handle_serves_changing_batch_splits():
    # batch sizes change every step; nothing is rebuilt per size and stale padding is harmless
    spec = synth.mlp_spec([128, 96, 10], "bf16")
    params = synth.init_params(spec, "he", 3)
    run = DeviceRun(spec, params, 300, 6)
    for step, b in enumerate(([50] * 6, [1, 9, 100, 120, 3, 67], [300], [0, 299, 1], [7, 7, 7, 7])):
        x, y = synth.make_batch(spec, "uniform", sum(b), 5, step)
        check_worker_gradients(spec, params, x, y, b, run=run, label=str(b))


def test_bf16_gemms_are_exact_on_exactly_representable_inputs():
    # small integers: every product and partial sum is exact in bf16 x bf16 -> fp32
    spec = synth.mlp_spec([64, 10], "bf16")
    rng = np.random.default_rng(0)
    W = rng.integers(-2, 3, (64, 10)).astype(np.float32) / 64
    params = [(W, np.zeros(10, np.float32))]
    x = rng.integers(-3, 4, (40, 64)).astype(np.float32)
    y = rng.integers(0, 10, 40).astype(np.int32)
    b = [16, 8, 16]
    run = DeviceRun(spec, params, 40, 3)
    g = run.forward_backward(x, y, b).cpu().numpy()
    _, ref = on.worker_gradients(spec, params, x, y, b, emulate_bf16=True)
    # logits are exact, so dlogits differ only by fp32 softmax rounding before the bf16 store
    for k in range(3):
        assert worst_relerr(g[k, :run.P], spec, ref[k]) < 4e-3


@pytest.mark.parametrize("K,n", [(1, 256), (2, 768), (3, 1024 * 33), (4, 256 * 1000 + 256),
                                 (7, 512), (16, 256 * 4097), (64, 2048)])
def test_weighted_aggregate_matches_definition(K, n):
    import torch
    rng = np.random.default_rng(K * 1000 + n)
    g = rng.standard_normal((K, n)).astype(np.float32)
    b = synth.ragged_split(4096, K, n)
    if sum(b) == 0:
        b[0] = 1
    gd = torch.from_numpy(g).cuda()
    out = torch.full((n,), float("nan"), device="cuda")
    binding.weighted_aggregate(gd, b, n, out)
    lam = np.array(b, np.float64) / sum(b)
    ref = (lam[:, None] * g.astype(np.float64)).sum(axis=0)
    assert relerr(out.cpu().numpy(), ref) < 1e-6


def test_equal_batches_aggregate_to_the_plain_mean():
    import torch
    g = torch.randn(4, 1024, device="cuda", generator=torch.Generator("cuda").manual_seed(1))
    out = torch.empty(1024, device="cuda")
    binding.weighted_aggregate(g, [7, 7, 7, 7], 1024, out)
    assert relerr(out.cpu().numpy(), g.double().mean(0).cpu().numpy()) < 1e-6


def test_sgd_and_momentum_updates_match_definition():
    import torch
    n = 256 * 513
    rng = np.random.default_rng(4)
    x0 = rng.standard_normal(n).astype(np.float32); g = rng.standard_normal(n).astype(np.float32)
    xd, gd = torch.from_numpy(x0).cuda(), torch.from_numpy(g).cuda()
    binding.sgd_update(xd, gd, n, 0.05)
    assert relerr(xd.cpu().numpy(), x0.astype(np.float64) - 0.05 * g) < 1e-6
    xd = torch.from_numpy(x0).cuda(); vd = torch.zeros(n, device="cuda")
    x, v = x0.astype(np.float64), np.zeros(n)
    for _ in range(5):
        binding.sgd_momentum_update(xd, vd, gd, n, 0.05, 0.9)
        v = 0.9 * v + g; x = x - 0.05 * v
    assert relerr(xd.cpu().numpy(), x) < 1e-5 and relerr(vd.cpu().numpy(), v) < 1e-5


def test_split_invariance_on_the_gpu():
    # weighted aggregate over any K-way split == gradient of the whole batch on one worker
    spec = synth.mlp_spec([96, 80, 10], "f32")
    params = synth.init_params(spec, "he", 8)
    x, y = synth.make_batch(spec, "normal", 120, 8, 0)
    run = DeviceRun(spec, params, 120, 8)
    run.forward_backward(x, y, [120]); whole = run.aggregate([120]).cpu().numpy().copy()
    for b in ([60, 60], [1, 119], [17, 0, 3, 100], [15] * 8):
        run.forward_backward(x, y, b)
        got = run.aggregate(b).cpu().numpy()
        # rows keep their position relative to an 8-row boundary only by chance, so the fp32
        # summation order of a row's products may differ between splits: 1e-5, not equality
        assert relerr(got, whole) < 1e-5, b


def applied_step_relerr(spec, before, after, step_ref, P):
    """Largest per-tensor error of the step a device update applied, (after - before) against the
    checker's step, normalised by the largest entry of the checker's step for that tensor (not by
    the parameters, next to which one step is invisible).  fp32 parameters cannot hold a step
    more finely than half a unit in the last place of the parameter: that much is allowed on top."""
    got = synth.unflatten_params(spec, (np.asarray(after[:P], np.float64) - np.asarray(before[:P], np.float64)))
    held = synth.unflatten_params(spec, np.asarray(before[:P], np.float64))
    worst = 0.0
    for (gW, gb), (rW, rb), (pW, pb) in zip(got, step_ref, held):
        for g, r, p in ((gW, rW, pW), (gb, rb, pb)):
            scale = np.max(np.abs(r))
            if scale == 0.0:
                assert np.max(np.abs(g)) == 0.0
                continue
            slack = 2.0 ** -24 * max(np.max(np.abs(p)), scale) / scale
            worst = max(worst, np.max(np.abs(g - r)) / scale - slack)
    return worst


def run_workload(ci, steps, gains=None, say=None, ambiguous_ceiling=None):
    """Runs `steps` training steps of workload ci, every step on both sides from the same state.

    The checker owns the trajectory (fp32 master parameters, like the GPU's): before each step
    its parameters (and velocity) are copied to the GPU, both sides take the step on the same
    seeded batch and the same b[K], and every worker's gradient, the aggregate, the step the
    update applied to the parameters (and the velocity) are compared.  Nothing flows from the GPU
    into the checker's trajectory: ReLU ties (tests/relu_ties.py) only select which admissible
    reference a gradient is compared with, the trajectory always continues from the checker's
    own decisions.  ambiguous_ceiling = (share of all ReLU units, multiple of the decisions
    found different): the band that excuses ties must stay that narrow.  (The band is laid out
    for the noisiest accumulation order, tests/test_relu_ties.py; the matrix cores are several
    times quieter, hence multiples in the hundreds rather than the ~100 of that case.)
    Returns the worst errors seen and the trace of batch sizes.
    """
    cfg = synth.config(ci)
    spec, seed = cfg["spec"], synth.BASE_SEED + ci
    bf = spec["dtype"] == "bf16"
    G, K = cfg["global_batch"], cfg["K"]
    gains = dict(cfg["gains"], **(gains or {}))
    ref_p = synth.init_params(spec, cfg["init"], seed)
    ref_v = on.zeros_like_params(ref_p)
    run = DeviceRun(spec, ref_p, G, K)
    b_gpu = list(cfg["b0"]); b_ref = list(cfg["b0"])
    worst_g = worst_agg = worst_p = 0.0
    amb = flips = units = 0
    trace = []
    for step in range(steps):
        assert b_gpu == b_ref
        trace.append(list(b_gpu))
        x, y = synth.make_batch(spec, cfg["x_dist"], G, seed, step)
        if step:
            run.set_params(ref_p)
            if cfg["momentum"]:
                run.set_velocity(ref_v)
        before = run.params.cpu().numpy().copy()
        if step % 2:      # both call forms: aggregate with the gradients / as a pass of its own
            g = run.forward_backward_aggregate(x, y, b_gpu).cpu().numpy()
            out = run.out.cpu().numpy()
        else:
            g = run.forward_backward(x, y, b_gpu).cpu().numpy()
            out = run.aggregate(b_gpu).cpu().numpy()
        run.update(cfg["lr"], cfg["momentum"])
        after = run.params.cpu().numpy()
        got = worker_grads_as_lists(spec, g, run.P)
        refs, _, a, f = resolved_worker_references(spec, ref_p, x, y, b_ref, got, bf)
        amb += a; flips += f
        worst_now = 0.0
        for k in range(K):
            e = worst_pair_relerr(got[k], refs[k])
            worst_now = max(worst_now, e)
        worst_g = max(worst_g, worst_now)
        # the aggregate and the update are compared given the same decisions as the gradients
        agg_given = on.weighted_aggregate(refs, b_ref)
        e_agg = worst_relerr(out[:run.P], spec, agg_given)
        worst_agg = max(worst_agg, e_agg)
        if cfg["momentum"]:
            _, v_given = on.momentum_update(ref_p, ref_v, agg_given, cfg["lr"], cfg["momentum"])
            step_given = [(-cfg["lr"] * vW, -cfg["lr"] * vb) for vW, vb in v_given]
            e_v = worst_relerr(run.velocity.cpu().numpy()[:run.P], spec, v_given)
        else:
            step_given = [(-cfg["lr"] * gW, -cfg["lr"] * gb) for gW, gb in agg_given]
            e_v = 0.0
        e_p = max(applied_step_relerr(spec, before, after, step_given, run.P), e_v)
        worst_p = max(worst_p, e_p)
        if say:
            say("workload %d step %d b=%s: grad %.2e agg %.2e applied step %.2e; ambiguous %d, "
                "decided differently %d" % (ci, step, b_gpu, worst_now, e_agg, e_p, a, f))
        # the checker's own step (its own decisions), fp32 master state
        _, gk = on.worker_gradients(spec, ref_p, x, y, b_ref, emulate_bf16=bf)
        agg = on.weighted_aggregate(gk, b_ref)
        if cfg["momentum"]:
            new_p, ref_v = on.momentum_update(ref_p, ref_v, agg, cfg["lr"], cfg["momentum"])
            ref_v = [(W.astype(np.float32).astype(np.float64), b.astype(np.float32).astype(np.float64))
                     for W, b in ref_v]
        else:
            new_p = on.sgd_update(ref_p, agg, cfg["lr"])
        ref_p = [(W.astype(np.float32), b.astype(np.float32)) for W, b in new_p]
        units += sum(int(np.prod(m.shape)) for m in on.relu_masks_of(spec, ref_p, x[:1], bf).values()) * G
        t = synth.iteration_times(b_gpu, cfg["speeds"])
        b_gpu = binding.controller_step(t, b_gpu, G, gains)
        b_ref = oc.controller_step(t, b_ref, G, **gains)
    trace.append(list(b_gpu))
    print("workload %d: worst grad %.2e agg %.2e applied step %.2e; ambiguous units %d of %d, decided "
          "differently %d" % (ci, worst_g, worst_agg, worst_p, amb, units, flips))
    if ambiguous_ceiling and units:
        share, multiple = ambiguous_ceiling
        assert amb <= share * units, (amb, units)
        assert amb <= multiple * max(flips, 50), (amb, flips)
    return worst_g, worst_agg, worst_p, trace


def test_workload0_softmax_regression_10_steps():
    g, agg, p, trace = run_workload(0, 10)
    assert max(g, agg, p) < 1e-4, (g, agg, p)
    assert trace[-1] == [43, 21]


def test_workload0_free_running_trajectories_agree():
    # no ReLU, hence no 0/1 decisions: two independent 10-step runs stay within tolerance
    cfg = synth.config(0)
    spec, seed = cfg["spec"], synth.BASE_SEED
    p = synth.init_params(spec, cfg["init"], seed)
    run = DeviceRun(spec, p, 64, 2)
    ref = p
    b = list(cfg["b0"])
    for step in range(cfg["steps"]):
        x, y = synth.make_batch(spec, cfg["x_dist"], 64, seed, step)
        run.forward_backward(x, y, b); run.aggregate(b); run.update(cfg["lr"])
        _, gk = on.worker_gradients(spec, ref, x, y, b)
        ref = on.sgd_update(ref, on.weighted_aggregate(gk, b), cfg["lr"])
        b = binding.controller_step(synth.iteration_times(b, cfg["speeds"]), b, 64, cfg["gains"])
    assert worst_relerr(run.params.cpu().numpy()[:run.P], spec, ref) < 1e-4
    # ... and the distance travelled, measured on its own scale
    start = synth.flatten_params(p).astype(np.float64)
    moved_ref = synth.flatten_params(ref).astype(np.float64) - start
    moved_got = run.params.cpu().numpy()[:run.P].astype(np.float64) - start
    assert relerr(moved_got, moved_ref) < 1e-4


def test_workload1_mlp_fp32_50_steps():
    g, agg, p, trace = run_workload(1, 50, ambiguous_ceiling=(1e-4, 1500))
    assert max(g, agg, p) < 1e-4, (g, agg, p)
    assert sum(trace[-1]) == 256 and trace[-1] != trace[0]


def test_workload2_mlp_bf16_momentum_100_steps():
    g, agg, p, trace = run_workload(2, 100, ambiguous_ceiling=(3e-4, 1500))
    # the applied step and the velocity are measured on their own scale
    assert max(g, agg, p) < TOL_EMULATED, (g, agg, p)
    assert sum(trace[-1]) == 1024


def test_workload3_cnn_bf16_full_size_steps(capsys):
    # full-size steps of the CNN workload (512 images of 32x32x3, b = 300/128/61/23); the
    # 50-step controller trace of this workload is checked bit for bit in tests/test_host.py
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    g, agg, p, trace = run_workload(3, 5, say=say, ambiguous_ceiling=(4e-4, 1500))
    assert max(g, agg, p) < TOL_EMULATED, (g, agg, p)
    assert all(b == [300, 128, 61, 23] for b in trace)   # inside the 5 % dead-band: never resized


def test_workload3_cnn_resized_by_the_controller(capsys):
    # the same workload without the dead-band: the first controller call moves the split to the
    # throughput-proportional one, and the kernels run the following steps on it
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    g, agg, p, trace = run_workload(3, 3, gains=dict(deadband=0.0), say=say,
                                    ambiguous_ceiling=(4e-4, 1500))
    assert max(g, agg, p) < TOL_EMULATED, (g, agg, p)
    assert trace[0] == [300, 128, 61, 23] and trace[1] == [305, 122, 61, 24] == trace[2]


def test_workload4_wide_mlp_first_three_steps_full_size(capsys):
    # the first three steps of the real run at full size, in the launch configuration the
    # benchmark times: the uniform start 256 x 16, the split the bounds clip the first
    # controller step to, and the converged ragged split 5 ... 1265 -- every worker's gradient,
    # the aggregate (in-kernel on the odd step, as a pass on the even ones) and the applied
    # update against the checker.  The checker needs minutes of fp64 work here: a line per step
    # goes to the terminal uncaptured.
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    g, agg, p, trace = run_workload(4, 3, say=say, ambiguous_ceiling=(2e-3, 1500))
    assert max(g, agg, p) < TOL_EMULATED, (g, agg, p)
    assert trace[0] == [256] * 16
    assert trace[1][0] > trace[0][0] and trace[1] != trace[2]          # clipped first adjustment
    assert min(trace[2]) <= 8 and max(trace[2]) > 1000                 # the ragged split
    assert trace[3] == trace[2]                                        # the dead-band holds it


def test_workload4_weight_copies_follow_the_update_at_full_width():
    # the 16-bit weight copies the next step reads are refreshed by the update kernel.  One real
    # step moves a weight by 3e-4 of its size, too little to see in the next gradients; so at the
    # workload's width (all weight tiles, few rows) a deliberately large step along a seeded
    # random direction is applied, and the next gradients, computed from the device's own
    # parameters and copies, are compared with the checker's at the same updated parameters
    import torch
    cfg = synth.config(4)
    spec, seed = cfg["spec"], synth.BASE_SEED + 4
    p0 = synth.init_params(spec, cfg["init"], seed)
    b = [40, 3, 21]
    run = DeviceRun(spec, p0, sum(b), len(b))
    rng = np.random.Generator(np.random.PCG64([seed, 9]))
    direction = [((0.1 * np.std(W) * rng.standard_normal(W.shape)).astype(np.float32),
                  (0.01 * rng.standard_normal(bb.shape)).astype(np.float32)) for W, bb in p0]
    run.out.copy_(torch.from_numpy(synth.flatten_params(direction, 256)))
    run.update(1.0)
    p1 = [(W - dW, bb - db) for (W, bb), (dW, db) in zip(p0, direction)]      # float32 arithmetic
    assert all(W.dtype == np.float32 for W, _ in p1)
    assert relerr(run.params.cpu().numpy()[:run.P], synth.flatten_params(p1)) < 1e-6
    x, y = synth.make_batch(spec, cfg["x_dist"], sum(b), seed, 1)
    check_worker_gradients(spec, p1, x, y, b, run=run, label="after a large step")
    _, stale = on.worker_gradients(spec, p0, x, y, b, emulate_bf16=True)
    got = worker_grads_as_lists(spec, run.grads[:len(b)].cpu().numpy(), run.P)
    assert worst_pair_relerr(got[0], stale[0]) > 0.05     # ... stale copies would have failed


def test_bf16_rounding_points_through_two_relu_layers():
    # where the 16-bit roundings sit (input, weight copies, every stored activation and stored
    # activation gradient; accumulation, bias, softmax and gradients in fp32) is part of what is
    # compared, but a rounding forgotten or added on either side moves results by 2^-9, inside
    # the 8e-3 the workload tests allow.  Here every rounding decision is clear-cut -- the
    # checker's gradient does not move when every pre-activation is shifted by the size of fp32 noise,
    # and no ReLU unit is near a tie -- so both sides must round alike and agree to fp32 accuracy.
    spec = synth.mlp_spec([24, 32, 16, 5], "bf16")
    b = [7, 9, 0, 16]
    tol = 2e-5
    for seed in range(40, 60):
        rng = np.random.Generator(np.random.PCG64([seed, 4]))
        params = [(rng.integers(-3, 4, ws).astype(np.float32) * np.float32(0.173),
                   (0.05 * rng.standard_normal(bs)).astype(np.float32))
                  for ws, bs in synth.param_shapes(spec)]
        x, y = synth.make_batch(spec, "normal", sum(b), seed, 0)
        _, ref = on.worker_gradients(spec, params, x, y, b, emulate_bf16=True)
        stable = True
        for shift in (4e-7, -4e-7):      # every pre-activation moved by a few fp32 units
            nudged = [(W, bb + np.float32(shift)) for W, bb in params]
            _, ref2 = on.worker_gradients(spec, nudged, x, y, b, emulate_bf16=True)
            stable &= all(worst_pair_relerr(ref2[k], ref[k]) < tol / 4 for k in range(len(b)))
        ties = sum(int(a.sum()) for a in on.ambiguous_relu_units(spec, params, x, True).values())
        if stable and ties == 0:
            break
    else:
        raise AssertionError("no seed with clear-cut roundings")
    _, exact = on.worker_gradients(spec, params, x, y, b, emulate_bf16=False)
    assert max(worst_pair_relerr(exact[k], ref[k]) for k in (0, 1, 3)) > 1e-3   # roundings matter
    run = DeviceRun(spec, params, sum(b), len(b))
    g = run.forward_backward(x, y, b).cpu().numpy()
    got = worker_grads_as_lists(spec, g, run.P)
    for k in range(len(b)):
        e = worst_pair_relerr(got[k], ref[k])
        assert e < tol, (seed, k, e)
