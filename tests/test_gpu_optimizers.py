"""GPU parity of the optimizer steps (SGD, momentum, Adam), alone and with the weighted
aggregation folded in, against the fp64 checker.  All inputs are seeded and synthetic: the
per-worker gradients fed to the update are random numbers, not the output of any kernel."""
import numpy as np
import pytest

from oracle import network as on
from paper_2305_12213_amd import binding, synth
from gpu_harness import DeviceRun, relerr, worst_relerr

pytestmark = pytest.mark.gpu


def test_adam_stream_matches_checker():
    import torch
    n = 256 * 517
    rng = np.random.default_rng(21)
    x0 = rng.standard_normal(n).astype(np.float32)
    xd = torch.from_numpy(x0).cuda(); md = torch.zeros(n, device="cuda"); vd = torch.zeros(n, device="cuda")
    p = [(x0.astype(np.float64).reshape(1, -1), np.zeros(0))]
    m = on.zeros_like_params(p); v = on.zeros_like_params(p)
    for t in range(1, 7):
        # gradients of very different sizes, some exactly zero
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 2, n)).astype(np.float32)
        g[rng.integers(0, n, 1000)] = 0.0
        binding.adam_update(xd, md, vd, torch.from_numpy(g).cuda(), n, 1e-3, 0.9, 0.999, 1e-8, t)
        p, m, v = on.adam_update(p, m, v, [(g.astype(np.float64).reshape(1, -1), np.zeros(0))],
                                 lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, t=t)
        # the steps themselves (<= lr each) against the exact ones
        step_got = xd.cpu().numpy().astype(np.float64) - x0
        step_ref = p[0][0][0] - x0
        assert np.max(np.abs(step_got - step_ref)) < 1e-4 * t * 1e-3 + 4e-7, t
    assert relerr(md.cpu().numpy(), m[0][0][0]) < 1e-5
    assert relerr(vd.cpu().numpy(), v[0][0][0]) < 1e-5


SPECS = [
    ("mlp f32 vector rows", lambda: synth.mlp_spec([96, 80, 12], "f32")),
    ("mlp f32 odd widths", lambda: synth.mlp_spec([33, 30, 10], "f32")),
    ("mlp bf16", lambda: synth.mlp_spec([200, 136, 10], "bf16")),
    # more dense matrices than one update launch takes (eight): two launches, the second without
    # the small tensors
    ("mlp f32 eleven layers", lambda: synth.mlp_spec([40, 36, 36, 36, 33, 36, 36, 36, 36, 36, 36, 7], "f32")),
    ("cnn bf16", lambda: {"dtype": "bf16", "input": (8, 8, 3), "classes": 5,
                          "layers": [synth.conv3x3(3, 8, 1), synth.conv3x3(8, 16, 2), synth.gap(),
                                     synth.dense(16, 5, relu=False)]}),
]
OPTS = [
    dict(kind="sgd", lr=0.05),
    dict(kind="momentum", lr=0.05, momentum=0.9),
    dict(kind="adam", lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8),
]


def ref_step(opt, p, s1, s2, agg, t):
    if opt["kind"] == "sgd":
        return on.sgd_update(p, agg, opt["lr"]), s1, s2
    if opt["kind"] == "momentum":
        p, s1 = on.momentum_update(p, s1, agg, opt["lr"], opt["momentum"])
        return p, s1, s2
    return on.adam_update(p, s1, s2, agg, lr=opt["lr"], beta1=opt["beta1"], beta2=opt["beta2"],
                          eps=opt["eps"], t=t)


@pytest.mark.parametrize("name,make_spec", SPECS, ids=[s[0] for s in SPECS])
@pytest.mark.parametrize("opt", OPTS, ids=[o["kind"] for o in OPTS])
def test_model_update_and_fused_aggregate_update(name, make_spec, opt):
    import torch
    spec = make_spec()
    K, G = 5, 40
    b = [13, 0, 7, 19, 1]
    p0 = synth.init_params(spec, "he", 31)
    sep = DeviceRun(spec, p0, G, K)          # weighted_aggregate, then model_update
    fus = DeviceRun(spec, p0, G, K)          # model_aggregate_update
    P, Pp = sep.P, sep.Pp
    rng = np.random.default_rng(77)
    st = {r: [torch.zeros(Pp, device="cuda"), torch.zeros(Pp, device="cuda")] for r in (sep, fus)}
    ref_p = [(W.astype(np.float64), bb.astype(np.float64)) for W, bb in p0]
    ref_s1 = on.zeros_like_params(ref_p); ref_s2 = on.zeros_like_params(ref_p)
    for t in range(1, 4):
        gk = rng.standard_normal((K, Pp)).astype(np.float32)
        gk[:, P:] = 0.0
        gd = torch.from_numpy(gk).cuda()
        o = binding.make_optimizer(step=t, **opt)
        binding.weighted_aggregate(gd, b, Pp, sep.out)
        binding.model_update(sep.model, sep.out, o, st[sep][0], st[sep][1])
        binding.model_aggregate_update(fus.model, gd, b, o, st[fus][0], st[fus][1])
        agg = on.weighted_aggregate([synth.unflatten_params(spec, gk[k, :P].astype(np.float64))
                                     for k in range(K)], b)
        ref_p, ref_s1, ref_s2 = ref_step(opt, ref_p, ref_s1, ref_s2, agg, t)
        for run in (sep, fus):
            assert worst_relerr(run.params.cpu().numpy()[:P], spec, ref_p) < 1e-5, (t, run is fus)
        # same arithmetic in the same order: the two paths agree to the last bits
        assert relerr(fus.params.cpu().numpy(), sep.params.cpu().numpy()) < 1e-6
    if opt["kind"] != "sgd":
        assert worst_relerr(st[fus][0].cpu().numpy()[:P], spec, ref_s1) < 1e-5
    if opt["kind"] == "adam":
        assert worst_relerr(st[fus][1].cpu().numpy()[:P], spec, ref_s2) < 1e-5
    # the kernels' 16-bit weight copies followed the update: losses of a forward pass on the
    # updated model match the checker's at its updated parameters, not at the old ones
    x, y = synth.make_batch(spec, "normal", G, 5, 0)
    bf = spec["dtype"] == "bf16"
    p32 = [(W.astype(np.float32), bb.astype(np.float32)) for W, bb in ref_p]
    want, _ = on.worker_gradients(spec, p32, x, y, b, emulate_bf16=bf)
    old, _ = on.worker_gradients(spec, p0, x, y, b, emulate_bf16=bf)
    for run in (sep, fus):
        run.forward_backward(x, y, b)
        got = run.losses(K)
        for k in range(K):
            if b[k]:
                assert abs(got[k] - want[k]) < (2e-2 if bf else 1e-4) * max(1.0, abs(want[k])), (k, got, want)
    assert max(abs(want[k] - old[k]) for k in range(K) if b[k]) > 0.05      # the step was visible


def test_update_argument_checks():
    import torch
    spec = synth.mlp_spec([16, 8, 4], "f32")
    run = DeviceRun(spec, synth.init_params(spec, "he", 1), 8, 2)
    g = torch.zeros(run.Pp, device="cuda"); s = torch.zeros(run.Pp, device="cuda")
    with pytest.raises(binding.DynbError):
        binding.model_update(run.model, g, binding.make_optimizer("momentum", lr=0.1))      # no state
    with pytest.raises(binding.DynbError):
        binding.model_update(run.model, g, binding.make_optimizer("adam", lr=0.1, step=0), s, s)
    with pytest.raises(binding.DynbError):
        binding.model_update(run.model, g, binding.make_optimizer(7, lr=0.1))
    with pytest.raises(binding.DynbError):
        binding.model_aggregate_update(run.model, run.grads, [0, 0], binding.make_optimizer("sgd", lr=0.1))
    with pytest.raises(binding.DynbError):
        binding.adam_update(g, s, s, g, run.Pp, 0.1, 1.0, 0.999, 1e-8, 1)


def test_forward_backward_aggregate_equals_the_two_call_form():
    # small models (aggregate by a pass over the written gradients), one whose weight gradients
    # are large enough for the in-kernel sum on 256 x 128 tiles (>= 256 of them), and one that
    # takes the in-kernel sum on 128 x 128 tiles (264 of them, edge tiles in both directions)
    import torch
    cases = [(synth.mlp_spec([96, 80, 12], "f32"), [13, 0, 7, 19, 1]),
             (synth.mlp_spec([200, 136, 10], "bf16"), [5, 60, 0, 31]),
             (SPECS[3][1](), [3, 9, 0, 4]),
             (synth.mlp_spec([2500, 4200, 16], "bf16"), [700, 1, 0, 257, 66]),
             (synth.mlp_spec([4100, 1000, 16], "bf16"), [300, 2, 0, 129, 40]),
             # ... and with a width that rules out 16-byte stores (the same kernel's element-wise path)
             (synth.mlp_spec([4100, 1001, 16], "bf16"), [300, 2, 0, 129, 40]),
             # 64 workers, several of them idle: both aggregating kernels at the largest K
             (synth.mlp_spec([2500, 4200, 16], "bf16"), [(i * 37) % 23 for i in range(64)]),
             (synth.mlp_spec([2100, 2100, 16], "bf16"), [(i * 29) % 19 for i in range(64)])]
    for spec, b in cases:
        G, K = sum(b), len(b)
        p0 = synth.init_params(spec, "he", 11)
        x, y = synth.make_batch(spec, "normal", G, 11, 0)
        two = DeviceRun(spec, p0, G, K); one = DeviceRun(spec, p0, G, K)
        xd = torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()
        yd = torch.from_numpy(np.ascontiguousarray(y, np.int32)).cuda()
        two.forward_backward(xd, yd, b); two.aggregate(b)
        binding.forward_backward_aggregate(one.model, xd, yd, b, one.grads, one.out)
        torch.cuda.synchronize()
        g2, g1 = two.grads[:K].cpu().numpy(), one.grads[:K].cpu().numpy()
        o2, o1 = two.out.cpu().numpy(), one.out.cpu().numpy()
        assert np.all(np.isfinite(o1)) and np.all(o1[one.P:] == 0.0)
        # per-worker gradients: same arithmetic up to the tile shape of the large case
        assert relerr(g1, g2) < 1e-6
        # the aggregate: the same products, summed in a rotation of the ascending-k order
        assert relerr(o1, o2) < 1e-6, spec["layers"][0]
        # and against the checker's definition, given the gradients the GPU wrote
        ref = np.zeros(one.Pp)
        for k in range(K):
            ref += (b[k] / G) * g1[k].astype(np.float64)
        assert relerr(o1, ref) < 1e-6
