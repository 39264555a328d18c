"""The tie-robust reference (tests/relu_ties.py) on the CPU: planted near-ties decided the
other way must be explained exactly; errors outside ambiguous units must not be."""
import numpy as np
import pytest

from oracle import network as on
from paper_2305_12213_amd import synth
from relu_ties import resolved_reference


def maxdiff(a, b):
    return max(max(np.abs(x[0] - y[0]).max(), np.abs(x[1] - y[1]).max()) for x, y in zip(a, b))


def test_planted_ties_in_two_layers_are_resolved_exactly():
    spec = synth.mlp_spec([32, 24, 16, 5], "f32")
    params = [(W.astype(np.float64), b.astype(np.float64)) for W, b in synth.init_params(spec, "he", 1)]
    x, y = synth.make_batch(spec, "normal", 60, 1, 0)
    x = x.astype(np.float64)
    # layer 0: put unit 5 of sample 7 and unit 5 of sample 9 (same column) next to zero
    z1 = x @ params[0][0]
    b1 = np.zeros(24); b1[5] = -z1[7, 5] + 1e-9
    x[9] += (-(z1[9, 5] + b1[5]) + 2e-9) * params[0][0][:, 5] / np.sum(params[0][0][:, 5] ** 2)
    params[0] = (params[0][0], b1)
    a1 = np.maximum(x @ params[0][0] + b1, 0)
    z2 = a1 @ params[1][0]
    b2 = np.zeros(16); b2[3] = -z2[7, 3] - 1e-9              # layer 1, same sample as a layer-0 tie
    params[1] = (params[1][0], b2)
    amb = on.ambiguous_relu_units(spec, params, x)
    assert amb[0][7, 5] and amb[0][9, 5] and amb[1][7, 3]
    masks = on.relu_masks_of(spec, params, x)
    other = {k: v.copy() for k, v in masks.items()}
    other[0][7, 5] ^= True; other[1][7, 3] ^= True           # the "other implementation"
    _, got = on.loss_and_gradient(spec, params, x, y, relu_masks=other)
    _, base = on.loss_and_gradient(spec, params, x, y)
    assert maxdiff(got, base) > 1e-4
    ref, _, n_amb, n_flip = resolved_reference(spec, params, x, y, got)
    assert n_flip == 2 and n_amb >= 3
    assert maxdiff(got, ref) < 1e-13


def test_errors_outside_ambiguous_units_are_not_explained_away():
    spec = synth.mlp_spec([32, 24, 5], "f32")
    params = synth.init_params(spec, "he", 2)
    x, y = synth.make_batch(spec, "normal", 40, 2, 0)
    masks = on.relu_masks_of(spec, params, x)
    amb = on.ambiguous_relu_units(spec, params, x)
    i, u = np.argwhere(~amb[0] & masks[0])[0]
    wrong = {0: masks[0].copy()}; wrong[0][i, u] = False       # a clear-cut unit decided wrongly
    _, got = on.loss_and_gradient(spec, params, x, y, relu_masks=wrong)
    ref, _, _, _ = resolved_reference(spec, params, x, y, got)
    assert maxdiff(got, ref) > 1e-5


def test_planted_tie_in_a_conv_layer_is_resolved():
    spec = {"dtype": "f32", "input": (6, 6, 2), "classes": 3,
            "layers": [synth.conv3x3(2, 3, 1), synth.conv3x3(3, 4, 2), synth.gap(),
                       synth.dense(4, 3, relu=False)]}
    rng = np.random.default_rng(3)
    params = [(rng.standard_normal(ws) * 0.4, np.zeros(bs)) for ws, bs in synth.param_shapes(spec)]
    x = rng.standard_normal((4, 6, 6, 2)); y = rng.integers(0, 3, 4)
    a1 = np.maximum(on.conv3x3_forward(x, params[0][0], params[0][1], 1), 0)
    z2 = on.conv3x3_forward(a1, params[1][0], np.zeros(4), 2)
    # shift one input pixel of sample 2 so that unit (2, 1, 2, channel 1) of conv 2 lands at ~1e-9
    b2 = np.zeros(4)
    params[1] = (params[1][0], b2)
    target = (2, 1, 2, 1)
    # adjust the bias for that channel only: it moves every unit of the channel, only one is near zero
    b2[1] = -z2[target] + 1e-9
    amb = on.ambiguous_relu_units(spec, params, x)
    assert amb[1][target] and amb[1].sum() == 1
    masks = on.relu_masks_of(spec, params, x)
    other = {k: v.copy() for k, v in masks.items()}
    other[1][target] ^= True
    _, got = on.loss_and_gradient(spec, params, x, y, relu_masks=other)
    ref, _, _, n_flip = resolved_reference(spec, params, x, y, got)
    assert n_flip == 1 and maxdiff(got, ref) < 1e-13


def _resnet_case():
    spec = synth.resnet_block_spec(channels=4, image=(6, 6, 2), classes=3)
    rng = np.random.default_rng(8)
    params = []
    for ws, bs in synth.param_shapes(spec):
        if len(ws) == 1:
            params.append((1.0 + 0.2 * rng.standard_normal(ws), 0.2 * rng.standard_normal(bs)))
        else:
            params.append((rng.standard_normal(ws) * 0.4, 0.1 * rng.standard_normal(bs)))
    x = rng.standard_normal((12, 6, 6, 2)); y = rng.integers(0, 3, 12)
    return spec, params, x, y


def test_ties_behind_batchnorm_and_residual_layers_are_resolved():
    # bfloat16 storage makes a good share of the units ambiguous; decide some of them, in the
    # ReLU behind the batch normalisation and in the one behind the residual addition, the other
    # way and let the generic route find them
    spec, params, x, y = _resnet_case()
    relu_layers = [li for li, L in enumerate(spec["layers"]) if L.get("relu")]
    assert relu_layers == [0, 2, 5]
    # put two units behind the first batch normalisation (channels 1 and 3) next to zero by
    # moving the shift of their channels
    _, stored = on.forward(spec, params, x, True)
    gamma, beta = params[2]
    z2 = on.batchnorm_forward(stored[2], gamma, beta, spec["layers"][2]["eps"])[0]
    beta = beta.copy()
    beta[1] -= z2[3, 2, 4, 1] - 1e-9
    beta[3] -= z2[7, 0, 1, 3] + 1e-9
    params[2] = (gamma, beta)
    amb = on.ambiguous_relu_units(spec, params, x, True)
    assert amb[2][3, 2, 4, 1] and amb[2][7, 0, 1, 3]
    masks = on.relu_masks_of(spec, params, x, True)
    other = {k: v.copy() for k, v in masks.items()}
    planted = 0
    for li in (2, 5):
        cand = np.argwhere(amb[li])
        assert len(cand) >= 2, (li, len(cand))
        for t in cand[:2]:
            other[li][tuple(t)] ^= True
            planted += 1
    _, got = on.loss_and_gradient(spec, params, x, y, True, relu_masks=other)
    _, base = on.loss_and_gradient(spec, params, x, y, True)
    assert maxdiff(got, base) > 1e-6
    ref, _, n_amb, n_flip = resolved_reference(spec, params, x, y, got, True)
    assert n_flip == planted and n_amb >= planted
    assert maxdiff(got, ref) < 1e-12


def test_generic_route_does_not_explain_away_a_wrong_clear_cut_unit():
    spec, params, x, y = _resnet_case()
    amb = on.ambiguous_relu_units(spec, params, x, True)
    masks = on.relu_masks_of(spec, params, x, True)
    t = tuple(np.argwhere(~amb[2] & masks[2])[0])
    wrong = {k: v.copy() for k, v in masks.items()}
    wrong[2][t] = False
    _, got = on.loss_and_gradient(spec, params, x, y, True, relu_masks=wrong)
    ref, _, _, _ = resolved_reference(spec, params, x, y, got, True)
    assert maxdiff(got, ref) > 1e-6


# ---- the band itself: pinned from below and from above by second implementations ----------
def _fp32_library_masks(spec, params, x, bf16):
    """ReLU decisions of an independent implementation: torch's fp32 CPU routines (their own
    summation orders), bfloat16 storage at the points where the checker emulates it."""
    import torch
    import torch.nn.functional as F
    q = (lambda t: t.bfloat16().float()) if bf16 else (lambda t: t)
    f32 = lambda v: torch.from_numpy(np.ascontiguousarray(v, np.float32))
    a = q(f32(x))
    if a.ndim == 4:
        a = a.permute(0, 3, 1, 2).contiguous()
    stored, masks, pi = [], {}, 0
    for li, L in enumerate(spec["layers"]):
        stored.append(a)
        if L["kind"] == "dense":
            W, b = params[pi]; pi += 1
            a = a.reshape(a.shape[0], -1) @ q(f32(W)) + f32(b)
        elif L["kind"] == "conv3x3":
            W, b = params[pi]; pi += 1
            a = F.conv2d(a, q(f32(W)).permute(3, 2, 0, 1).contiguous(), f32(b), stride=L["stride"],
                         padding=1)
        elif L["kind"] == "bn":
            g, b = params[pi]; pi += 1
            a = F.batch_norm(a, None, None, f32(g), f32(b), True, 0.0, L["eps"])
        elif L["kind"] == "add":
            a = a + stored[L["skip_from"] + 1]
        else:
            a = a.mean(dim=(2, 3))
        if L.get("relu"):
            a = torch.relu(a)
        if li < len(spec["layers"]) - 1:
            a = q(a)
        if L.get("relu"):
            m = (a > 0).numpy()
            masks[li] = m.transpose(0, 2, 3, 1) if m.ndim == 4 else m
    return masks


def _sequential_fp32_masks(spec, params, x):
    """ReLU decisions of a dense bf16 model whose products are accumulated one by one in fp32,
    in index order -- the least accurate order an implementation would use."""
    P = [(on.round_bf16(W).astype(np.float32), np.asarray(b, np.float32)) for W, b in params]
    a = on.round_bf16(x).astype(np.float32)
    masks = {}
    for li, (W, b) in enumerate(P[:-1]):
        acc = np.zeros((a.shape[0], W.shape[1]), np.float32)
        for k in range(W.shape[0]):
            acc += a[:, k:k + 1] * W[k:k + 1, :]        # (float32 product, float32 sum)
        a = on.round_bf16(np.maximum(acc + b, 0.0)).astype(np.float32)
        masks[li] = a > 0
    return masks


def _varied_norm_params(params, seed):
    rng = np.random.default_rng(seed)
    return [(W, b) if np.ndim(W) > 1 else
            ((1 + 0.2 * rng.standard_normal(W.shape)).astype(np.float32),
             (0.2 * rng.standard_normal(b.shape)).astype(np.float32)) for W, b in params]


BAND_CASES = {
    "mlp bf16": (lambda: synth.mlp_spec([1024, 1024, 1024, 1024, 10], "bf16"), 256, "normal"),
    "mlp fp32": (lambda: synth.mlp_spec([512, 512, 512, 10], "f32"), 256, "normal"),
    "cnn bf16": (lambda: synth.cnn_spec("bf16"), 24, "uniform"),
    "residual bf16 (normalisation, addition, pooling)":
        (lambda: synth.resnet_block_spec(32, (16, 16, 3), 10, 2), 32, "uniform"),
}


@pytest.mark.parametrize("name", list(BAND_CASES))
def test_band_contains_every_decision_of_an_fp32_library_implementation(name):
    make, n, dist = BAND_CASES[name]
    spec = make()
    bf = spec["dtype"] == "bf16"
    params = _varied_norm_params(synth.init_params(spec, "he", 5), 1)
    x, _ = synth.make_batch(spec, dist, n, 5, 0)
    theirs = _fp32_library_masks(spec, params, x, bf)
    ours = on.relu_masks_of(spec, params, x, bf)
    amb = on.ambiguous_relu_units(spec, params, x, bf)
    assert sorted(amb) == sorted(ours)
    for li in ours:
        differ = theirs[li] != ours[li]
        assert not (differ & ~amb[li]).any(), (name, li, int((differ & ~amb[li]).sum()))
        # ... and the band is a band: a small part of the layer even behind two residual blocks
        assert amb[li].mean() < (0.15 if "residual" in name else 2e-3), (name, li, amb[li].mean())


def test_band_against_sequential_fp32_accumulation_from_below_and_above():
    # the noisiest plausible implementation of the wide-MLP workload's layers: every decision it
    # takes differently lies inside the band, and the band is not much larger than what it has
    # to cover: a band of `band` = 6 standard deviations around zero holds about 2.5 * 6 times as
    # many units as a noise of one standard deviation flips; the noise constant (taken 1.5 times
    # the sequential sum's), the variance bound of rounded values and the single-jump term make
    # up the rest.  (The interval-arithmetic band this replaced held 2400 times the flips.)
    spec = synth.mlp_spec([2048, 2048, 2048, 2048, 10], "bf16")
    params = synth.init_params(spec, "he", 6)
    x, _ = synth.make_batch(spec, "normal", 1024, 6, 0)
    theirs = _sequential_fp32_masks(spec, params, x)
    ours = on.relu_masks_of(spec, params, x, True)
    amb = on.ambiguous_relu_units(spec, params, x, True)
    flips = sum(int((theirs[li] != ours[li]).sum()) for li in ours)
    inside = sum(int(((theirs[li] != ours[li]) & amb[li]).sum()) for li in ours)
    n_amb = sum(int(a.sum()) for a in amb.values())
    assert flips >= 10, flips                        # the test bites
    assert inside == flips
    print("sequential fp32: %d decisions differ, %d units in the band" % (flips, n_amb))
    assert n_amb <= 200 * flips, (n_amb, flips)


def test_accumulation_noise_constant_covers_sequential_fp32_sums():
    rng = np.random.default_rng(0)
    K = 2048
    a = on.round_bf16(rng.standard_normal((64, K)))
    W = on.round_bf16(rng.standard_normal((K, 128)) * K ** -0.5)
    acc = np.zeros((64, 128), np.float32)
    for k in range(K):
        acc += a[:, k:k + 1].astype(np.float32) * W[k:k + 1, :].astype(np.float32)
    unit = 2.0 ** -24 * np.sqrt(K) * np.sqrt((a * a) @ (W * W))
    sd = float(np.std((acc.astype(np.float64) - a @ W) / unit))
    assert 0.08 < sd < on.ACCUMULATION_NOISE, sd
