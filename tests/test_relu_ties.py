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
