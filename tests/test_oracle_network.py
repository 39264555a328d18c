"""Pins for oracle/network.py against things other than itself."""
import itertools

import numpy as np
import pytest
import scipy.signal
import scipy.special
import torch

from oracle import network as on
from paper_2305_12213_amd import synth


def tiny_mlp():
    return synth.mlp_spec([5, 4, 4, 3], "f32")


def tiny_cnn():
    return {"dtype": "f32", "input": (6, 6, 2), "classes": 3,
            "layers": [synth.conv3x3(2, 3, 1), synth.conv3x3(3, 4, 2), synth.gap(),
                       synth.dense(4, 3, relu=False)]}


def tiny_resnet():
    # stem, one residual block (conv-BN-ReLU-conv-BN, + skip, ReLU), pool, classifier
    spec = synth.resnet_block_spec(channels=3, image=(4, 4, 2), classes=3)
    spec["dtype"] = "f32"
    return spec


def rand_params(spec, seed, bias=True):
    rng = np.random.default_rng(seed)
    out = []
    for ws, bs in synth.param_shapes(spec):
        out.append((rng.standard_normal(ws) * 0.5,
                    rng.standard_normal(bs) * (0.3 if bias else 0.0)))
    return out


def mean_loss(spec, params, x, y):
    z, _ = on.forward(spec, params, x)
    lse = scipy.special.logsumexp(z, axis=1)
    return float(np.mean(lse - z[np.arange(len(y)), y]))


@pytest.mark.parametrize("make_spec", [tiny_mlp, tiny_cnn, tiny_resnet])
def test_gradient_matches_central_finite_differences(make_spec):
    spec = make_spec()
    rng = np.random.default_rng(3)
    params = rand_params(spec, 5)
    n = 3
    x = rng.standard_normal((n,) + tuple(spec["input"]))
    y = rng.integers(0, spec["classes"], n)
    loss, grads = on.loss_and_gradient(spec, params, x, y)
    assert abs(loss - mean_loss(spec, params, x, y)) < 1e-12
    h = 1e-6
    worst = 0.0
    for li, (W, b) in enumerate(params):
        for which, arr in enumerate((W, b)):
            flat = arr.reshape(-1)
            g = grads[li][which].reshape(-1)
            for i in range(flat.size):
                old = flat[i]
                flat[i] = old + h; lp = mean_loss(spec, params, x, y)
                flat[i] = old - h; lm = mean_loss(spec, params, x, y)
                flat[i] = old
                fd = (lp - lm) / (2 * h)
                worst = max(worst, abs(fd - g[i]) / max(1e-3, abs(fd)))
    assert worst < 2e-6, worst


def conv_loops(x, W, bias, stride):
    n, H, Wd, Cin = x.shape
    Cout = W.shape[3]
    Ho, Wo = (H - 1) // stride + 1, (Wd - 1) // stride + 1
    out = np.zeros((n, Ho, Wo, Cout))
    for i, ho, wo, co in itertools.product(range(n), range(Ho), range(Wo), range(Cout)):
        acc = bias[co]
        for kh, kw, ci in itertools.product(range(3), range(3), range(Cin)):
            h, w = ho * stride + kh - 1, wo * stride + kw - 1
            if 0 <= h < H and 0 <= w < Wd:
                acc += x[i, h, w, ci] * W[kh, kw, ci, co]
        out[i, ho, wo, co] = acc
    return out


@pytest.mark.parametrize("stride,H,Wd", [(1, 5, 4), (2, 6, 6), (2, 5, 7)])
def test_conv_forward_matches_brute_force_loops(stride, H, Wd):
    rng = np.random.default_rng(stride * 10 + H)
    x = rng.standard_normal((2, H, Wd, 3))
    W = rng.standard_normal((3, 3, 3, 2))
    bias = rng.standard_normal(2)
    np.testing.assert_allclose(on.conv3x3_forward(x, W, bias, stride),
                               conv_loops(x, W, bias, stride), atol=1e-12)


def test_conv_single_channel_is_scipy_correlate2d():
    rng = np.random.default_rng(11)
    img = rng.standard_normal((7, 9))
    ker = rng.standard_normal((3, 3))
    got = on.conv3x3_forward(img[None, :, :, None], ker[:, :, None, None], np.zeros(1), 1)
    want = scipy.signal.correlate2d(img, ker, mode="same", boundary="fill")
    np.testing.assert_allclose(got[0, :, :, 0], want, atol=1e-12)


def test_conv_of_delta_image_returns_flipped_kernel():
    ker = np.arange(9.0).reshape(3, 3) + 1
    img = np.zeros((5, 5)); img[2, 2] = 1.0
    out = on.conv3x3_forward(img[None, :, :, None], ker[:, :, None, None], np.zeros(1), 1)
    np.testing.assert_array_equal(out[0, 1:4, 1:4, 0], ker[::-1, ::-1])


def test_centre_tap_conv_is_a_dense_layer_per_pixel():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 4, 4, 3))
    M = rng.standard_normal((3, 5))
    W = np.zeros((3, 3, 3, 5)); W[1, 1] = M
    b = rng.standard_normal(5)
    np.testing.assert_allclose(on.conv3x3_forward(x, W, b, 1), x @ M + b, atol=1e-12)


def test_conv_backward_is_the_adjoint_of_forward():
    # <conv(x; W), dy> has gradient dW wrt W and dx wrt x: check both inner products.
    rng = np.random.default_rng(8)
    for stride in (1, 2):
        x = rng.standard_normal((2, 6, 6, 3)); W = rng.standard_normal((3, 3, 3, 4))
        y = on.conv3x3_forward(x, W, np.zeros(4), stride)
        dy = rng.standard_normal(y.shape)
        dW, db, dx = on.conv3x3_backward(x, W, dy, stride)
        x2 = rng.standard_normal(x.shape); W2 = rng.standard_normal(W.shape)
        lhs = np.sum(on.conv3x3_forward(x2, W, np.zeros(4), stride) * dy)
        assert abs(lhs - np.sum(x2 * dx)) < 1e-9
        lhs = np.sum(on.conv3x3_forward(x, W2, np.zeros(4), stride) * dy)
        assert abs(lhs - np.sum(W2 * dW)) < 1e-9
        np.testing.assert_allclose(db, dy.reshape(-1, 4).sum(0), atol=1e-12)


def test_softmax_regression_closed_form():
    # one linear layer: dW = X^T (P - Y) / b, dbias = colsum(P - Y) / b
    spec = synth.mlp_spec([6, 4], "f32")
    rng = np.random.default_rng(4)
    X = rng.standard_normal((7, 6)); y = rng.integers(0, 4, 7)
    params = rand_params(spec, 1)
    W, b = params[0]
    Pm = scipy.special.softmax(X @ W + b, axis=1)
    Y = np.eye(4)[y]
    _, g = on.loss_and_gradient(spec, params, X, y)
    np.testing.assert_allclose(g[0][0], X.T @ (Pm - Y) / 7, atol=1e-13)
    np.testing.assert_allclose(g[0][1], (Pm - Y).sum(0) / 7, atol=1e-13)


def test_dlogits_rows_sum_to_zero_and_probabilities_to_one():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((5, 9)) * 30
    y = rng.integers(0, 9, 5)
    loss, dz = on.softmax_xent(z, y)
    assert np.all(np.abs(dz.sum(axis=1)) < 1e-15)
    assert np.isfinite(loss)
    want = -np.mean(scipy.special.log_softmax(z, axis=1)[np.arange(5), y])
    assert abs(loss - want) < 1e-12


def test_relu_derivative_at_zero_is_zero():
    spec = synth.mlp_spec([2, 2, 2], "f32")
    params = [(np.eye(2), np.zeros(2)), (np.ones((2, 2)), np.zeros(2))]
    x = np.array([[0.0, 1.0]])           # first hidden unit sits exactly at 0
    _, g = on.loss_and_gradient(spec, params, x, np.array([0]))
    assert np.all(g[0][0][:, 0] == 0.0) and g[0][1][0] == 0.0


@pytest.mark.parametrize("make_spec", [tiny_mlp, tiny_cnn])
def test_weighted_average_over_any_split_is_the_full_batch_gradient(make_spec):
    spec = make_spec()
    rng = np.random.default_rng(9)
    params = rand_params(spec, 2)
    n = 12
    x = rng.standard_normal((n,) + tuple(spec["input"])); y = rng.integers(0, 3, n)
    _, full = on.loss_and_gradient(spec, params, x, y)
    for b in ([12], [6, 6], [1, 11], [5, 0, 7], [1, 1, 1, 9], [3, 3, 3, 3], [0, 12, 0]):
        _, gk = on.worker_gradients(spec, params, x, y, b)
        agg = on.weighted_aggregate(gk, b)
        for (aW, ab), (fW, fb) in zip(agg, full):
            np.testing.assert_allclose(aW, fW, atol=1e-12)
            np.testing.assert_allclose(ab, fb, atol=1e-12)


def test_equal_split_reduces_to_the_plain_mean_of_eq1():
    spec = tiny_mlp()
    rng = np.random.default_rng(1)
    params = rand_params(spec, 3)
    x = rng.standard_normal((8, 5)); y = rng.integers(0, 3, 8)
    _, gk = on.worker_gradients(spec, params, x, y, [2, 2, 2, 2])
    agg = on.weighted_aggregate(gk, [2, 2, 2, 2])
    for li in range(len(params)):
        np.testing.assert_allclose(agg[li][0], sum(g[li][0] for g in gk) / 4, atol=1e-14)
    # Eq. 1 is written with per-worker gradient *sums*: (1/K)(1/b) sum_k sum_i grad_i
    sums = [[(2 * dW, 2 * db) for dW, db in g] for g in gk]
    for li in range(len(params)):
        eq1 = sum(s[li][0] for s in sums) / 4 / 2
        np.testing.assert_allclose(agg[li][0], eq1, atol=1e-14)


def test_lambda_sums_to_one_via_constant_gradients():
    g = [[(np.ones((2, 2)), np.ones(2))] for _ in range(3)]
    agg = on.weighted_aggregate(g, [5, 1, 10])
    np.testing.assert_allclose(agg[0][0], 1.0, atol=1e-15)


def test_sgd_and_momentum_closed_forms():
    p = [(np.zeros((2, 2)), np.zeros(2))]
    g = [(np.ones((2, 2)), np.ones(2))]
    q = on.sgd_update(p, g, 0.1)
    np.testing.assert_allclose(q[0][0], -0.1); np.testing.assert_allclose(q[0][1], -0.1)
    v = on.zeros_like_params(p)
    mu, lr = 0.9, 0.05
    x_expected = 0.0
    for n in range(1, 8):
        p, v = on.momentum_update(p, v, g, lr, mu)
        vn = (1 - mu ** n) / (1 - mu)              # v_n = g (1 - mu^n) / (1 - mu)
        np.testing.assert_allclose(v[0][0], vn, rtol=1e-13)
        x_expected -= lr * vn
        np.testing.assert_allclose(p[0][0], x_expected, rtol=1e-12)


def test_bf16_rounding_matches_torch_and_ties_go_to_even():
    vals = np.array([1.0, 1 + 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -16, 1 + 3 * 2.0 ** -8,
                     -0.1, 3.14159, 1e-30, 65504.0, 0.0], np.float32)
    want = np.array([1.0, 1.0, 1.0078125, 1.015625], np.float64)
    got = on.round_bf16(vals)
    np.testing.assert_array_equal(got[:4], want)
    rng = np.random.default_rng(0)
    r = (rng.standard_normal(10000) * 10.0 ** rng.integers(-5, 5, 10000)).astype(np.float32)
    t = torch.from_numpy(r).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(on.round_bf16(r), t)


def test_bf16_emulation_stays_close_to_the_exact_gradient():
    spec = synth.mlp_spec([32, 16, 16, 5], "bf16")
    params = synth.init_params(spec, "he", 3)
    x, y = synth.make_batch(spec, "normal", 24, 3, 0)
    _, g = on.loss_and_gradient(spec, params, x, y)
    _, ge = on.loss_and_gradient(spec, params, x, y, emulate_bf16=True)
    for (a, _), (e, _) in zip(g, ge):
        assert np.max(np.abs(a - e)) / np.max(np.abs(a)) < 2e-2


def test_ambiguous_units_are_exactly_the_near_ties():
    spec = synth.mlp_spec([4, 3, 2], "f32")
    W1 = np.array([[1.0, 1.0, 1.0], [1.0, -1.0, 0.5], [0.0, 0.0, 0.0], [0.0, 0.0, 0.0]])
    params = [(W1, np.zeros(3)), (np.ones((3, 2)), np.zeros(2))]
    x = np.array([[1.0, 1.0, 0, 0],            # unit 1: z = 0 exactly
                  [1.0, 1.0 - 1e-7, 0, 0],      # unit 1: z = 1e-7, inside the noise band
                  [1.0, 1.0 - 1e-3, 0, 0],      # unit 1: z = 1e-3, far outside
                  [1.0, 0.5, 0, 0]])
    amb = on.ambiguous_relu_units(spec, params, x)
    assert list(amb) == [0]
    np.testing.assert_array_equal(amb[0], [[0, 1, 0], [0, 1, 0], [0, 0, 0], [0, 0, 0]])


def test_bf16_rounding_boundaries_widen_the_next_layers_band():
    # layer-1 output 1 + 2^-8 sits exactly on a bfloat16 rounding boundary: the stored value
    # may be 1 or 1 + 2^-7, so a layer-2 unit with |z| below 2^-7 |w| is ambiguous -- but only
    # when rounding is emulated
    spec = synth.mlp_spec([1, 1, 1, 1], "bf16")
    w2 = 0.5
    params = [(np.array([[1.0]]), np.zeros(1)), (np.array([[w2]]), np.array([-w2 * (1 + 2.0 ** -8)])),
              (np.ones((1, 1)), np.zeros(1))]
    x = np.array([[1.0 + 2.0 ** -8]])
    params_e = [(W, b) for W, b in params]
    amb = on.ambiguous_relu_units(spec, params_e, x, emulate_bf16=False)
    assert not amb[0][0, 0] and amb[1][0, 0]          # exact: z2 = 0 -> tie
    params_e[1] = (params[1][0], np.array([-w2 * (1 + 2.0 ** -8) + 2.0 ** -10]))
    assert not on.ambiguous_relu_units(spec, params_e, x, emulate_bf16=False)[1][0, 0]
    # emulated: x rounds to 1.0 (ties to even) exactly, layer 1 stores 1.0: no ambiguity there;
    # make layer 1 produce the boundary value through its bias instead
    params_b = [(np.array([[1.0]]), np.array([2.0 ** -8])), (np.array([[w2]]), np.array([-w2 + 2.0 ** -10])),
                (np.ones((1, 1)), np.zeros(1))]
    amb = on.ambiguous_relu_units(spec, params_b, np.array([[1.0]]), emulate_bf16=True)
    assert amb[1][0, 0]                                 # |z2| ~ 2^-10 < 2^-7 * 0.5


def test_forced_relu_masks_change_exactly_the_flipped_units_contribution():
    spec = tiny_mlp()
    rng = np.random.default_rng(12)
    params = rand_params(spec, 4)
    x = rng.standard_normal((3, 5)); y = rng.integers(0, 3, 3)
    masks = on.relu_masks_of(spec, params, x)
    trace = {}
    _, g0 = on.loss_and_gradient(spec, params, x, y, relu_masks=masks, trace=trace)
    _, g_plain = on.loss_and_gradient(spec, params, x, y)
    for (a, b), (c, d) in zip(g0, g_plain):
        np.testing.assert_array_equal(a, c); np.testing.assert_array_equal(b, d)
    # flip unit (sample 1, unit 2) of the second hidden layer (layer index 1)
    m2 = {k: v.copy() for k, v in masks.items()}
    was_on = m2[1][1, 2]
    m2[1][1, 2] = not was_on
    _, g1 = on.loss_and_gradient(spec, params, x, y, relu_masks=m2)
    a_in, incoming = trace[1]
    sign = -1.0 if was_on else 1.0
    want = np.zeros_like(g0[1][0]); want[:, 2] = sign * a_in[1] * incoming[1, 2]
    np.testing.assert_allclose(g1[1][0] - g0[1][0], want, atol=1e-14)
    np.testing.assert_allclose(g1[2][0], g0[2][0], atol=0)          # layers above: untouched


def test_adam_closed_forms():
    rng = np.random.default_rng(9)
    W = rng.normal(size=(5, 3)); b = rng.normal(size=3)
    gW = rng.normal(size=(5, 3)); gb = rng.normal(size=3)
    z = on.zeros_like_params([(W, b)])
    # first step from zero state: bias correction makes m_hat = g, v_hat = g^2
    p, m, v = on.adam_update([(W, b)], z, z, [(gW, gb)], lr=1e-2, eps=1e-8, t=1)
    np.testing.assert_allclose(p[0][0], W - 1e-2 * gW / (np.abs(gW) + 1e-8), rtol=1e-12)
    np.testing.assert_allclose(p[0][1], b - 1e-2 * gb / (np.abs(gb) + 1e-8), rtol=1e-12)
    np.testing.assert_allclose(m[0][0], 0.1 * gW, rtol=1e-12)
    np.testing.assert_allclose(v[0][0], 0.001 * gW * gW, rtol=1e-12)
    # a constant gradient keeps m_hat = g and v_hat = g^2 at every step: x_t = x_0 - t lr g/(|g|+eps)
    params, mm, vv = [(W, b)], z, z
    for t in range(1, 8):
        params, mm, vv = on.adam_update(params, mm, vv, [(gW, gb)], lr=1e-3, eps=1e-6, t=t)
    np.testing.assert_allclose(params[0][0], W - 7 * 1e-3 * gW / (np.abs(gW) + 1e-6), rtol=1e-10)
    # eps = 0: the step does not depend on the gradient's scale; its sign opposes the gradient
    p1, _, _ = on.adam_update([(W, b)], z, z, [(gW, gb)], lr=1e-2, eps=0.0, t=1)
    p2, _, _ = on.adam_update([(W, b)], z, z, [(1e3 * gW, 1e3 * gb)], lr=1e-2, eps=0.0, t=1)
    np.testing.assert_allclose(p1[0][0], p2[0][0], rtol=1e-12)
    assert np.all(np.sign(W - p1[0][0]) == np.sign(gW))
    # two different gradients, second step, one scalar worked by hand:
    # g1 = 1, g2 = 3: m = 0.9*0.1 + 0.1*3 = 0.39, v = 0.999*0.001 + 0.001*9 = 0.009999
    # m_hat = 0.39/0.19, v_hat = 0.009999/0.001999
    one = [(np.array([[0.0]]), np.array([0.0]))]
    p, m, v = on.adam_update(one, on.zeros_like_params(one), on.zeros_like_params(one),
                             [(np.array([[1.0]]), np.array([1.0]))], lr=0.0, t=1)
    p, m, v = on.adam_update(p, m, v, [(np.array([[3.0]]), np.array([3.0]))], lr=0.5, eps=0.0, t=2)
    want = -0.5 * (0.39 / 0.19) / np.sqrt(0.009999 / 0.001999)
    assert abs(p[0][0][0, 0] - want) < 1e-12


def test_stepwise_learning_rate_uses_the_papers_values():
    values = [0.1, 0.01, 0.001, 0.0002]
    bounds = [100, 150, 200]
    got = [on.stepwise_learning_rate(s, bounds, values) for s in (0, 99, 100, 149, 150, 199, 200, 10**6)]
    assert got == [0.1, 0.1, 0.01, 0.01, 0.001, 0.001, 0.0002, 0.0002]
    assert on.stepwise_learning_rate(5, [], [0.3]) == 0.3


def test_batchnorm_textbook_properties():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((6, 3, 2, 5)) * 3.0 + 1.5
    gamma, beta = rng.standard_normal(5), rng.standard_normal(5)
    y, xhat, rstd = on.batchnorm_forward(x, gamma, beta, 0.0)
    # normalised activations: zero mean, unit (biased) variance per channel; y is affine in xhat
    np.testing.assert_allclose(xhat.mean(axis=(0, 1, 2)), 0.0, atol=1e-12)
    np.testing.assert_allclose((xhat ** 2).mean(axis=(0, 1, 2)), 1.0, rtol=1e-12)
    np.testing.assert_allclose(y, gamma * xhat + beta, rtol=1e-12)
    # against the library routine (training mode, biased variance, eps as given)
    t = torch.nn.functional.batch_norm(torch.from_numpy(x).permute(0, 3, 1, 2), None, None,
                                       torch.from_numpy(gamma), torch.from_numpy(beta),
                                       training=True, eps=1e-5)
    y5 = on.batchnorm_forward(x, gamma, beta, 1e-5)[0]
    np.testing.assert_allclose(y5, t.permute(0, 2, 3, 1).numpy(), rtol=1e-10, atol=1e-10)
    # invariance: shifting and scaling a channel of the input does not change the output
    y2 = on.batchnorm_forward(x * 7.0 - 3.0, gamma, beta, 0.0)[0]
    np.testing.assert_allclose(y2, y, rtol=1e-10, atol=1e-10)
    # the input gradient is orthogonal to the two directions the layer ignores
    dy = rng.standard_normal(x.shape)
    dx, dgamma, dbeta = on.batchnorm_backward(dy, xhat, rstd, gamma)
    np.testing.assert_allclose(dx.sum(axis=(0, 1, 2)), 0.0, atol=1e-10)
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 1, 2)), 0.0, atol=1e-10)
    np.testing.assert_allclose(dbeta, dy.sum(axis=(0, 1, 2)), rtol=1e-12)
    # and matches autograd of the library routine
    xt = torch.from_numpy(x).permute(0, 3, 1, 2).clone().requires_grad_(True)
    gt = torch.from_numpy(gamma).clone().requires_grad_(True)
    bt = torch.from_numpy(beta).clone().requires_grad_(True)
    out = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=1e-5)
    out.backward(torch.from_numpy(dy).permute(0, 3, 1, 2))
    _, xhat5, rstd5 = on.batchnorm_forward(x, gamma, beta, 1e-5)
    dx5, dgamma5, _ = on.batchnorm_backward(dy, xhat5, rstd5, gamma)
    np.testing.assert_allclose(dx5, xt.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(dgamma5, gt.grad.numpy(), rtol=1e-10)


def test_batchnorm_statistics_are_per_worker_so_split_invariance_is_lost():
    # the weighted average over workers is NOT the whole-batch gradient once a layer normalises
    # over each worker's own samples; with a single worker it trivially is
    spec = tiny_resnet()
    params = rand_params(spec, 2)
    rng = np.random.default_rng(4)
    x = rng.standard_normal((8,) + tuple(spec["input"])); y = rng.integers(0, 3, 8)
    _, whole = on.worker_gradients(spec, params, x, y, [8])
    _, parts = on.worker_gradients(spec, params, x, y, [5, 3])
    agg = on.weighted_aggregate(parts, [5, 3])
    diff = max(np.max(np.abs(a[0] - w[0])) for a, w in zip(agg, whole[0]))
    assert diff > 1e-3
    one = on.weighted_aggregate(whole, [8])
    assert max(np.max(np.abs(a[0] - w[0])) for a, w in zip(one, whole[0])) < 1e-15


def test_residual_add_sends_the_same_gradient_down_both_branches():
    # y = a + skip with no ReLU anywhere in between: d/d(skip source) gets the sum of both paths
    spec = {"dtype": "f32", "input": (3, 3, 2), "classes": 2,
            "layers": [synth.conv3x3(2, 2, 1, relu=False), synth.conv3x3(2, 2, 1, relu=False),
                       synth.add(0, relu=False), synth.gap(), synth.dense(2, 2, relu=False)]}
    rng = np.random.default_rng(6)
    params = rand_params(spec, 7)
    x = rng.standard_normal((2, 3, 3, 2)); y = rng.integers(0, 2, 2)
    _, g = on.loss_and_gradient(spec, params, x, y)
    # zeroing the second convolution leaves the identity path: layer 0's gradient is then the
    # gradient of the network conv -> pool -> classifier
    params0 = [params[0], (np.zeros_like(params[1][0]), np.zeros_like(params[1][1])), params[2]]
    plain = {"dtype": "f32", "input": (3, 3, 2), "classes": 2,
             "layers": [synth.conv3x3(2, 2, 1, relu=False), synth.gap(), synth.dense(2, 2, relu=False)]}
    _, g0 = on.loss_and_gradient(spec, params0, x, y)
    _, gp = on.loss_and_gradient(plain, [params[0], params[2]], x, y)
    np.testing.assert_allclose(g0[0][0], gp[0][0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g0[2][0], gp[1][0], rtol=1e-12, atol=1e-14)
    assert np.max(np.abs(g[0][0] - gp[0][0])) > 1e-6      # with the branch it differs


# --------------------------------------------------------------------------
# asynchronous (stale-gradient) variant
# --------------------------------------------------------------------------
def test_asynchronous_updates_follow_the_delay_recurrence_on_a_quadratic():
    # f(w) = a w^2 / 2 for both workers, arrivals alternate 0,1,0,1,...: every gradient but the
    # first two is one update stale, w_{t+1} = w_t - c w_{t-1} with c = eta a, whose solution is
    # A r1^t + B r2^t with r = (1 +- sqrt(1 - 4c)) / 2 (textbook linear recurrence)
    a, eta, w0 = 2.0, 0.1, 3.0
    c = eta * a
    grad = lambda k, p: [(a * p[0][0], 0.0 * p[0][1])]
    steps = 12
    got = on.asynchronous_updates(grad, [(np.array([w0]), np.array([0.0]))], [t % 2 for t in range(steps)], eta)
    # arrivals: t=0 worker 0 at w0 -> w1 = w0 - c w0; t=1 worker 1 at w0 (never pulled) -> w2 = w1 - c w0;
    # from then on the arriving worker pulled two arrivals ago: w_{t+1} = w_t - c w_{t-1}
    w1 = w0 - c * w0
    r1, r2 = (1 + np.sqrt(1 - 4 * c)) / 2, (1 - np.sqrt(1 - 4 * c)) / 2
    B = (w1 - w0 * r1) / (r2 - r1)
    A = w0 - B
    assert got[0][0][0] == pytest.approx(A * r1 ** steps + B * r2 ** steps, rel=1e-12)


def test_asynchronous_updates_with_one_worker_are_plain_sgd():
    spec = synth.mlp_spec([6, 5, 3], "f32")
    params = synth.init_params(spec, "he", 4)
    x, y = synth.make_batch(spec, "normal", 7, 4, 0)
    grad = lambda k, p: on.loss_and_gradient(spec, p, x, y)[1]
    got = on.asynchronous_updates(grad, params, [0, 0, 0], 0.05)
    want = params
    for _ in range(3):
        want = on.sgd_update(want, on.loss_and_gradient(spec, want, x, y)[1], 0.05)
    for (gW, gb), (wW, wb) in zip(got, want):
        assert np.array_equal(gW, wW) and np.array_equal(gb, wb)


def test_asynchronous_updates_use_stale_parameters():
    # two workers, worker 1 arrives after two updates by worker 0: its gradient must be the one
    # at the START parameters, not at the current ones (a dropped snapshot would pass the other two)
    a, eta = 1.5, 0.2
    seen = []
    def grad(k, p):
        seen.append((k, float(p[0][0][0])))
        return [(a * p[0][0], 0.0 * p[0][1])]
    on.asynchronous_updates(grad, [(np.array([1.0]), np.array([0.0]))], [0, 0, 1, 1], eta)
    assert seen[0] == (0, 1.0)
    assert seen[1][1] == pytest.approx(1.0 - eta * a)          # worker 0 pulled after its update
    assert seen[2] == (1, 1.0)                                  # worker 1 still holds the start
    assert seen[3][0] == 1 and seen[3][1] != 1.0                # and has pulled since
