"""CPU checker for the per-worker gradient, its weighted aggregation and the
SGD update.  TEST INFRASTRUCTURE ONLY: nothing in the product path may import
this package; it exists so that the GPU kernels can be compared with a plain,
slow, obviously-correct computation.

Everything is float64 numpy, written as the textbook definition:

* per-worker gradient  grad f(x_{b_k,t})  (Section "Key Idea: Variable
  Mini-Batch Sizes"): the gradient of the mean softmax-cross-entropy loss over
  the worker's own b_k samples, by hand-written back-propagation;
* lambda_k = b_k / sum_i b_i and the weighted average sum_k lambda_k grad_k
  (same section, the lambda definition and Eq. 2);
* x_{t+1} = x_t - eta * sum_k lambda_k grad_k (Eq. 3, with the stray 1/K read
  as a typo: with sum_k lambda_k = 1 the update must reduce to Eq. 1 when all
  b_k are equal), and heavy-ball momentum for the workload that names it.

Pins (tests/test_oracle_network.py): central finite differences, a pure
Python loop convolution, closed forms for softmax regression, the delta-image
convolution, and the split-invariance of the weighted average; the
asynchronous variant by the closed-form solution of its delay recurrence on
a quadratic and by its reduction to plain SGD with one worker.

`emulate_bf16=True` additionally rounds to bfloat16 (round-to-nearest-even)
the quantities a bf16 implementation stores in 16 bits: the weights (not the
biases), the input, every stored hidden activation and every stored
activation-gradient.  Accumulation stays float64.  This switch has no pin of
its own beyond "rounding moves a value by at most 2^-9 relative" (parity
unpinned for the rounding emulation itself; the un-rounded path is pinned).
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# bfloat16 rounding emulation
# --------------------------------------------------------------------------
def round_bf16(a):
    """Round float values to the nearest bfloat16 (ties to even); returns float64."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = r.astype(np.uint32).view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out[nan] = np.nan
    return out.reshape(np.shape(a))


def _q(a, emulate):
    return round_bf16(a) if emulate else a


# --------------------------------------------------------------------------
# layers (forward and backward), float64
# --------------------------------------------------------------------------
def conv3x3_forward(x, W, bias, stride):
    """x [n,H,W,Cin] (NHWC), W [3,3,Cin,Cout], zero padding 1 -> [n,Ho,Wo,Cout]."""
    n, H, Wd, _ = x.shape
    Ho = (H + 2 - 3) // stride + 1
    Wo = (Wd + 2 - 3) // stride + 1
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    out = np.zeros((n, Ho, Wo, W.shape[3])) + bias
    for kh in range(3):
        for kw in range(3):
            patch = xp[:, kh:kh + stride * (Ho - 1) + 1:stride,
                       kw:kw + stride * (Wo - 1) + 1:stride, :]
            out += patch @ W[kh, kw]
    return out


def conv3x3_backward(x, W, dy, stride, need_dx=True):
    """Gradients of conv3x3_forward wrt W, bias and (optionally) x."""
    n, H, Wd, _ = x.shape
    _, Ho, Wo, _ = dy.shape
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    dW = np.zeros_like(W)
    dxp = np.zeros_like(xp)
    for kh in range(3):
        for kw in range(3):
            sl = (slice(None), slice(kh, kh + stride * (Ho - 1) + 1, stride),
                  slice(kw, kw + stride * (Wo - 1) + 1, stride), slice(None))
            patch = xp[sl]
            dW[kh, kw] = np.tensordot(patch, dy, axes=([0, 1, 2], [0, 1, 2]))
            if need_dx:
                dxp[sl] += dy @ W[kh, kw].T
    db = dy.sum(axis=(0, 1, 2))
    dx = dxp[:, 1:-1, 1:-1, :] if need_dx else None
    return dW, db, dx


def softmax_xent(z, y):
    """Mean cross-entropy over the rows of z and its gradient wrt z.

    p = softmax(z) (max-subtracted), loss = -(1/n) sum_i log p[i, y_i],
    dz = (p - onehot(y)) / n.
    """
    n = z.shape[0]
    zs = z - z.max(axis=1, keepdims=True)
    e = np.exp(zs)
    p = e / e.sum(axis=1, keepdims=True)
    loss = -np.mean(np.log(p[np.arange(n), y]))
    dz = p.copy()
    dz[np.arange(n), y] -= 1.0
    return loss, dz / n


def _f64_params(params, emulate):
    # 16-bit copies exist of the matrix weights only; biases and batch-norm scale/shift stay fp32
    return [(_q(np.asarray(W, np.float64), emulate and np.ndim(W) > 1), np.asarray(b, np.float64))
            for W, b in params]


def batchnorm_forward(x, gamma, beta, eps):
    """Batch normalisation (Ioffe & Szegedy, Algorithm 1) over all axes but the last:
    mu, var (biased) per channel; xhat = (x - mu) / sqrt(var + eps); y = gamma xhat + beta.
    The statistics are those of the given mini-batch, i.e. of one worker's own samples.
    Returns (y, xhat, rstd)."""
    axes = tuple(range(x.ndim - 1))
    mu = x.mean(axis=axes)
    var = ((x - mu) ** 2).mean(axis=axes)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, xhat, rstd


def batchnorm_backward(dy, xhat, rstd, gamma):
    """Gradients of batch normalisation given dL/dy: (dx, dgamma, dbeta) with
    dx = gamma rstd (dy - mean(dy) - xhat mean(dy xhat)) (means over the batch axes)."""
    axes = tuple(range(dy.ndim - 1))
    dbeta = dy.sum(axis=axes)
    dgamma = (dy * xhat).sum(axis=axes)
    n = dy.size // dy.shape[-1]
    dx = gamma * rstd * (dy - dbeta / n - xhat * (dgamma / n))
    return dx, dgamma, dbeta


def forward(spec, params, x, emulate_bf16=False):
    """Logits [n, classes] and the list of stored layer inputs (for backward)."""
    P = _f64_params(params, emulate_bf16)
    a = _q(np.asarray(x, np.float64), emulate_bf16)
    stored, pi = [], 0
    n_layers = len(spec["layers"])
    for li, L in enumerate(spec["layers"]):
        last = li == n_layers - 1
        stored.append(a)
        if L["kind"] == "dense":
            W, b = P[pi]; pi += 1
            a = a.reshape(a.shape[0], -1) @ W + b
        elif L["kind"] == "conv3x3":
            W, b = P[pi]; pi += 1
            a = conv3x3_forward(a, W, b, L["stride"])
        elif L["kind"] == "gap":
            a = a.mean(axis=(1, 2))
        elif L["kind"] == "bn":
            gamma, beta = P[pi]; pi += 1
            a = batchnorm_forward(a, gamma, beta, L["eps"])[0]
        elif L["kind"] == "add":
            a = a + stored[L["skip_from"] + 1]   # stored[i + 1] is the stored output of layer i
        else:
            raise ValueError(L["kind"])
        if L.get("relu"):
            a = np.maximum(a, 0.0)
        if not last:
            a = _q(a, emulate_bf16)          # stored hidden activation
    stored.append(a)                          # logits (kept in full precision)
    return a, stored


# A sum of K products accumulated in fp32 differs from the exact sum by a random amount; the
# scale 2^-24 sqrt(K) sqrt(sum_j a_j^2 w_j^2) is called one noise unit below.  Measured on the
# CPU (tests/test_oracle_network.py emulates it): strictly sequential fp32 accumulation has a
# standard deviation of 0.16 noise units, blocked or pairwise orders less.  0.25 is taken.
ACCUMULATION_NOISE = 0.25


def _storage_ulp(v, emulate_bf16):
    """Spacing of the storage format (bfloat16 when emulated, else fp32) at magnitude |v|."""
    v = np.abs(np.asarray(v, np.float64))
    out = np.zeros_like(v)
    nz = v > 0
    out[nz] = 2.0 ** (np.floor(np.log2(v[nz])) - (7 if emulate_bf16 else 23))
    return out


def _largest_single_term(jump, absW, top=16):
    """Upper bound of max_j jump[i, j] * absW[j, k] for every (i, k): exact over each row's `top`
    largest jumps, and (largest remaining jump of the row) * (largest |w| of the column) for the
    rest.  jump >= 0, mostly zero."""
    n, J = jump.shape
    t = min(top, J)
    idx = np.argpartition(-jump, t - 1, axis=1)[:, :t] if t < J else np.tile(np.arange(J), (n, 1))
    best = np.zeros((n, absW.shape[1]))
    rest = jump.copy()
    for c in range(t):
        jc = idx[:, c]
        vals = jump[np.arange(n), jc]
        live = vals > 0
        if live.any():
            best[live] = np.maximum(best[live], vals[live, None] * absW[jc[live]])
        rest[np.arange(n), jc] = 0.0
    return np.maximum(best, rest.max(axis=1)[:, None] * absW.max(axis=0)[None, :])


def _largest_single_term_conv(jump, absW, stride):
    """The same bound for a 3x3 convolution (zero padding 1): rows are the output pixels'
    3 x 3 x Cin patches of `jump`, taken a few samples at a time."""
    n, H, Wd, C = jump.shape
    Ho = (H + 2 - 3) // stride + 1
    Wo = (Wd + 2 - 3) // stride + 1
    out = np.zeros((n, Ho, Wo, absW.shape[3]))
    Wm = absW.reshape(9 * C, -1)
    step = max(1, (1 << 22) // max(1, Ho * Wo * 9 * C))
    for i0 in range(0, n, step):
        jp = np.pad(jump[i0:i0 + step], ((0, 0), (1, 1), (1, 1), (0, 0)))
        if not jp.any():
            continue
        taps = [jp[:, kh:kh + stride * (Ho - 1) + 1:stride, kw:kw + stride * (Wo - 1) + 1:stride, :]
                for kh in range(3) for kw in range(3)]
        rows = np.stack(taps, axis=3).reshape(-1, 9 * C)
        out[i0:i0 + step] = _largest_single_term(rows, Wm).reshape(-1, Ho, Wo, Wm.shape[1])
    return out


def ambiguous_relu_units(spec, params, x, emulate_bf16=False, band=6.0):
    """ReLU units whose 0/1 derivative two correct implementations may decide differently.

    relu'(z) is a decision on a computed number.  Two implementations' values of a
    pre-activation differ by a random dz.  For every stored tensor two things are carried along:

    * var and mad: the variance and the mean absolute value of the difference of the two
      implementations' STORED values.  A pre-activation that differs by dz (standard deviation
      s, mean absolute value e <= 0.8 s), stored in a format whose spacing at that magnitude is
      u, is rounded to different neighbours with probability E|dz| / u (a rounding boundary lies
      between the two values) and then differs by u: the stored values differ by e on average
      again, and var = s^2 + min(e u, u^2).  Mean absolute values add through a layer
      (triangle inequality), e' <= 0.8 (accumulation noise) + mad @ |W|; next to e' <= 0.8 s' this
      matters where upstream differences are rare, so that s' overstates the typical dz'.
    * jump: the largest difference the storage rounding alone can cause with a probability
      worth counting, q(z + band s) - q(z - band s) (zero unless a rounding boundary lies
      inside; always zero for fp32 storage, whose differences are the continuous part already
      counted in var).

    A layer z' = a W + b then has s'^2 = (ACCUMULATION_NOISE noise units)^2 + var @ W^2
    (independent contributions add in variance), and its half-width is
        h' = band * s' + max_j jump_j |W_jk|
    -- `band` standard deviations for the many small contributions, plus, in full, the largest
    single rounding jump: upstream differences are rare (a handful per row) and one of them alone
    can be several standard deviations, which a variance cannot bound.  A unit is ambiguous when
    |z| <= h.  Normalisation, addition and pooling propagate (var, jump) by the same rules.

    Returns {layer index: boolean array shaped like that layer's output}.  Everything outside
    these sets is decided identically by any implementation within the noise model.
    """
    P = _f64_params(params, emulate_bf16)
    a = _q(np.asarray(x, np.float64), emulate_bf16)
    var = np.zeros_like(a)
    mad = np.zeros_like(a)
    jump = np.zeros_like(a)
    n = a.shape[0]
    out, pi = {}, 0
    kept = {}                                   # layer index -> (stored output, var, mad, jump)
    n_layers = len(spec["layers"])
    for li, L in enumerate(spec["layers"]):
        if L["kind"] == "dense":
            W, b = P[pi]; pi += 1
            a2, v2, j2 = a.reshape(n, -1), var.reshape(n, -1), jump.reshape(n, -1)
            z = a2 @ W + b
            unit = 2.0 ** -24 * np.sqrt(W.shape[0]) * np.sqrt((a2 * a2) @ (W * W))
            s = np.sqrt((ACCUMULATION_NOISE * unit) ** 2 + v2 @ (W * W))
            e = 0.8 * ACCUMULATION_NOISE * unit + mad.reshape(n, -1) @ np.abs(W)
            single = _largest_single_term(j2, np.abs(W)) if j2.any() else 0.0
        elif L["kind"] == "conv3x3":
            W, b = P[pi]; pi += 1
            z = conv3x3_forward(a, W, b, L["stride"])
            unit = 2.0 ** -24 * np.sqrt(9 * W.shape[2]) * \
                np.sqrt(conv3x3_forward(a * a, W * W, 0.0, L["stride"]))
            s = np.sqrt((ACCUMULATION_NOISE * unit) ** 2 + conv3x3_forward(var, W * W, 0.0, L["stride"]))
            e = 0.8 * ACCUMULATION_NOISE * unit + conv3x3_forward(mad, np.abs(W), 0.0, L["stride"])
            single = _largest_single_term_conv(jump, np.abs(W), L["stride"])
        elif L["kind"] == "bn":
            # y = gamma (x - mu) rstd + beta over this mini-batch.  dx moves x - mu by dx - mean(dx)
            # and the variance by mean(2 (x - mu) dx): relative to rstd that is a standard
            # deviation of rstd sqrt(mean(var) / m) over the m rows, plus 2^-20 for the fp32
            # statistics of an implementation.
            gamma, beta = P[pi]; pi += 1
            z, xhat, rstd = batchnorm_forward(a, gamma, beta, L["eps"])
            axes = tuple(range(a.ndim - 1))
            m_rows = a.size // a.shape[-1]
            mean_var = var.mean(axis=axes)
            rel = rstd * np.sqrt(mean_var / m_rows) + 2.0 ** -20
            s = np.sqrt((gamma * rstd) ** 2 * (var + mean_var / m_rows) + (gamma * xhat * rel) ** 2
                        + (2.0 ** -22 * z) ** 2)
            single = np.abs(gamma) * rstd * (jump + jump.max(axis=axes) / m_rows)
            e = 0.8 * s
        elif L["kind"] == "add":
            s_a, s_var, s_mad, s_jump = kept[L["skip_from"]]
            z = a + s_a
            s = np.sqrt(var + s_var + (2.0 ** -23 * z) ** 2)
            single = jump + s_jump
            e = mad + s_mad + 2.0 ** -23 * np.abs(z)
        else:                                   # global average pool over m pixels
            m_pix = a.shape[1] * a.shape[2]
            z = a.mean(axis=(1, 2))
            s = np.sqrt(var.mean(axis=(1, 2)) / m_pix + (2.0 ** -22 * z) ** 2)
            single = jump.max(axis=(1, 2)) / m_pix
            e = mad.mean(axis=(1, 2)) + 2.0 ** -22 * np.abs(z)
        e = np.minimum(e, 0.8 * s)
        h = band * s + single
        if L.get("relu"):
            out[li] = np.abs(z) <= h
        if li == n_layers - 1:
            break
        relu = bool(L.get("relu"))
        clip = (lambda t: np.maximum(t, 0.0)) if relu else (lambda t: t)
        a = _q(clip(z), emulate_bf16)
        u = _storage_ulp(clip(z + h) if relu else np.abs(z) + h, emulate_bf16)
        var = s * s + np.minimum(e * u, u * u)
        mad = e
        if relu:                                    # where both implementations store zero
            var = np.where(z + h > 0.0, var, 0.0)
            mad = np.where(z + h > 0.0, mad, 0.0)
        g = band * s          # (not h: a rare jump caused by a rare jump upstream is not counted)
        jump = (_q(clip(z + g), True) - _q(clip(z - g), True)) if emulate_bf16 else np.zeros_like(z)
        kept[li] = (a, var, mad, jump)
    return out


def loss_and_gradient(spec, params, x, y, emulate_bf16=False, relu_masks=None, trace=None):
    """Mean loss over the given samples and its gradient as [(dW, dbias)].

    This is grad f(x_{b_k,t}) for one worker when (x, y) is that worker's
    mini-batch.  An empty mini-batch yields loss 0 and a zero gradient.

    relu_masks ({layer index: boolean array}) replaces the derivative decision
    "stored output > 0" of those layers (used to evaluate the gradient under another
    admissible decision of ambiguous units).  If `trace` is a dict, trace[layer index] =
    (layer input, gradient arriving at the layer output before the ReLU mask) is recorded
    for every ReLU layer.
    """
    n = int(np.shape(x)[0])
    if n == 0:
        return 0.0, [(np.zeros(np.shape(W)), np.zeros(np.shape(b))) for W, b in params]
    P = _f64_params(params, emulate_bf16)
    z, stored = forward(spec, params, x, emulate_bf16)
    loss, dz = softmax_xent(z, np.asarray(y, np.int64))
    da = _q(dz, emulate_bf16)                 # stored dlogits
    grads = [None] * len(P)
    pi = len(P)
    first_param_layer = next(i for i, L in enumerate(spec["layers"])
                             if L["kind"] in ("dense", "conv3x3", "bn"))
    skip_grad = {}                            # layer index -> stored gradient arriving by a skip
    for li in range(len(spec["layers"]) - 1, -1, -1):
        L = spec["layers"][li]
        a_in, a_out = stored[li], stored[li + 1]
        if li in skip_grad:                   # two consumers: both stored gradients, summed, stored
            da = _q(da + skip_grad.pop(li), emulate_bf16)
        if L.get("relu"):
            if trace is not None:
                trace[li] = (a_in, da)
            mask = (a_out > 0.0) if relu_masks is None or li not in relu_masks else relu_masks[li]
            da = da * mask                    # relu'(0) = 0; exact, needs no re-rounding
        need_dx = li > first_param_layer
        if L["kind"] == "dense":
            pi -= 1
            W, _ = P[pi]
            a2 = a_in.reshape(a_in.shape[0], -1)
            grads[pi] = (a2.T @ da, da.sum(axis=0))
            if need_dx:
                da = _q((da @ W.T).reshape(a_in.shape), emulate_bf16)
        elif L["kind"] == "conv3x3":
            pi -= 1
            W, _ = P[pi]
            dW, db, dx = conv3x3_backward(a_in, W, da, L["stride"], need_dx)
            grads[pi] = (dW, db)
            if need_dx:
                da = _q(dx, emulate_bf16)
        elif L["kind"] == "gap":
            _, H, Wd, _ = a_in.shape
            da = _q(np.broadcast_to(da[:, None, None, :] / (H * Wd), a_in.shape), emulate_bf16)
        elif L["kind"] == "bn":
            pi -= 1
            gamma, beta = P[pi]
            _, xhat, rstd = batchnorm_forward(a_in, gamma, beta, L["eps"])
            dx, dgamma, dbeta = batchnorm_backward(da, xhat, rstd, gamma)
            grads[pi] = (dgamma, dbeta)
            if need_dx:
                da = _q(dx, emulate_bf16)
        elif L["kind"] == "add":
            src = L["skip_from"]
            assert src not in skip_grad, "one skip connection per source layer"
            skip_grad[src] = da               # (already a stored value; the main branch keeps da)
    return loss, grads


def relu_masks_of(spec, params, x, emulate_bf16=False):
    """{layer index: stored output > 0} for every ReLU layer (the checker's own decisions)."""
    _, stored = forward(spec, params, x, emulate_bf16)
    return {li: stored[li + 1] > 0.0 for li, L in enumerate(spec["layers"]) if L.get("relu")}


def worker_gradients(spec, params, x, y, b, emulate_bf16=False):
    """Per-worker losses and gradients: worker k owns rows [off_k, off_k + b_k)."""
    losses, grads, off = [], [], 0
    for bk in b:
        l, g = loss_and_gradient(spec, params, x[off:off + bk], y[off:off + bk], emulate_bf16)
        losses.append(l); grads.append(g); off += bk
    assert off == np.shape(x)[0], "sum(b) must equal the number of rows"
    return losses, grads


# --------------------------------------------------------------------------
# aggregation and update
# --------------------------------------------------------------------------
def weighted_aggregate(worker_grads, b):
    """sum_k lambda_k g_k with lambda_k = b_k / sum_i b_i (fixed k order)."""
    total = float(sum(b))
    out = None
    for bk, g in zip(b, worker_grads):
        lam = float(bk) / total
        if out is None:
            out = [(lam * dW, lam * db) for dW, db in g]
        else:
            out = [(oW + lam * dW, ob + lam * db) for (oW, ob), (dW, db) in zip(out, g)]
    return out


def sgd_update(params, g, lr):
    """x <- x - eta * g."""
    return [(np.asarray(W, np.float64) - lr * gW, np.asarray(b, np.float64) - lr * gb)
            for (W, b), (gW, gb) in zip(params, g)]


def asynchronous_updates(gradient_of, params, order, lr):
    """Asynchronous-parallel training as the paper describes it in words (Section "Distributed
    Training": workers push gradients and pull parameters without waiting for one another; no
    update rule is printed).  Reading: the workers arrive in the sequence `order`; an arriving
    worker k delivers the gradient it computed at the parameters it pulled at its previous
    arrival (the start parameters the first time) -- stale by however many other arrivals lay
    in between --, the server applies it at once, x <- x - eta * g_k, and the worker pulls the
    new parameters.  `gradient_of(k, params)` is worker k's gradient in the shape of `params`.
    Returns the final parameters."""
    pulled = {}
    cur = [(np.asarray(W, np.float64), np.asarray(b, np.float64)) for W, b in params]
    for k in order:
        g = gradient_of(k, pulled.get(k, params))
        cur = sgd_update(cur, g, lr)
        pulled[k] = cur
    return cur


def momentum_update(params, velocity, g, lr, mu):
    """Heavy ball: v <- mu v + g ; x <- x - eta v.  Returns (params, velocity)."""
    v = [(mu * vW + gW, mu * vb + gb) for (vW, vb), (gW, gb) in zip(velocity, g)]
    p = [(np.asarray(W, np.float64) - lr * vW, np.asarray(b, np.float64) - lr * vb)
         for (W, b), (vW, vb) in zip(params, v)]
    return p, v


def adam_update(params, m, v, g, lr, beta1=0.9, beta2=0.999, eps=1e-8, t=1):
    """Adam (Kingma & Ba, Algorithm 1; the optimizer the paper names for its MNIST workload),
    step number t >= 1:
        m <- beta1 m + (1 - beta1) g ;  v <- beta2 v + (1 - beta2) g^2
        x <- x - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
    Returns (params, m, v)."""
    c1 = 1.0 - beta1 ** t
    c2 = 1.0 - beta2 ** t
    def one(x, mm, vv, gg):
        x = np.asarray(x, np.float64); gg = np.asarray(gg, np.float64)
        mm = beta1 * np.asarray(mm, np.float64) + (1.0 - beta1) * gg
        vv = beta2 * np.asarray(vv, np.float64) + (1.0 - beta2) * gg * gg
        return x - lr * (mm / c1) / (np.sqrt(vv / c2) + eps), mm, vv
    out_p, out_m, out_v = [], [], []
    for (W, b), (mW, mb), (vW, vb), (gW, gb) in zip(params, m, v, g):
        pW, nmW, nvW = one(W, mW, vW, gW)
        pb, nmb, nvb = one(b, mb, vb, gb)
        out_p.append((pW, pb)); out_m.append((nmW, nmb)); out_v.append((nvW, nvb))
    return out_p, out_m, out_v


def stepwise_learning_rate(step, boundaries, values):
    """Piecewise-constant schedule (the paper lists the values [0.1, 0.01, 0.001, 0.0002] for
    its ResNet workload, not the switching points): values[i] holds for
    boundaries[i-1] <= step < boundaries[i]."""
    i = 0
    while i < len(boundaries) and step >= boundaries[i]:
        i += 1
    return float(values[i])


def zeros_like_params(params):
    return [(np.zeros(np.shape(W)), np.zeros(np.shape(b))) for W, b in params]
