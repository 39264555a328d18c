"""Reference gradients that are robust to ReLU ties.

relu'(z) is a 0/1 decision on a rounded number.  Two correct implementations (different
summation order; a stored bfloat16 activation that rounds the other way) can decide a unit with
|z| inside the rounding band differently, and one such unit changes a worker's gradient by
O(1/b_k) -- far above any element-wise tolerance.  What is unique is the gradient *given* the
decisions; what is valid is any decision for the units the checker itself finds ambiguous
(oracle.network.ambiguous_relu_units) and the checker's own decision everywhere else.

`resolved_reference` therefore returns the checker's gradient under the admissible decision that
best explains the gradient under test: layer by layer from the top, every ambiguous unit's direct
signature (its column of that layer's weight gradient) is fitted against the residual, and the unit
is flipped when the fit says so.  The result is then compared element-wise, at the ordinary
tolerance, over ALL entries.  Only decisions of ambiguous units are ever changed, so an error
anywhere else still fails.
"""
import numpy as np

from oracle import network as on


PARAM_KINDS = ("dense", "conv3x3", "bn")


def _param_index(spec, li):
    return sum(1 for L in spec["layers"][:li] if L["kind"] in PARAM_KINDS)


def _needs_generic(spec):
    """The column signatures below exist for ReLUs that sit directly on a dense or convolution
    layer; anything else (batch normalisation, residual additions) takes the generic route."""
    return any(L["kind"] in ("bn", "add") for L in spec["layers"])


def _resolved_generic(spec, params, x, y, got, emulate_bf16, band):
    """Same idea with signatures obtained by re-evaluation: flipping one ambiguous unit of a ReLU
    layer changes the gradient by a fixed vector (the backward pass is linear in the gradient
    signal, so the flips of one layer add up).  That vector is measured on the parameters between
    this ReLU layer and the next one below -- they feel this layer's decisions and none of the
    lower layers' -- and the flips are fitted to the residual there."""
    loss, base = on.loss_and_gradient(spec, params, x, y, emulate_bf16)
    amb = on.ambiguous_relu_units(spec, params, x, emulate_bf16, band)
    n_amb = int(sum(a.sum() for a in amb.values()))
    if n_amb == 0:
        return base, loss, 0, 0
    masks = on.relu_masks_of(spec, params, x, emulate_bf16)
    relu_layers = sorted(masks)
    flipped = 0

    def flat(g, pis):
        return np.concatenate([np.concatenate([np.ravel(g[pi][0]), np.ravel(g[pi][1])]) for pi in pis])

    for li in sorted(amb, reverse=True):
        units = [tuple(t) for t in np.argwhere(amb[li])]
        if not units:
            continue
        lower = max([r for r in relu_layers if r < li], default=-1)
        pis = [_param_index(spec, l) for l in range(lower + 1, li + 1)
               if spec["layers"][l]["kind"] in PARAM_KINDS]
        if not pis:
            continue
        _, cur = on.loss_and_gradient(spec, params, x, y, emulate_bf16, relu_masks=masks)
        resid = flat([(np.asarray(W, np.float64), np.asarray(b, np.float64)) for W, b in got], pis) \
            - flat(cur, pis)
        cols = []
        for t in units:
            masks[li][t] ^= True
            _, g1 = on.loss_and_gradient(spec, params, x, y, emulate_bf16, relu_masks=masks)
            masks[li][t] ^= True
            cols.append(flat(g1, pis) - flat(cur, pis))
        S = np.stack(cols, axis=1)
        live = np.abs(S).max(axis=0) > 0
        if not live.any():
            continue
        c = np.zeros(S.shape[1])
        c[live] = np.linalg.lstsq(S[:, live], resid, rcond=None)[0]
        for t, cj in zip(units, c):
            if cj > 0.5:
                masks[li][t] ^= True
                flipped += 1
    _, final = on.loss_and_gradient(spec, params, x, y, emulate_bf16, relu_masks=masks)
    return final, loss, n_amb, flipped


def resolved_reference(spec, params, x, y, got, emulate_bf16=False, band=6.0):
    """(reference [(dW, db)], loss, #ambiguous units, #units decided differently from the checker).

    x, y: one worker's mini-batch; got: that worker's gradient under test as [(dW, db)].
    """
    loss, base = on.loss_and_gradient(spec, params, x, y, emulate_bf16)
    if np.shape(x)[0] == 0:
        return base, loss, 0, 0
    if _needs_generic(spec):
        return _resolved_generic(spec, params, x, y, got, emulate_bf16, band)
    amb = on.ambiguous_relu_units(spec, params, x, emulate_bf16, band)
    n_amb = int(sum(a.sum() for a in amb.values()))
    if n_amb == 0:
        return base, loss, 0, 0
    masks = on.relu_masks_of(spec, params, x, emulate_bf16)
    flipped = 0
    for li in sorted(amb, reverse=True):
        if not amb[li].any():
            continue
        trace = {}
        _, cur = on.loss_and_gradient(spec, params, x, y, emulate_bf16, relu_masks=masks, trace=trace)
        a_in, incoming = trace[li]
        L = spec["layers"][li]
        pi = _param_index(spec, li)
        resid_W = np.asarray(got[pi][0], np.float64) - cur[pi][0]
        resid_b = np.asarray(got[pi][1], np.float64) - cur[pi][1]
        idx = np.argwhere(amb[li])
        chan = idx[:, -1]
        if L["kind"] == "conv3x3":
            a_pad = np.pad(a_in, ((0, 0), (1, 1), (1, 1), (0, 0)))
            s = L["stride"]
        for u in np.unique(chan):
            units = idx[chan == u]
            cols = []
            for t in units:
                t = tuple(t)
                g = incoming[t] * (-1.0 if masks[li][t] else 1.0)
                if L["kind"] == "dense":
                    sig = a_in.reshape(a_in.shape[0], -1)[t[0]]
                else:
                    i, ho, wo, _ = t
                    sig = a_pad[i, ho * s:ho * s + 3, wo * s:wo * s + 3, :].ravel()
                cols.append(np.concatenate([sig * g, [g]]))
            S = np.stack(cols, axis=1)
            if L["kind"] == "dense":
                r = np.concatenate([resid_W[:, u], [resid_b[u]]])
            else:
                r = np.concatenate([resid_W[:, :, :, u].ravel(), [resid_b[u]]])
            live = np.abs(S).max(axis=0) > 0
            if not live.any():
                continue
            c = np.zeros(S.shape[1])
            c[live] = np.linalg.lstsq(S[:, live], r, rcond=None)[0]
            for t, cj in zip(units, c):
                if cj > 0.5:
                    masks[li][tuple(t)] ^= True
                    flipped += 1
    _, final = on.loss_and_gradient(spec, params, x, y, emulate_bf16, relu_masks=masks)
    return final, loss, n_amb, flipped


def resolved_worker_references(spec, params, x, y, b, got_by_worker, emulate_bf16=False):
    """Per worker: resolved reference gradients and losses; plus total (#ambiguous, #flipped)."""
    refs, losses, off, n_amb, n_flip = [], [], 0, 0, 0
    for k, bk in enumerate(b):
        ref, loss, a, f = resolved_reference(spec, params, x[off:off + bk], y[off:off + bk],
                                             got_by_worker[k], emulate_bf16)
        refs.append(ref); losses.append(loss)
        n_amb += a; n_flip += f
        off += bk
    return refs, losses, n_amb, n_flip
