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


def _param_index(spec, li):
    return sum(1 for L in spec["layers"][:li] if L["kind"] in ("dense", "conv3x3"))


def resolved_reference(spec, params, x, y, got, emulate_bf16=False, band=8.0):
    """(reference [(dW, db)], loss, #ambiguous units, #units decided differently from the checker).

    x, y: one worker's mini-batch; got: that worker's gradient under test as [(dW, db)].
    """
    loss, base = on.loss_and_gradient(spec, params, x, y, emulate_bf16)
    if np.shape(x)[0] == 0:
        return base, loss, 0, 0
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
