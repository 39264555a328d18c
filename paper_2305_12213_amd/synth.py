"""Seeded synthetic inputs and workload descriptions.

This module holds *descriptions* (model shapes, worker speed profiles,
controller constants) and *random draws* (parameters, batches, labels).  It
contains none of the method's arithmetic: no forward/backward pass, no
aggregation, no update and no controller rule live here, so that the GPU path
and the CPU checker can both be fed from it without sharing any computation.

The workloads stand in for the image-classification and linear workloads of
the paper's evaluation section (CIFAR-10-shaped 32x32x3 inputs with 10
classes, a small linear model): only the shapes are borrowed, every value is
drawn from a seeded generator.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 12213


def dense(n_in, n_out, relu):
    return {"kind": "dense", "in": int(n_in), "out": int(n_out), "relu": bool(relu)}


def conv3x3(cin, cout, stride, relu=True):
    return {"kind": "conv3x3", "cin": int(cin), "cout": int(cout),
            "stride": int(stride), "relu": bool(relu)}


def gap():
    return {"kind": "gap"}


def batchnorm(channels, relu, eps=1e-5):
    """Batch normalisation over each worker's own rows (samples x pixels), learnable scale
    and shift per channel, optional ReLU."""
    return {"kind": "bn", "channels": int(channels), "relu": bool(relu), "eps": float(eps)}


def add(skip_from, relu):
    """Residual connection: adds the output of layer `skip_from` (same shape), optional ReLU."""
    return {"kind": "add", "skip_from": int(skip_from), "relu": bool(relu)}


def resnet_block_spec(channels=16, image=(8, 8, 3), classes=10, blocks=1):
    """conv stem, then `blocks` basic residual blocks (conv-BN-ReLU-conv-BN, + skip, ReLU),
    global average pool and a linear classifier (the shape of the paper's ResNet workload,
    scaled down; bf16)."""
    C = int(channels)
    layers = [conv3x3(image[2], C, 1, relu=True)]
    for _ in range(blocks):
        src = len(layers) - 1
        layers += [conv3x3(C, C, 1, relu=False), batchnorm(C, relu=True),
                   conv3x3(C, C, 1, relu=False), batchnorm(C, relu=False),
                   add(src, relu=True)]
    layers += [gap(), dense(C, classes, relu=False)]
    return {"dtype": "bf16", "input": tuple(image), "layers": layers, "classes": int(classes)}


def mlp_spec(dims, dtype):
    layers = [dense(dims[i], dims[i + 1], relu=(i + 2 < len(dims)))
              for i in range(len(dims) - 1)]
    return {"dtype": dtype, "input": (int(dims[0]),), "layers": layers,
            "classes": int(dims[-1])}


def cnn_spec(dtype="bf16"):
    layers = [conv3x3(3, 32, 1), conv3x3(32, 64, 2), conv3x3(64, 128, 2), gap(),
              dense(128, 10, relu=False)]
    return {"dtype": dtype, "input": (32, 32, 3), "layers": layers, "classes": 10}


def _cfg4_speeds():
    return [0.004 ** (k / 15.0) for k in range(16)]


def _cfg2_speeds():
    rng = np.random.Generator(np.random.PCG64([BASE_SEED + 2, 777]))
    return [float(v) for v in rng.choice([1.0, 0.5, 0.25], size=8)]


def config(i):
    """Workload i: the five benchmark/parity workloads, and (5) a residual network with batch
    normalisation at the image size of the paper's ResNet workload."""
    if i == 0:
        return dict(index=0, name="softmax-regression 64-10 fp32",
                    spec=mlp_spec([64, 10], "f32"), x_dist="normal", init="normal0.01",
                    K=2, speeds=[1.0, 0.5], global_batch=64, b0=[32, 32],
                    gains=dict(kp=1.0, deadband=0.05, b_min=1, b_max=64, ewma_alpha=1.0),
                    lr=0.1, momentum=0.0, steps=10)
    if i == 1:
        return dict(index=1, name="MLP 3072-512-512-10 fp32",
                    spec=mlp_spec([3072, 512, 512, 10], "f32"), x_dist="uniform", init="he",
                    K=4, speeds=[1.0, 1.0, 0.5, 0.25], global_batch=256, b0=[64] * 4,
                    gains=dict(kp=0.5, deadband=0.05, b_min=1, b_max=256, ewma_alpha=1.0),
                    lr=0.05, momentum=0.0, steps=50)
    if i == 2:
        return dict(index=2, name="MLP 3072-1024-1024-10 bf16",
                    spec=mlp_spec([3072, 1024, 1024, 10], "bf16"), x_dist="uniform", init="he",
                    K=8, speeds=_cfg2_speeds(), global_batch=1024, b0=[128] * 8,
                    gains=dict(kp=1.0, deadband=0.05, b_min=1, b_max=1024, ewma_alpha=1.0),
                    lr=0.05, momentum=0.9, steps=100)
    if i == 3:
        return dict(index=3, name="CNN 3-32-64-128-GAP-10 bf16 NHWC",
                    spec=cnn_spec("bf16"), x_dist="uniform", init="he",
                    K=4, speeds=[1.0, 0.4, 0.2, 0.08], global_batch=512,
                    b0=[300, 128, 61, 23],
                    gains=dict(kp=1.0, deadband=0.05, b_min=1, b_max=512, ewma_alpha=1.0),
                    lr=0.05, momentum=0.0, steps=50)
    if i == 4:
        return dict(index=4, name="MLP 4096-4096-4096-4096-1000 bf16",
                    spec=mlp_spec([4096, 4096, 4096, 4096, 1000], "bf16"), x_dist="normal",
                    init="he", K=16, speeds=_cfg4_speeds(), global_batch=4096, b0=[256] * 16,
                    gains=dict(kp=1.0, deadband=0.05, b_min=1, b_max=4096, ewma_alpha=1.0),
                    lr=0.01, momentum=0.0, steps=20)
    if i == 5:
        return dict(index=5, name="residual CNN 3 blocks x 64 channels, 32x32x3, batch-norm, bf16 NHWC",
                    spec=resnet_block_spec(64, (32, 32, 3), 10, 3), x_dist="uniform", init="he",
                    K=8, speeds=[1.0, 1.0, 0.5, 0.5, 0.25, 0.25, 0.125, 0.0625],
                    global_batch=512, b0=[64] * 8,
                    gains=dict(kp=1.0, deadband=0.05, b_min=1, b_max=512, ewma_alpha=1.0),
                    lr=0.1, momentum=0.9, steps=20)
    raise ValueError("config index must be 0..5")


def param_shapes(spec):
    """[(W_shape, bias_shape)] for every layer that has parameters, in order."""
    shapes = []
    for L in spec["layers"]:
        if L["kind"] == "dense":
            shapes.append(((L["in"], L["out"]), (L["out"],)))
        elif L["kind"] == "conv3x3":
            shapes.append(((3, 3, L["cin"], L["cout"]), (L["cout"],)))
        elif L["kind"] == "bn":                      # scale ("W") and shift ("bias")
            shapes.append(((L["channels"],), (L["channels"],)))
    return shapes


def n_params(spec):
    return sum(int(np.prod(w)) + int(np.prod(b)) for w, b in param_shapes(spec))


def init_params(spec, init, seed):
    """Random initial parameters as a list of (W, bias) float32 arrays.

    'he'         : W ~ N(0, 2/fan_in), bias 0
    'normal0.01' : W ~ N(0, 0.01^2),   bias 0
    """
    rng = np.random.Generator(np.random.PCG64([int(seed), 1]))
    out = []
    for wshape, bshape in param_shapes(spec):
        if len(wshape) == 1:                         # batch-norm scale 1, shift 0
            out.append((np.ones(wshape, np.float32), np.zeros(bshape, np.float32)))
            continue
        fan_in = int(np.prod(wshape[:-1]))
        std = np.sqrt(2.0 / fan_in) if init == "he" else 0.01
        W = (rng.standard_normal(wshape) * std).astype(np.float32)
        out.append((W, np.zeros(bshape, np.float32)))
    return out


def make_batch(spec, x_dist, n, seed, step):
    """One global batch: x float32 [n, *input], y int32 [n] uniform over classes."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 2, int(step)]))
    shape = (int(n),) + tuple(spec["input"])
    if x_dist == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
    else:
        x = rng.random(shape, dtype=np.float32)
    y = rng.integers(0, spec["classes"], size=int(n)).astype(np.int32)
    return x, y


def flatten_params(params, pad_to=1):
    """Concatenate (W, bias) pairs, layer by layer, into one float32 vector.

    This is the flat parameter/gradient layout of the C interface: for each
    parametrised layer its W in C order ([in][out], or [3][3][cin][cout]) and
    then its bias; the tail is zero-padded to a multiple of `pad_to`.
    """
    flat = np.concatenate([np.concatenate([np.asarray(W, np.float32).ravel(),
                                           np.asarray(b, np.float32).ravel()])
                           for W, b in params])
    n = flat.size
    n_pad = (n + pad_to - 1) // pad_to * pad_to
    if n_pad != n:
        flat = np.concatenate([flat, np.zeros(n_pad - n, np.float32)])
    return flat


def unflatten_params(spec, flat):
    out, o = [], 0
    for wshape, bshape in param_shapes(spec):
        nw, nb = int(np.prod(wshape)), int(np.prod(bshape))
        W = np.asarray(flat[o:o + nw]).reshape(wshape)
        b = np.asarray(flat[o + nw:o + nw + nb]).reshape(bshape)
        out.append((W, b))
        o += nw + nb
    return out


def iteration_times(b, speeds):
    """Synthetic plant: worker k needs b_k / s_k time units for its batch.

    An idle worker (b_k = 0) reports the mean time of the busy ones, i.e. a
    zero error signal.
    """
    t = [float(bk) / float(s) if bk > 0 else None for bk, s in zip(b, speeds)]
    busy = [v for v in t if v is not None]
    fill = (sum(busy) / len(busy)) if busy else 1.0
    return [v if v is not None else fill for v in t]


def plant_times(b, speeds, overhead=None, knee=None, knee_penalty=1.0, noise=0.0, seed=0,
                step=0):
    """Synthetic plant with the effects the linear model leaves out:

        t_k = (c_k + b_k / s_k * (knee_penalty if b_k > knee_k else 1)) * (1 + noise * u_k)

    c_k is a fixed per-iteration overhead, knee_k the batch size past which worker k's
    throughput falls (memory exhaustion), u_k uniform in [-1, 1) drawn from (seed, step).
    An idle worker reports the mean time of the busy ones.
    """
    K = len(b)
    c = [0.0] * K if overhead is None else [float(v) for v in overhead]
    u = np.random.Generator(np.random.PCG64([int(seed), 5, int(step)])).uniform(-1.0, 1.0, size=K)
    t = []
    for k in range(K):
        if b[k] <= 0:
            t.append(None)
            continue
        work = float(b[k]) / float(speeds[k])
        if knee is not None and knee[k] is not None and b[k] > knee[k]:
            work = work * float(knee_penalty)
        t.append((c[k] + work) * (1.0 + float(noise) * float(u[k])))
    busy = [v for v in t if v is not None]
    fill = (sum(busy) / len(busy)) if busy else 1.0
    return [v if v is not None else fill for v in t]


def ragged_split(total, K, seed):
    """A random K-way split of `total` (entries may be 0), for parity tests."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 3]))
    cuts = np.sort(rng.integers(0, total + 1, size=K - 1))
    edges = np.concatenate([[0], cuts, [total]])
    return [int(v) for v in np.diff(edges)]
