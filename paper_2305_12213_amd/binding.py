"""ctypes binding of include/dynb.h: argument marshalling only.

Device arguments are anything with a ``data_ptr()`` (torch tensors) or plain
integer addresses; ``stream`` is a raw hipStream_t value (``None`` picks
torch's current stream when torch is importable and a GPU is present, else
the default stream).  Every function raises ``DynbError`` on a non-zero
status.  There is no fallback: if the HIP library is missing, ``load()``
raises.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdynb.so")

F32, BF16 = 0, 1
LAYER_DENSE, LAYER_CONV3X3, LAYER_GAP, LAYER_BN, LAYER_ADD = 0, 1, 2, 3, 4
MAX_WORKERS = 64

SYMBOLS = [
    "dynb_last_error", "dynb_model_create", "dynb_model_destroy", "dynb_model_num_params",
    "dynb_model_padded_params", "dynb_model_workspace_bytes", "dynb_model_bind",
    "dynb_model_sync_weights", "dynb_model_worker_loss", "dynb_model_read_worker_loss", "dynb_forward_backward", "dynb_forward_backward_aggregate",
    "dynb_weighted_aggregate", "dynb_sgd_update", "dynb_sgd_momentum_update",
    "dynb_model_sgd_update", "dynb_controller_step", "dynb_ewma_update", "dynb_static_allocate",
    "dynb_adam_update", "dynb_model_update", "dynb_model_aggregate_update", "dynb_lr_schedule",
    "dynb_controller_create", "dynb_controller_destroy", "dynb_controller_observe",
    "dynb_controller_read",
    "dynb_profile_enable", "dynb_profile_reset", "dynb_profile_collect",
    "dynb_profile_num_classes", "dynb_profile_name", "dynb_profile_get",
    "dynb_static_scratch_bytes", "dynb_forward_backward_static", "dynb_estimate_throughput",
]


class DynbError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("dynb error %d: %s" % (code, message))
        self.code = code


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_in", C.c_int32), ("n_out", C.c_int32),
                ("stride", C.c_int32), ("relu", C.c_int32), ("skip_from", C.c_int32),
                ("eps", C.c_float)]


class ModelDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("in_c", C.c_int32), ("n_classes", C.c_int32), ("n_layers", C.c_int32),
                ("layers", C.POINTER(LayerDesc))]


class Gains(C.Structure):
    _fields_ = [("kp", C.c_double), ("deadband", C.c_double), ("ewma_alpha", C.c_double),
                ("b_min", C.c_int32), ("b_max", C.c_int32)]


OPT_SGD, OPT_MOMENTUM, OPT_ADAM = 0, 1, 2


class Optimizer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("momentum", C.c_float),
                ("eps", C.c_float), ("beta1", C.c_double), ("beta2", C.c_double),
                ("step", C.c_int64)]


class ControllerConfig(C.Structure):
    _fields_ = [("gains", Gains), ("drop_tolerance", C.c_double),
                ("min_observations", C.c_int32), ("adaptive_b_max", C.c_int32)]


class WorkerResources(C.Structure):
    _fields_ = [("cpu_cores", C.c_int32), ("half_precision_flops", C.c_double)]


_lib = None


def load():
    """Loads libdynb.so (built by paper_2305_12213_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime; it must be in the process before libdynb.so so that
    # both resolve to one runtime instance (same soname) and can share device pointers.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError("libdynb.so is not built: run `python -m paper_2305_12213_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_double
    pi32, pf64 = C.POINTER(C.c_int32), C.POINTER(C.c_double)
    sig = {
        "dynb_last_error": (C.c_char_p, []),
        "dynb_model_create": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(vp)]),
        "dynb_model_destroy": (None, [vp]),
        "dynb_model_num_params": (i64, [vp]),
        "dynb_model_padded_params": (i64, [vp]),
        "dynb_model_workspace_bytes": (C.c_size_t, [vp, i32, i32]),
        "dynb_model_bind": (C.c_int, [vp, vp, vp, C.c_size_t, i32, i32, vp]),
        "dynb_model_sync_weights": (C.c_int, [vp, vp]),
        "dynb_model_worker_loss": (vp, [vp]),
        "dynb_model_read_worker_loss": (C.c_int, [vp, C.POINTER(C.c_float), i32, vp]),
        "dynb_forward_backward": (C.c_int, [vp, vp, vp, pi32, i32, vp, vp]),
        "dynb_forward_backward_aggregate": (C.c_int, [vp, vp, vp, pi32, i32, vp, vp, vp]),
        "dynb_weighted_aggregate": (C.c_int, [vp, pi32, i32, i64, vp, vp]),
        "dynb_sgd_update": (C.c_int, [vp, vp, i64, f32, vp]),
        "dynb_sgd_momentum_update": (C.c_int, [vp, vp, vp, i64, f32, f32, vp]),
        "dynb_model_sgd_update": (C.c_int, [vp, vp, f32, f32, vp, vp]),
        "dynb_controller_step": (C.c_int, [pf64, pi32, i32, i32, C.POINTER(Gains), pi32]),
        "dynb_ewma_update": (C.c_int, [pf64, pf64, i32, f64, i32]),
        "dynb_static_allocate": (C.c_int, [pf64, i32, i32, pi32]),
        "dynb_adam_update": (C.c_int, [vp, vp, vp, vp, i64, f32, f64, f64, f32, i64, vp]),
        "dynb_model_update": (C.c_int, [vp, vp, C.POINTER(Optimizer), vp, vp, vp]),
        "dynb_model_aggregate_update": (C.c_int, [vp, vp, pi32, i32, C.POINTER(Optimizer), vp, vp,
                                                  vp]),
        "dynb_lr_schedule": (C.c_int, [i64, C.POINTER(i64), pf64, i32, pf64]),
        "dynb_controller_create": (C.c_int, [C.POINTER(ControllerConfig), pi32, i32, i32,
                                             C.POINTER(vp)]),
        "dynb_controller_destroy": (None, [vp]),
        "dynb_controller_observe": (C.c_int, [vp, pf64, pi32, pi32]),
        "dynb_controller_read": (C.c_int, [vp, pi32, pf64, pi32, pi32, pi32]),
        "dynb_profile_enable": (C.c_int, [i32]),
        "dynb_profile_reset": (C.c_int, []),
        "dynb_profile_collect": (C.c_int, []),
        "dynb_profile_num_classes": (i32, []),
        "dynb_profile_name": (C.c_char_p, [i32]),
        "dynb_profile_get": (C.c_int, [i32, pf64, C.POINTER(i64), pf64, pf64]),
        "dynb_estimate_throughput": (C.c_int, [C.POINTER(WorkerResources), i32, pf64]),
        "dynb_static_scratch_bytes": (C.c_size_t, []),
        "dynb_forward_backward_static": (C.c_int, [vp, vp, vp, vp, pi32, i32, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise DynbError(rc, load().dynb_last_error().decode())


def _ptr(t):
    if t is None:
        return None
    return t.data_ptr() if hasattr(t, "data_ptr") else int(t)


def _stream(stream):
    if stream is not None:
        return stream
    try:
        import torch
        if torch.cuda.is_available():
            return torch.cuda.current_stream().cuda_stream
    except ImportError:
        pass
    return None


def _i32(values):
    return (C.c_int32 * len(values))(*[int(v) for v in values])


def _f64(values):
    return (C.c_double * len(values))(*[float(v) for v in values])


def model_desc_from_spec(spec):
    """Marshals a workload description (paper_2305_12213_amd.synth) into a ModelDesc."""
    layers = (LayerDesc * len(spec["layers"]))()
    for i, L in enumerate(spec["layers"]):
        if L["kind"] == "dense":
            layers[i] = LayerDesc(LAYER_DENSE, L["in"], L["out"], 1, int(L["relu"]))
        elif L["kind"] == "conv3x3":
            layers[i] = LayerDesc(LAYER_CONV3X3, L["cin"], L["cout"], L["stride"], int(L["relu"]))
        elif L["kind"] == "gap":
            layers[i] = LayerDesc(LAYER_GAP, 0, 0, 1, 0)
        elif L["kind"] == "bn":
            layers[i] = LayerDesc(LAYER_BN, L["channels"], L["channels"], 1, int(L["relu"]), -1,
                                  L["eps"])
        elif L["kind"] == "add":
            layers[i] = LayerDesc(LAYER_ADD, 0, 0, 1, int(L["relu"]), L["skip_from"], 0.0)
        else:
            raise ValueError(L["kind"])
    inp = tuple(spec["input"])
    h, w, c = inp if len(inp) == 3 else (1, 1, inp[0])
    d = ModelDesc(BF16 if spec["dtype"] == "bf16" else F32, h, w, c, spec["classes"],
                  len(spec["layers"]), layers)
    d._keep = layers
    return d


class Model:
    """Owner of a dynb_model handle."""

    def __init__(self, spec_or_desc):
        lib = load()
        desc = spec_or_desc if isinstance(spec_or_desc, ModelDesc) else \
            model_desc_from_spec(spec_or_desc)
        h = C.c_void_p()
        _check(lib.dynb_model_create(C.byref(desc), C.byref(h)))
        self._h = h
        self._keep = []

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.dynb_model_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        return self._h

    def num_params(self):
        return int(load().dynb_model_num_params(self._h))

    def padded_params(self):
        return int(load().dynb_model_padded_params(self._h))

    def workspace_bytes(self, max_global_batch, max_workers):
        return int(load().dynb_model_workspace_bytes(self._h, max_global_batch, max_workers))

    def bind(self, params, workspace, workspace_bytes, max_global_batch, max_workers, stream=None):
        self._keep = [params, workspace]
        _check(load().dynb_model_bind(self._h, _ptr(params), _ptr(workspace), workspace_bytes,
                                      max_global_batch, max_workers, _stream(stream)))

    def sync_weights(self, stream=None):
        _check(load().dynb_model_sync_weights(self._h, _stream(stream)))

    def worker_loss_ptr(self):
        return load().dynb_model_worker_loss(self._h)


def read_worker_loss(model, K, stream=None):
    """The K per-worker mean losses of the last forward_backward, as host floats (blocks)."""
    buf = (C.c_float * K)()
    _check(load().dynb_model_read_worker_loss(model.handle, buf, K, _stream(stream)))
    return [float(v) for v in buf]


def forward_backward(model, x, y, b, grads, stream=None):
    _check(load().dynb_forward_backward(model.handle, _ptr(x), _ptr(y), _i32(b), len(b),
                                        _ptr(grads), _stream(stream)))


def static_scratch_bytes():
    return int(load().dynb_static_scratch_bytes())


def forward_backward_static(model, params, x, y, b, grads, stream=None):
    _check(load().dynb_forward_backward_static(model.handle, _ptr(params), _ptr(x), _ptr(y),
                                               _i32(b), len(b), _ptr(grads), _stream(stream)))


def forward_backward_aggregate(model, x, y, b, grads, out, stream=None):
    _check(load().dynb_forward_backward_aggregate(model.handle, _ptr(x), _ptr(y), _i32(b), len(b),
                                                  _ptr(grads), _ptr(out), _stream(stream)))


def weighted_aggregate(grads, b, n, out, stream=None):
    _check(load().dynb_weighted_aggregate(_ptr(grads), _i32(b), len(b), n, _ptr(out),
                                          _stream(stream)))


def sgd_update(params, g, n, lr, stream=None):
    _check(load().dynb_sgd_update(_ptr(params), _ptr(g), n, lr, _stream(stream)))


def sgd_momentum_update(params, velocity, g, n, lr, mu, stream=None):
    _check(load().dynb_sgd_momentum_update(_ptr(params), _ptr(velocity), _ptr(g), n, lr, mu,
                                           _stream(stream)))


def model_sgd_update(model, g, lr, mu=0.0, velocity=None, stream=None):
    _check(load().dynb_model_sgd_update(model.handle, _ptr(g), lr, mu, _ptr(velocity),
                                        _stream(stream)))


def make_optimizer(kind="sgd", lr=0.0, momentum=0.0, beta1=0.9, beta2=0.999, eps=1e-8, step=1):
    kinds = {"sgd": OPT_SGD, "momentum": OPT_MOMENTUM, "adam": OPT_ADAM}
    return Optimizer(kinds[kind] if isinstance(kind, str) else int(kind), float(lr),
                     float(momentum), float(eps), float(beta1), float(beta2), int(step))


def adam_update(params, m, v, g, n, lr, beta1=0.9, beta2=0.999, eps=1e-8, step=1, stream=None):
    _check(load().dynb_adam_update(_ptr(params), _ptr(m), _ptr(v), _ptr(g), n, lr, beta1, beta2,
                                   eps, int(step), _stream(stream)))


def model_update(model, g, opt, state1=None, state2=None, stream=None):
    _check(load().dynb_model_update(model.handle, _ptr(g), C.byref(opt), _ptr(state1),
                                    _ptr(state2), _stream(stream)))


def model_aggregate_update(model, grads, b, opt, state1=None, state2=None, stream=None):
    _check(load().dynb_model_aggregate_update(model.handle, _ptr(grads), _i32(b), len(b),
                                              C.byref(opt), _ptr(state1), _ptr(state2),
                                              _stream(stream)))


def lr_schedule(step, boundaries, values):
    n = len(values)
    bd = (C.c_int64 * max(1, n - 1))(*[int(v) for v in boundaries]) if n > 1 else None
    out = C.c_double()
    _check(load().dynb_lr_schedule(int(step), bd, _f64(values), n, C.byref(out)))
    return out.value


def make_gains(kp=1.0, deadband=0.05, ewma_alpha=1.0, b_min=1, b_max=1 << 30, **_ignored):
    return Gains(float(kp), float(deadband), float(ewma_alpha), int(b_min), int(b_max))


def controller_step(iter_times, b, global_batch, gains):
    K = len(b)
    out = (C.c_int32 * K)()
    g = gains if isinstance(gains, Gains) else make_gains(**gains)
    _check(load().dynb_controller_step(_f64(iter_times), _i32(b), K, int(global_batch),
                                       C.byref(g), out))
    return [int(v) for v in out]


def ewma_update(mu, t, alpha, reset):
    K = len(t)
    m = _f64(mu if mu is not None else [0.0] * K)
    _check(load().dynb_ewma_update(m, _f64(t), K, float(alpha), int(bool(reset))))
    return [float(v) for v in m]


def static_allocate(X, b0):
    K = len(X)
    out = (C.c_int32 * K)()
    _check(load().dynb_static_allocate(_f64(X), K, int(b0), out))
    return [int(v) for v in out]


def estimate_throughput(cpu_cores, half_precision_flops):
    K = len(cpu_cores)
    r = (WorkerResources * K)(*[WorkerResources(int(c), float(f))
                                for c, f in zip(cpu_cores, half_precision_flops)])
    out = (C.c_double * K)()
    _check(load().dynb_estimate_throughput(r, K, out))
    return [float(v) for v in out]


class Controller:
    """Handle of the stateful controller (dynb_controller_*)."""

    def __init__(self, b0, global_batch, gains, drop_tolerance=0.0, min_observations=1,
                 adaptive_b_max=True):
        g = gains if isinstance(gains, Gains) else make_gains(**gains)
        cfg = ControllerConfig(g, float(drop_tolerance), int(min_observations),
                               int(bool(adaptive_b_max)))
        self.K = len(b0)
        self.handle = C.c_void_p()
        _check(load().dynb_controller_create(C.byref(cfg), _i32(b0), self.K, int(global_batch),
                                             C.byref(self.handle)))

    def observe(self, iter_times):
        if len(iter_times) != self.K:
            raise ValueError("one iteration time per worker")
        out = (C.c_int32 * self.K)()
        resized = C.c_int32()
        _check(load().dynb_controller_observe(self.handle, _f64(iter_times), out,
                                              C.byref(resized)))
        return [int(v) for v in out], bool(resized.value)

    def read(self):
        b = (C.c_int32 * self.K)(); mu = (C.c_double * self.K)(); hi = (C.c_int32 * self.K)()
        obs = C.c_int32(); adj = C.c_int32()
        _check(load().dynb_controller_read(self.handle, b, mu, hi, C.byref(obs), C.byref(adj)))
        return {"b": [int(v) for v in b], "mu": [float(v) for v in mu],
                "b_hi": [int(v) for v in hi], "observations": obs.value,
                "readjustments": adj.value}

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.dynb_controller_destroy(self.handle)
            self.handle = None


def profile_enable(on):
    _check(load().dynb_profile_enable(int(bool(on))))


def profile_reset():
    _check(load().dynb_profile_reset())


def profile_read():
    """{class name: dict(ms, launches, flops, bytes)} after folding pending events."""
    lib = load()
    _check(lib.dynb_profile_collect())
    out = {}
    for c in range(lib.dynb_profile_num_classes()):
        ms, fl, by = C.c_double(), C.c_double(), C.c_double()
        n = C.c_int64()
        _check(lib.dynb_profile_get(c, C.byref(ms), C.byref(n), C.byref(fl), C.byref(by)))
        out[lib.dynb_profile_name(c).decode()] = dict(ms=ms.value, launches=n.value,
                                                      flops=fl.value, bytes=by.value)
    return out
