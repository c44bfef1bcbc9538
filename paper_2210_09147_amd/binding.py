"""ctypes binding of libpartime.so: argument marshalling only.

Every function has the name and the arguments of its C counterpart in
``include/partime.h``; device buffers are passed as integer addresses
(``tensor.data_ptr()``).  There is no CPU fallback: if the HIP library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PARTIME_LIB") or os.path.join(_HERE, "libpartime.so")

PT_DENSE, PT_CONV3X3, PT_GAP_DENSE = 0, 1, 2
PT_ID, PT_RELU, PT_GELU = 0, 1, 2
PT_LOSS_NONE, PT_LOSS_MSE, PT_LOSS_CE = 0, 1, 2
PT_F32, PT_BF16 = 0, 1
PT_EXEC_AUTO, PT_EXEC_LAUNCH_PER_TICK, PT_EXEC_PERSISTENT = 0, 1, 2
PT_OPT_SGD, PT_OPT_ADAM = 0, 1
PT_OK, PT_EINVAL, PT_ESHAPE, PT_ENOMEM, PT_EHIP, PT_EUNSUPPORTED = 0, -1, -2, -3, -4, -5

EXPORTS = [
    "partime_init", "partime_step", "partime_infer", "partime_get_state", "partime_set_state",
    "partime_get_buffer", "partime_set_buffer", "partime_get_tick", "partime_set_tick", "partime_set_lr",
    "partime_reset", "partime_sync", "partime_destroy", "partime_last_error", "partime_last_launch_count",
    "partime_bandwidth_probe", "partime_get_opt_state", "partime_set_opt_state", "partime_step_noalloc",
]


class pt_layer(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("kind", "act", "in_dim", "out_dim", "c_in", "c_out", "h", "w", "skip_from")]


class partime_config(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int), ("layers", ctypes.POINTER(pt_layer)),
        ("depth", ctypes.c_int), ("balance", ctypes.POINTER(ctypes.c_int)),
        ("n_streams", ctypes.c_int), ("w_dtype", ctypes.c_int), ("loss", ctypes.c_int),
        ("lr", ctypes.c_float), ("target_delay", ctypes.c_int), ("exec_mode", ctypes.c_int),
        ("hip_stream", ctypes.c_void_p),
        ("optimizer", ctypes.c_int), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
    ]


class PartimeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"partime error {code}: {msg}")
        self.code = code


_lib = None


def load():
    """Load libpartime.so (built in-tree by ``build.build_library``); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, fpp = ctypes.c_void_p, ctypes.POINTER(ctypes.POINTER(ctypes.c_float))
    fp = ctypes.POINTER(ctypes.c_float)
    lib.partime_init.argtypes = [ctypes.POINTER(partime_config), fpp, fpp, ctypes.POINTER(vp)]
    lib.partime_step.argtypes = [vp, vp, vp, ctypes.c_int, vp, vp]
    lib.partime_step_noalloc.argtypes = [vp, vp, vp, ctypes.c_int, vp, vp]
    lib.partime_infer.argtypes = [vp, vp, ctypes.c_int, vp]
    lib.partime_get_state.argtypes = [vp, ctypes.c_int, fp, fp]
    lib.partime_set_state.argtypes = [vp, ctypes.c_int, fp, fp]
    lib.partime_get_buffer.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp]
    lib.partime_set_buffer.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp]
    lib.partime_get_tick.argtypes = [vp, ctypes.POINTER(ctypes.c_int64)]
    lib.partime_set_tick.argtypes = [vp, ctypes.c_int64]
    lib.partime_set_lr.argtypes = [vp, ctypes.c_float]
    lib.partime_reset.argtypes = [vp]
    lib.partime_sync.argtypes = [vp]
    lib.partime_destroy.argtypes = [vp]
    lib.partime_destroy.restype = None
    lib.partime_last_error.restype = ctypes.c_char_p
    lib.partime_last_launch_count.argtypes = [vp]
    lib.partime_get_opt_state.argtypes = [vp, ctypes.c_int, fp, fp, fp, fp]
    lib.partime_set_opt_state.argtypes = [vp, ctypes.c_int, fp, fp, fp, fp]
    lib.partime_bandwidth_probe.argtypes = [ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    _lib = lib
    return lib


def _check(rc):
    if rc != PT_OK:
        raise PartimeError(rc, load().partime_last_error().decode())


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def partime_last_error() -> str:
    return load().partime_last_error().decode()


def partime_init(layers, weights, biases, *, balance=None, n_streams=1, w_dtype=PT_F32, loss=PT_LOSS_MSE,
                 lr=0.0, target_delay=0, exec_mode=PT_EXEC_AUTO, hip_stream=0, adam=None):
    """layers: records with kind/act/in_dim/out_dim/c_in/c_out/h/w; weights/biases: fp32 numpy arrays;
    adam: None (plain SGD) or (beta1, beta2, eps)."""
    lib = load()
    L = len(layers)
    arr = (pt_layer * L)(*[pt_layer(l.kind, l.act, l.in_dim, l.out_dim, l.c_in, l.c_out, l.h, l.w, getattr(l, "skip_from", -1))
                           for l in layers])
    bal = None
    depth = L
    if balance is not None:
        depth = len(balance)
        bal = (ctypes.c_int * depth)(*balance)
    opt = (PT_OPT_SGD, 0.0, 0.0, 0.0) if adam is None else (PT_OPT_ADAM, float(adam[0]), float(adam[1]), float(adam[2]))
    cfg = partime_config(L, arr, depth, bal, n_streams, w_dtype, loss, lr, target_delay, exec_mode,
                         ctypes.c_void_p(hip_stream), *opt)
    ws = [np.ascontiguousarray(w, dtype=np.float32) for w in weights]
    bs = [np.ascontiguousarray(b, dtype=np.float32) for b in biases]
    fp = ctypes.POINTER(ctypes.c_float)
    wp = (fp * L)(*[_fptr(w) for w in ws])
    bp = (fp * L)(*[_fptr(b) for b in bs])
    ctx = ctypes.c_void_p()
    _check(lib.partime_init(ctypes.byref(cfg), wp, bp, ctypes.byref(ctx)))
    return ctx


def partime_step(ctx, x_dev: int, target_dev: int, n_ticks: int, out_dev: int, loss_dev: int):
    _check(load().partime_step(ctx, x_dev, target_dev, n_ticks, out_dev, loss_dev))


def partime_step_noalloc(ctx, x_dev: int, target_dev: int, n_ticks: int, out_dev: int, loss_dev: int):
    _check(load().partime_step_noalloc(ctx, x_dev, target_dev, n_ticks, out_dev, loss_dev))


def partime_infer(ctx, x_dev: int, n_ticks: int, out_dev: int):
    _check(load().partime_infer(ctx, x_dev, n_ticks, out_dev))


def partime_get_state(ctx, layer: int, w_shape, b_shape):
    W = np.empty(w_shape, dtype=np.float32)
    b = np.empty(b_shape, dtype=np.float32)
    _check(load().partime_get_state(ctx, layer, _fptr(W), _fptr(b)))
    return W, b


def partime_set_state(ctx, layer: int, W=None, b=None):
    W = None if W is None else np.ascontiguousarray(W, dtype=np.float32)
    b = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
    _check(load().partime_set_state(ctx, layer, None if W is None else _fptr(W), None if b is None else _fptr(b)))


def partime_get_buffer(ctx, which: int, stage: int, half: int, n: int):
    a = np.empty((n,), dtype=np.float32)
    _check(load().partime_get_buffer(ctx, which, stage, half, _fptr(a)))
    return a


def partime_set_buffer(ctx, which: int, stage: int, half: int, a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    _check(load().partime_set_buffer(ctx, which, stage, half, _fptr(a)))


def partime_get_tick(ctx) -> int:
    t = ctypes.c_int64()
    _check(load().partime_get_tick(ctx, ctypes.byref(t)))
    return t.value


def partime_set_tick(ctx, tick: int):
    _check(load().partime_set_tick(ctx, tick))


def partime_set_lr(ctx, lr: float):
    _check(load().partime_set_lr(ctx, lr))


def partime_reset(ctx):
    _check(load().partime_reset(ctx))


def partime_sync(ctx):
    _check(load().partime_sync(ctx))


def partime_destroy(ctx):
    load().partime_destroy(ctx)


def partime_last_launch_count(ctx) -> int:
    return load().partime_last_launch_count(ctx)


def partime_bandwidth_probe(n_bytes: int, mode: int, iters: int = 20) -> float:
    """GB/s of a plain streaming kernel (0 read, 1 write, 2 in-place read+write) over n_bytes on the current device."""
    g = ctypes.c_double()
    _check(load().partime_bandwidth_probe(n_bytes, mode, iters, ctypes.byref(g)))
    return g.value


def partime_get_opt_state(ctx, layer: int, w_shape, b_shape):
    a = [np.empty(w_shape, dtype=np.float32), np.empty(w_shape, dtype=np.float32),
         np.empty(b_shape, dtype=np.float32), np.empty(b_shape, dtype=np.float32)]
    _check(load().partime_get_opt_state(ctx, layer, *[_fptr(t) for t in a]))
    return tuple(a)


def partime_set_opt_state(ctx, layer: int, mW, vW, mb, vb):
    a = [np.ascontiguousarray(t, dtype=np.float32) for t in (mW, vW, mb, vb)]
    _check(load().partime_set_opt_state(ctx, layer, *[_fptr(t) for t in a]))
