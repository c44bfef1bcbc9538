"""CPU oracle of the pipelined online learner (test infrastructure only).

Thin ctypes wrapper around ``partime_oracle.c`` (plain C, fp64 arithmetic).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the HIP library never does.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "partime_oracle.c")
_LIB = os.path.join(_HERE, "libpartime_oracle.so")
_lock = threading.Lock()
_lib = None

DENSE, CONV3X3, GAP_DENSE = 0, 1, 2
ACT_ID, ACT_RELU, ACT_GELU = 0, 1, 2
LOSS_NONE, LOSS_MSE, LOSS_CE = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp); returns the library path."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + f".tmp{os.getpid()}"
            subprocess.check_call(
                ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=gnu99", "-fno-fast-math",
                 "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, ip, fp, dp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)
        lib.oracle_create.restype = vp
        lib.oracle_create.argtypes = [ctypes.c_int, ip, ctypes.c_int, ip, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_float, ctypes.c_int]
        lib.oracle_destroy.argtypes = [vp]
        lib.oracle_set_weights.argtypes = [vp, ctypes.c_int, fp, fp]
        lib.oracle_get_weights.argtypes = [vp, ctypes.c_int, fp, fp]
        lib.oracle_get_grads.argtypes = [vp, ctypes.c_int, dp, dp]
        lib.oracle_get_buffer.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp]
        lib.oracle_set_buffer.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp]
        lib.oracle_lane.restype = ctypes.c_int
        lib.oracle_lane.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, fp, ctypes.c_int]
        lib.oracle_get_history.argtypes = [vp, vp]
        lib.oracle_set_history.argtypes = [vp, vp]
        lib.oracle_get_tick.restype = ctypes.c_long
        lib.oracle_get_tick.argtypes = [vp]
        lib.oracle_set_tick.argtypes = [vp, ctypes.c_long]
        lib.oracle_set_lr.argtypes = [vp, ctypes.c_float]
        lib.oracle_reset.argtypes = [vp]
        lib.oracle_set_operand_rounding.argtypes = [vp, ctypes.c_int]
        lib.oracle_set_adam.argtypes = [vp, ctypes.c_double, ctypes.c_double, ctypes.c_double]
        lib.oracle_get_moments.argtypes = [vp, ctypes.c_int, fp, fp, fp, fp]
        lib.oracle_set_moments.argtypes = [vp, ctypes.c_int, fp, fp, fp, fp]
        lib.oracle_clone.restype = vp
        lib.oracle_clone.argtypes = [vp]
        lib.oracle_set_kink_band.argtypes = [vp, ctypes.c_double, ctypes.c_int, ctypes.c_long]
        lib.oracle_take_kink_events.restype = ctypes.c_long
        lib.oracle_take_kink_events.argtypes = [vp, ctypes.POINTER(ctypes.c_long)]
        lib.oracle_take_kink_margin.restype = ctypes.c_double
        lib.oracle_take_kink_margin.argtypes = [vp]
        lib.oracle_step.argtypes = [vp, fp, vp, ctypes.c_int, fp, fp, ip]
        lib.oracle_infer.argtypes = [vp, fp, ctypes.c_int, fp]
        lib.oracle_round_bf16.restype = ctypes.c_float
        lib.oracle_round_bf16.argtypes = [ctypes.c_float]
        _lib = lib
    return _lib


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def round_bf16(v: float) -> float:
    return float(_load().oracle_round_bf16(ctypes.c_float(v)))


class Layer:
    """Shape record of one layer (kind, activation, sizes)."""

    def __init__(self, kind=DENSE, act=ACT_ID, in_dim=0, out_dim=0, c_in=0, c_out=0, h=0, w=0, skip_from=-1):
        self.kind, self.act, self.in_dim, self.out_dim = kind, act, in_dim, out_dim
        self.c_in, self.c_out, self.h, self.w = c_in, c_out, h, w
        self.skip_from = skip_from   # index of the layer whose output is added to this layer's output (-1: none)

    def desc(self):
        return [self.kind, self.act, self.in_dim, self.out_dim, self.c_in, self.c_out, self.h, self.w, self.skip_from]

    @property
    def w_shape(self):
        if self.kind == DENSE:
            return (self.out_dim, self.in_dim)
        if self.kind == CONV3X3:
            return (self.c_out, self.c_in, 3, 3)
        return (self.out_dim, self.c_in)

    @property
    def b_shape(self):
        return (self.c_out,) if self.kind == CONV3X3 else (self.out_dim,)

    @property
    def in_size(self):
        return self.in_dim if self.kind == DENSE else self.c_in * self.h * self.w

    @property
    def out_size(self):
        return self.c_out * self.h * self.w if self.kind == CONV3X3 else self.out_dim


class Oracle:
    """Pipelined online learner, one tick at a time, on the CPU in fp64."""

    def __init__(self, layers, weights, biases, *, balance=None, n_streams=1, w_bf16=False,
                 loss=LOSS_MSE, lr=0.0, target_delay=0, operands_bf16=False, adam=None):
        self.lib = _load()
        self.layers = [Layer(l.kind, l.act, l.in_dim, l.out_dim, l.c_in, l.c_out, l.h, l.w, getattr(l, "skip_from", -1))
                       for l in layers]
        for j, l in enumerate(self.layers):
            s = l.skip_from
            assert s < j and (s < 0 or self.layers[s].out_size == l.out_size), "a skip adds an earlier output of equal size"
            assert s < 0 or sum(1 for q in self.layers if q.skip_from == s) == 1, "one skip per source layer"
        L = len(self.layers)
        self.balance = list(balance) if balance is not None else [1] * L
        assert sum(self.balance) == L
        self.depth = len(self.balance)
        self.S, self.loss, self.k = n_streams, loss, target_delay
        desc = np.asarray([d for l in self.layers for d in l.desc()], dtype=np.int32)
        bal = np.asarray(self.balance, dtype=np.int32)
        ip = ctypes.POINTER(ctypes.c_int)
        self.h = self.lib.oracle_create(L, desc.ctypes.data_as(ip), self.depth, bal.ctypes.data_as(ip),
                                        n_streams, int(w_bf16), loss, float(lr), target_delay)
        if operands_bf16:
            self.lib.oracle_set_operand_rounding(self.h, 1)
        if adam is not None:   # (beta1, beta2, eps): fp32 values, like the learning rate (the arithmetic is fp64)
            self.lib.oracle_set_adam(self.h, *[float(np.float32(v)) for v in adam[:3]])
        for i, (W, b) in enumerate(zip(weights, biases)):
            self.set_weights(i, W, b)
        first = np.concatenate([[0], np.cumsum(self.balance)])
        self.stage_in = [self.layers[first[h]].in_size for h in range(self.depth)]
        self.stage_out = [self.layers[first[h + 1] - 1].out_size for h in range(self.depth)]

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.oracle_destroy(self.h)
            self.h = None

    def set_weights(self, i, W, b):
        W = np.ascontiguousarray(W, dtype=np.float32).reshape(self.layers[i].w_shape)
        b = np.ascontiguousarray(b, dtype=np.float32).reshape(self.layers[i].b_shape)
        self.lib.oracle_set_weights(self.h, i, _fp(W), _fp(b))

    def get_weights(self, i):
        W = np.empty(self.layers[i].w_shape, dtype=np.float32)
        b = np.empty(self.layers[i].b_shape, dtype=np.float32)
        self.lib.oracle_get_weights(self.h, i, _fp(W), _fp(b))
        return W, b

    def get_moments(self, i):
        l = self.layers[i]
        mW, vW = np.empty(l.w_shape, dtype=np.float32), np.empty(l.w_shape, dtype=np.float32)
        mb, vb = np.empty(l.b_shape, dtype=np.float32), np.empty(l.b_shape, dtype=np.float32)
        self.lib.oracle_get_moments(self.h, i, _fp(mW), _fp(vW), _fp(mb), _fp(vb))
        return mW, vW, mb, vb

    def set_moments(self, i, mW, vW, mb, vb):
        a = [np.ascontiguousarray(t, dtype=np.float32) for t in (mW, vW, mb, vb)]
        self.lib.oracle_set_moments(self.h, i, *[_fp(t) for t in a])

    def get_grads(self, i):
        dW = np.empty(self.layers[i].w_shape, dtype=np.float64)
        db = np.empty(self.layers[i].b_shape, dtype=np.float64)
        dp = ctypes.POINTER(ctypes.c_double)
        self.lib.oracle_get_grads(self.h, i, dW.ctypes.data_as(dp), db.ctypes.data_as(dp))
        return dW, db

    def get_buffer(self, which, stage, half):
        n = self.stage_out[stage] if which == "act" else self.stage_in[stage]
        a = np.empty((self.S, n), dtype=np.float32)
        self.lib.oracle_get_buffer(self.h, 0 if which == "act" else 1, stage, half, _fp(a))
        return a

    def set_buffer(self, which, stage, half, a):
        n = self.stage_out[stage] if which == "act" else self.stage_in[stage]
        a = np.ascontiguousarray(a, dtype=np.float32).reshape(self.S, n)
        self.lib.oracle_set_buffer(self.h, 0 if which == "act" else 1, stage, half, _fp(a))

    def skip_delay(self, layer):
        """Stage boundaries the skip into `layer` crosses (0: none, or no skip)."""
        src = self.layers[layer].skip_from
        if src < 0:
            return 0
        stage_of = [h for h, c in enumerate(self.balance) for _ in range(c)]
        return stage_of[layer] - stage_of[src]

    def get_lane(self, kind, layer, age):
        """Delay line of the skip into `layer`: kind 0 the skipped tensor, 1 its gradient; age 0 = written in the last tick."""
        a = np.empty((self.S, self.layers[layer].out_size), dtype=np.float32)
        assert self.lib.oracle_lane(self.h, layer, kind, age, _fp(a), 0) == 0
        return a

    def set_lane(self, kind, layer, age, a):
        a = np.ascontiguousarray(a, dtype=np.float32).reshape(self.S, self.layers[layer].out_size)
        assert self.lib.oracle_lane(self.h, layer, kind, age, _fp(a), 1) == 0

    def get_history(self):
        """The targets of the last target_delay ticks, oldest first, as raw 4-byte elements (float32 view)."""
        per = self.S * (self.stage_out[-1] if self.loss == LOSS_MSE else 1)
        a = np.zeros((max(self.k, 0) * per,), dtype=np.float32)
        if a.size:
            self.lib.oracle_get_history(self.h, a.ctypes.data_as(ctypes.c_void_p))
        return a

    def set_history(self, a):
        a = np.ascontiguousarray(a)
        assert a.dtype.itemsize == 4
        if a.size:
            self.lib.oracle_set_history(self.h, a.ctypes.data_as(ctypes.c_void_p))

    @property
    def tick(self):
        return int(self.lib.oracle_get_tick(self.h))

    @tick.setter
    def tick(self, t):
        self.lib.oracle_set_tick(self.h, int(t))

    def set_lr(self, lr):
        self.lib.oracle_set_lr(self.h, float(lr))

    def take_kink_margin(self) -> float:
        """Smallest |z| at which a ReLU derivative entered a non-zero delta since the last call (diagnostic)."""
        return float(self.lib.oracle_take_kink_margin(self.h))

    def set_kink_band(self, eps: float, side: int = 0, cap: int = 4096):
        """Test diagnostic: record ReLU units with |z| < eps and a non-zero error signal; side +1 / -1 also takes
        1 / 0 as their derivative (side 0 leaves the arithmetic alone)."""
        self._band_cap = cap
        self.lib.oracle_set_kink_band(self.h, float(eps), int(side), cap)

    def take_kink_events(self):
        """(count, int64 array [min(count, cap)][3] of (tick, layer, stream * out_size + unit)) since the last call."""
        cap = getattr(self, "_band_cap", 0)
        buf = np.zeros((max(cap, 1), 3), dtype=np.int64)
        cnt = int(self.lib.oracle_take_kink_events(self.h, buf.ctypes.data_as(ctypes.POINTER(ctypes.c_long))))
        return cnt, buf[:min(cnt, cap)]

    def clone(self):
        """Deep copy: weights, moments, buffers, lanes, target history, tick and switches."""
        import copy
        c = copy.copy(self)
        c.h = self.lib.oracle_clone(self.h)
        return c

    def reset(self):
        self.lib.oracle_reset(self.h)

    def _x(self, x):
        x = np.ascontiguousarray(x, dtype=np.float32)
        n = x.size // (self.S * self.stage_in[0])
        assert n * self.S * self.stage_in[0] == x.size
        return x, n

    def step(self, x, target, order=None):
        """Run len(x) learning ticks; returns (out [n,S,out], loss [n])."""
        x, n = self._x(x)
        if self.loss == LOSS_CE:
            tg = np.ascontiguousarray(target, dtype=np.int32)
            assert tg.size == n * self.S
        else:
            tg = np.ascontiguousarray(target, dtype=np.float32)
            assert tg.size == n * self.S * self.stage_out[-1]
        out = np.zeros((n, self.S, self.stage_out[-1]), dtype=np.float32)
        loss = np.zeros((n,), dtype=np.float32)
        op = None
        if order is not None:
            order = np.ascontiguousarray(order, dtype=np.int32)
            assert sorted(order.tolist()) == list(range(self.depth))
            op = order.ctypes.data_as(ctypes.POINTER(ctypes.c_int))
        self.lib.oracle_step(self.h, _fp(x), tg.ctypes.data_as(ctypes.c_void_p), n, _fp(out), _fp(loss), op)
        return out, loss

    def infer(self, x):
        x, n = self._x(x)
        out = np.zeros((n, self.S, self.stage_out[-1]), dtype=np.float32)
        self.lib.oracle_infer(self.h, _fp(x), n, _fp(out))
        return out
