"""ctypes loader for the C part of the oracle (fixed_order_f32.c).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fixed_order_f32.c")
_LIB = os.path.join(_HERE, "libslora_oracle_c.so")


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared",
                               _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_fedavg_weights_f32.restype = ctypes.c_int
    return _lib


def fedavg_weights_f32(counts):
    counts = np.ascontiguousarray(counts, dtype=np.int64)
    w = np.empty(len(counts), dtype=np.float32)
    rc = _load().oracle_fedavg_weights_f32(len(counts), counts.ctypes.data_as(ctypes.c_void_p),
                                           w.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("sample counts must be non-negative with a positive sum")
    return w


def fedavg_f32(client_params, counts):
    """Fixed-order fp32 FedAvg (Eq. 8-9) of K flat float32 vectors."""
    xs = [np.ascontiguousarray(x, dtype=np.float32).ravel() for x in client_params]
    n = xs[0].size
    assert all(x.size == n for x in xs)
    w = fedavg_weights_f32(counts)
    ptrs = (ctypes.c_void_p * len(xs))(*[x.ctypes.data for x in xs])
    out = np.empty(n, dtype=np.float32)
    _load().oracle_fedavg_f32(len(xs), ptrs, w.ctypes.data_as(ctypes.c_void_p),
                              ctypes.c_size_t(n), out.ctypes.data_as(ctypes.c_void_p))
    return out


def sgd_f32(p, g, lr):
    """Eq. (4)-(5) in fp32: returns p - lr*g evaluated as fmaf(-lr, g, p)."""
    out = np.ascontiguousarray(p, dtype=np.float32).copy().ravel()
    g = np.ascontiguousarray(g, dtype=np.float32).ravel()
    _load().oracle_sgd_f32(out.ctypes.data_as(ctypes.c_void_p), g.ctypes.data_as(ctypes.c_void_p),
                           ctypes.c_float(lr), ctypes.c_size_t(out.size))
    return out.reshape(np.shape(p))


def adamw_f32(p, g, m, v, lr, beta1, beta2, eps, weight_decay, step):
    """Fixed-order fp32 AdamW step on flat vectors; returns new (p, m, v)."""
    p = np.ascontiguousarray(p, dtype=np.float32).copy().ravel()
    m = np.ascontiguousarray(m, dtype=np.float32).copy().ravel()
    v = np.ascontiguousarray(v, dtype=np.float32).copy().ravel()
    g = np.ascontiguousarray(g, dtype=np.float32).ravel()
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    _load().oracle_adamw_f32(vp(p), vp(g), vp(m), vp(v), ctypes.c_size_t(p.size), ctypes.c_float(lr),
                             ctypes.c_float(beta1), ctypes.c_float(beta2), ctypes.c_float(eps),
                             ctypes.c_float(weight_decay), ctypes.c_int(step))
    return p, m, v
