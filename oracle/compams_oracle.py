"""ctypes front end of the CPU oracle (test infrastructure, not the product).

Thin marshalling over oracle/compams_oracle.cpp: numpy arrays in, numpy arrays
out.  None of the method's arithmetic lives here.
"""
import ctypes
import os

import numpy as np

from . import build_oracle

NONE, TOPK, BLOCKSIGN = 0, 1, 2
EPS_IN_SQRT, EPS_OUT_SQRT = 0, 1

_Q = {"theta": 0, "m": 1, "v": 2, "vhat": 3, "e": 4, "idx": 5, "val": 6, "bits": 7, "mu": 8,
      "gbar": 9, "ctil": 10}
_DT = {"idx": np.int32, "bits": np.uint32}

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.build()
        L = ctypes.CDLL(path)
        f32p = ctypes.POINTER(ctypes.c_float)
        i64p = ctypes.POINTER(ctypes.c_int64)
        i32p = ctypes.POINTER(ctypes.c_int32)
        L.oracle_compams_create.restype = ctypes.c_void_p
        L.oracle_compams_create.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int64,
                                            ctypes.c_int64, i64p, ctypes.c_float, ctypes.c_float,
                                            ctypes.c_float, ctypes.c_int, f32p]
        L.oracle_compams_destroy.argtypes = [ctypes.c_void_p]
        L.oracle_compams_step.argtypes = [ctypes.c_void_p, f32p, ctypes.c_float]
        L.oracle_compams_set_state.argtypes = [ctypes.c_void_p, f32p, f32p, f32p, f32p, f32p]
        L.oracle_compams_get.restype = ctypes.c_void_p
        L.oracle_compams_get.argtypes = [ctypes.c_void_p, ctypes.c_int, i64p]
        L.oracle_topk_select.argtypes = [f32p, ctypes.c_int64, ctypes.c_int64, i32p]
        L.oracle_topk_select_fullsort.argtypes = [f32p, ctypes.c_int64, ctypes.c_int64, i32p]
        L.oracle_block_l1_mean.restype = ctypes.c_float
        L.oracle_block_l1_mean.argtypes = [f32p, ctypes.c_int64]
        L.oracle_exact_abs_sum.restype = ctypes.c_double
        L.oracle_exact_abs_sum.argtypes = [f32p, ctypes.c_int64]
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def topk_select(x, k, fullsort=False):
    x, px = _f32(x)
    out = np.empty(k, dtype=np.int32)
    fn = lib().oracle_topk_select_fullsort if fullsort else lib().oracle_topk_select
    fn(px, x.size, k, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return out


def block_l1_mean(x):
    x, px = _f32(x)
    return np.float32(lib().oracle_block_l1_mean(px, x.size))


def exact_abs_sum(x):
    x, px = _f32(x)
    return float(lib().oracle_exact_abs_sum(px, x.size))


class Oracle:
    """One COMP-AMS optimizer: n workers, d coordinates, state on the host."""

    def __init__(self, n, d, theta0, compressor=TOPK, k=0, block_offsets=None,
                 beta1=0.9, beta2=0.999, eps=1e-8, eps_mode=EPS_IN_SQRT):
        self.n, self.d, self.k, self.compressor = int(n), int(d), int(k), compressor
        off = None
        M = 0
        if block_offsets is not None:
            off = np.ascontiguousarray(block_offsets, dtype=np.int64)
            M = off.size - 1
        self.M = M
        th, pth = _f32(theta0)
        assert th.size == d
        poff = off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)) if off is not None else None
        self._h = lib().oracle_compams_create(self.n, self.d, compressor, self.k, M, poff,
                                              beta1, beta2, eps, eps_mode, pth)
        if not self._h:
            raise ValueError("oracle_compams_create rejected the configuration")

    def step(self, g, lr):
        g, pg = _f32(g)
        assert g.size == self.n * self.d
        lib().oracle_compams_step(self._h, pg, lr)

    def set_state(self, theta=None, m=None, v=None, vhat=None, e=None):
        keep = []
        ptrs = []
        for a in (theta, m, v, vhat, e):
            if a is None:
                ptrs.append(None)
            else:
                arr, p = _f32(a)
                keep.append(arr)
                ptrs.append(p)
        lib().oracle_compams_set_state(self._h, *ptrs)

    def get(self, name):
        cnt = ctypes.c_int64(0)
        p = lib().oracle_compams_get(self._h, _Q[name], ctypes.byref(cnt))
        dt = _DT.get(name, np.float32)
        if cnt.value == 0:
            return np.empty(0, dtype=dt)
        buf = (ctypes.c_char * (cnt.value * np.dtype(dt).itemsize)).from_address(p)
        a = np.frombuffer(buf, dtype=dt).copy()
        if name in ("e", "ctil"):
            a = a.reshape(self.n, self.d)
        elif name in ("idx", "val"):
            a = a.reshape(self.n, self.k)
        elif name == "bits":
            a = a.reshape(self.n, -1)
        elif name == "mu":
            a = a.reshape(self.n, self.M)
        return a

    def close(self):
        if self._h:
            lib().oracle_compams_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
