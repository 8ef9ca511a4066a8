"""ctypes front end of the CPU oracle (test infrastructure, not the product).

Thin marshalling over oracle/compams_oracle.cpp: numpy arrays in, numpy arrays
out.  None of the method's arithmetic lives here.
"""
import ctypes
import os

import numpy as np

from . import build_oracle

NONE, TOPK, BLOCKSIGN, TOPK_BLOCKS = 0, 1, 2, 3
EPS_IN_SQRT, EPS_OUT_SQRT = 0, 1

_Q = {"theta": 0, "m": 1, "v": 2, "vhat": 3, "e": 4, "idx": 5, "val": 6, "bits": 7, "mu": 8,
      "gbar": 9, "ctil": 10}
_DT = {"idx": np.int32, "bits": np.uint32}

_lib = None


def lib():
    global _lib
    if _lib is None:
        # COMPAMS_ORACLE_SANITIZE=1: the AddressSanitizer / UBSan build of the same source (the process must have
        # been started with the sanitizer runtime preloaded)
        path = build_oracle.build(sanitize=os.environ.get("COMPAMS_ORACLE_SANITIZE") == "1")
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
        L.oracle_compams_create_topk_blocks.restype = ctypes.c_void_p
        L.oracle_compams_create_topk_blocks.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, i64p, i64p,
                                                        ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int,
                                                        f32p]
        u32p = ctypes.POINTER(ctypes.c_uint32)
        L.oracle_wire_encode_topk.restype = ctypes.c_int64
        L.oracle_wire_encode_topk.argtypes = [ctypes.c_int64, i32p, f32p, u32p]
        L.oracle_wire_decode_topk.restype = ctypes.c_int64
        L.oracle_wire_decode_topk.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, i32p, f32p]
        L.oracle_wire_encode_blocksign.restype = ctypes.c_int64
        L.oracle_wire_encode_blocksign.argtypes = [ctypes.c_int64, ctypes.c_int64, u32p, f32p, u32p]
        L.oracle_wire_decode_blocksign.restype = ctypes.c_int64
        L.oracle_wire_decode_blocksign.argtypes = [u32p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, u32p, f32p]
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


def _u32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))


def wire_encode_topk(idx, val):
    """One worker's top-k message as uint32 words."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val, pv = _f32(val)
    k = idx.size
    out = np.zeros(4 + (k + 1023) // 1024 + 2 * k, dtype=np.uint32)
    n = lib().oracle_wire_encode_topk(k, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), pv, _u32p(out))
    return out[:n].copy()


def wire_decode_topk(msg, k, d):
    """(idx, val) of a top-k message, or raises ValueError if the words are not one for (k, d)."""
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float32)
    rc = lib().oracle_wire_decode_topk(_u32p(msg), msg.size, k, d, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                       val.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError(f"not a top-k message (code {rc})")
    return idx, val


def wire_encode_blocksign(d, bits, mu):
    bits = np.ascontiguousarray(bits, dtype=np.uint32)
    mu, pm = _f32(mu)
    out = np.zeros(3 + bits.size + mu.size, dtype=np.uint32)
    n = lib().oracle_wire_encode_blocksign(d, mu.size, _u32p(bits), pm, _u32p(out))
    return out[:n].copy()


def wire_decode_blocksign(msg, d, M):
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    bits = np.empty((d + 31) // 32, dtype=np.uint32)
    mu = np.empty(M, dtype=np.float32)
    rc = lib().oracle_wire_decode_blocksign(_u32p(msg), msg.size, d, M, _u32p(bits),
                                            mu.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc != 0:
        raise ValueError(f"not a block-sign message (code {rc})")
    return bits, mu


class Oracle:
    """One COMP-AMS optimizer: n workers, d coordinates, state on the host."""

    def __init__(self, n, d, theta0, compressor=TOPK, k=0, block_offsets=None,
                 beta1=0.9, beta2=0.999, eps=1e-8, eps_mode=EPS_IN_SQRT, block_k=None):
        """compressor TOPK_BLOCKS: Definition 1 per block, block b keeping block_k[b] coordinates."""
        self.n, self.d, self.k, self.compressor = int(n), int(d), int(k), compressor
        if compressor == TOPK_BLOCKS:
            off = np.ascontiguousarray(block_offsets, dtype=np.int64)
            kb = np.ascontiguousarray(block_k, dtype=np.int64)
            assert kb.size == off.size - 1
            self.M, self.k = kb.size, int(kb.sum())
            th, pth = _f32(theta0)
            assert th.size == d
            i64 = ctypes.POINTER(ctypes.c_int64)
            self._h = lib().oracle_compams_create_topk_blocks(self.n, self.d, self.M, off.ctypes.data_as(i64),
                                                              kb.ctypes.data_as(i64), beta1, beta2, eps, eps_mode, pth)
            if not self._h:
                raise ValueError("oracle_compams_create_topk_blocks rejected the configuration")
            return
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
