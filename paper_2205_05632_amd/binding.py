"""Python binding of libcompams: argument marshalling only.

Same names as the C ABI (include/compams.h).  PyTorch provides device memory and the current
stream; every step of the optimizer runs in the library's HIP kernels.  There is no fallback: if
the shared library has not been built, importing the functions raises.
"""
import ctypes
import os
from typing import Dict, Optional

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcompams.so")

NONE, TOPK, BLOCKSIGN, TOPK_BLOCKS = 0, 1, 2, 3
EPS_IN_SQRT, EPS_OUT_SQRT = 0, 1
KEEP_STATE = 1
OPT_CANDIDATE_CAP, OPT_PREDICT, OPT_FORCE_DENSE, OPT_BAND, OPT_CACHED_ARRAYS = 0, 1, 2, 3, 4
COUNTERS_PER_ROW = 8

STATE = {"theta": 0, "m": 1, "v": 2, "vhat": 3, "e": 4, "last_idx": 5, "last_val": 6, "last_signbits": 7,
         "last_scales": 8, "last_threshold": 9, "counters": 10, "last_count_gt": 11, "pending": 12}
_STATE_DTYPE = {"last_idx": torch.int32, "last_signbits": torch.int32, "last_threshold": torch.int32,
                "counters": torch.int32, "last_count_gt": torch.int32}

EXPORTS = ["compams_workspace_size", "compams_init", "compams_step", "compams_state", "compams_set_option",
           "compams_profile_enable", "compams_profile_read", "compams_destroy", "compams_strerror", "compams_copy", "compams_inplace_probe", "compams_cached_state_arrays",
           "compams_wire_capacity", "compams_encode", "compams_decode", "compams_worker_step", "compams_server_step",
           "compams_step_static"]
STATIC_SCRATCH_BYTES = 32 << 20


class compams_config(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("d", ctypes.c_int64), ("ld", ctypes.c_int64),
                ("compressor", ctypes.c_int32), ("k", ctypes.c_int64), ("num_blocks", ctypes.c_int64),
                ("block_offsets", ctypes.POINTER(ctypes.c_int64)),
                ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("eps_mode", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("theta", ctypes.c_void_p), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("vhat", ctypes.c_void_p), ("e", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("block_k", ctypes.POINTER(ctypes.c_int64))]


class CompamsError(RuntimeError):
    pass


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise CompamsError(f"{LIB_PATH} is missing: build it with `python -m paper_2205_05632_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        cfgp = ctypes.POINTER(compams_config)
        L.compams_workspace_size.restype = ctypes.c_size_t
        L.compams_workspace_size.argtypes = [cfgp]
        L.compams_init.argtypes = [cfgp, ctypes.POINTER(ctypes.c_void_p)]
        L.compams_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p]
        L.compams_state.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p),
                                    ctypes.POINTER(ctypes.c_int64)]
        L.compams_set_option.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64]
        L.compams_profile_enable.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.compams_profile_read.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_char_p),
                                           ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64),
                                           ctypes.POINTER(ctypes.c_int)]
        L.compams_destroy.argtypes = [ctypes.c_void_p]
        L.compams_strerror.restype = ctypes.c_char_p
        L.compams_strerror.argtypes = [ctypes.c_int]
        L.compams_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.compams_cached_state_arrays.argtypes = [ctypes.c_int64]
        L.compams_inplace_probe.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_size_t,
                                            ctypes.c_int, ctypes.c_void_p]
        L.compams_wire_capacity.restype = ctypes.c_size_t
        L.compams_wire_capacity.argtypes = [cfgp]
        L.compams_encode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        L.compams_decode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.compams_worker_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.compams_server_step.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                          ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p]
        L.compams_step_static.argtypes = [cfgp, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p]
        _lib = L
    return _lib


def _check(status: int, what: str):
    if status != 0:
        raise CompamsError(f"{what}: {lib().compams_strerror(status).decode()} ({status})")


def compams_strerror(status: int) -> str:
    return lib().compams_strerror(status).decode()


def _current_stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


def padded_ld(d: int) -> int:
    """Row stride the binding picks by default.  Any multiple of 4 elements >= d is legal (16-byte aligned
    rows); rows that start on a 4 KiB boundary stream measurably faster (whole cache lines and DRAM bursts
    per wavefront access), so large rows are padded to a multiple of 1024 elements."""
    d = int(d)
    return (d + 1023) // 1024 * 1024 if d >= 4096 else (d + 3) // 4 * 4


class Compams:
    """One optimizer context: owns the torch tensors that the library borrows.

    compams_init / compams_step / compams_state map one-to-one onto the C entry points.
    """

    def __init__(self, n: int, d: int, theta0: torch.Tensor, compressor: int = TOPK, k: int = 0,
                 block_offsets=None, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                 eps_mode: int = EPS_IN_SQRT, ld: Optional[int] = None, device="cuda:0",
                 state: Optional[Dict[str, torch.Tensor]] = None,
                 views: Optional[Dict[str, torch.Tensor]] = None, block_k=None):
        """block_k (TOPK_BLOCKS): coordinates kept in every block; a worker's list then has sum(block_k) entries,
        block after block, and k is ignored.
        views: instead of allocating, borrow the caller's tensors (theta, m, v, vhat: d floats each; e: a view
        whose first element is row 0, column 0 of this context's residuals and whose row stride is ld) -- how a
        context is laid over a slice of larger buffers; theta0 is then ignored."""
        self.n, self.d, self.k, self.compressor = int(n), int(d), int(k), int(compressor)
        self._kb = None
        if block_k is not None:
            self._kb = np.ascontiguousarray(block_k, dtype=np.int64)
            self.k = int(self._kb.sum())
        self.ld = padded_ld(d) if ld is None else int(ld)
        self.device = torch.device(device)
        dev = self.device
        f32 = dict(dtype=torch.float32, device=dev)
        if views is not None:
            self.theta, self.m, self.v, self.vhat = views["theta"], views["m"], views["v"], views["vhat"]
            self.e = views.get("e")
            for t in (self.theta, self.m, self.v, self.vhat):
                assert t.is_cuda and t.dtype == torch.float32 and t.numel() == self.d and t.is_contiguous()
            assert self.e is None or (self.e.stride(0) == self.ld and self.e.stride(1) == 1)
        else:
            self.theta = theta0.detach().to(**f32).clone().contiguous()
            assert self.theta.numel() == self.d
            self.m = torch.empty(self.d, **f32)
            self.v = torch.empty(self.d, **f32)
            self.vhat = torch.empty(self.d, **f32)
            self.e = torch.zeros((self.n, self.ld), **f32) if compressor != NONE else None
        flags = 0
        if state is not None:
            flags |= KEEP_STATE
            self.m.copy_(state["m"]); self.v.copy_(state["v"]); self.vhat.copy_(state["vhat"])
            if self.e is not None:
                self.e.zero_()
                self.e[:, : self.d].copy_(state["e"])
        cfg = compams_config()
        cfg.n, cfg.d, cfg.ld, cfg.compressor, cfg.k = self.n, self.d, self.ld, compressor, self.k
        self._off = None
        self.M = 0
        if block_offsets is not None:
            self._off = np.ascontiguousarray(block_offsets, dtype=np.int64)
            self.M = self._off.size - 1
            cfg.block_offsets = self._off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        cfg.num_blocks = self.M
        if self._kb is not None:
            cfg.block_k = self._kb.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        cfg.beta1, cfg.beta2, cfg.eps, cfg.eps_mode, cfg.flags = beta1, beta2, eps, eps_mode, flags
        cfg.theta, cfg.m, cfg.v, cfg.vhat = (self.theta.data_ptr(), self.m.data_ptr(), self.v.data_ptr(),
                                             self.vhat.data_ptr())
        cfg.e = self.e.data_ptr() if self.e is not None else None
        L = lib()
        with torch.cuda.device(dev):
            nbytes = L.compams_workspace_size(ctypes.byref(cfg))
            if nbytes == 0:
                raise CompamsError("compams_workspace_size: invalid configuration")
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            cfg.workspace, cfg.workspace_bytes = self.workspace.data_ptr(), nbytes
            torch.cuda.synchronize(dev)
            h = ctypes.c_void_p()
            _check(L.compams_init(ctypes.byref(cfg), ctypes.byref(h)), "compams_init")
        self._h = h
        self._cfg = cfg

    # -- the three calls of the boundary ---------------------------------------------------------
    def compams_step(self, g: torch.Tensor, lr: float):
        """g: n x ld fp32 tensor on the context's device (columns >= d ignored)."""
        assert g.dtype == torch.float32 and g.is_cuda and g.is_contiguous()
        assert g.shape == (self.n, self.ld), f"g must be {self.n} x {self.ld}, got {tuple(g.shape)}"
        with torch.cuda.device(self.device):
            _check(lib().compams_step(self._h, g.data_ptr(), lr, _current_stream_handle()), "compams_step")

    def compams_state(self, name: str):
        """A torch view (no copy) of a state tensor or of the last step's messages ("pending": a bool)."""
        p = ctypes.c_void_p()
        cnt = ctypes.c_int64()
        _check(lib().compams_state(self._h, STATE[name], ctypes.byref(p), ctypes.byref(cnt)), "compams_state")
        if name == "pending":   # a host-side answer: is the last step's error line still to be applied?
            return bool(cnt.value)
        dt = _STATE_DTYPE.get(name, torch.float32)
        t = _tensor_from_ptr(p.value, cnt.value, dt, self.device, keepalive=self)
        if name == "e":
            return t.view(self.n, self.ld)[:, : self.d]
        if name in ("last_idx", "last_val"):
            return t.view(self.n, self.k)
        if name in ("last_signbits",):
            return t.view(self.n, -1)
        if name == "last_scales":
            return t.view(self.n, self.M)
        if name == "counters":
            return t.view(-1, COUNTERS_PER_ROW)
        return t

    # -- the messages on the wire ----------------------------------------------------------------
    def compams_wire_capacity(self) -> int:
        """Largest message of one worker, in 32-bit words."""
        return int(lib().compams_wire_capacity(ctypes.byref(self._cfg)))

    def compams_encode(self, stride_words=None):
        """Packs the last step's messages: (messages int32[n, stride] viewed as raw words, words int32[n])."""
        stride = self.compams_wire_capacity() if stride_words is None else int(stride_words)
        messages = torch.empty((self.n, stride), dtype=torch.int32, device=self.device)
        words = torch.empty(self.n, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib().compams_encode(self._h, messages.data_ptr(), stride, words.data_ptr(),
                                        _current_stream_handle()), "compams_encode")
        return messages, words

    def compams_decode(self, messages: torch.Tensor, words=None):
        """Unpacks n messages: (idx int32[n, k], val float[n, k]) or (sign words int32[n, W], scales float[n, M]),
        and the per-message status words."""
        assert messages.dtype == torch.int32 and messages.is_cuda and messages.is_contiguous()
        assert messages.shape[0] == self.n
        if self.compressor in (TOPK, TOPK_BLOCKS):
            a = torch.empty((self.n, self.k), dtype=torch.int32, device=self.device)
            b = torch.empty((self.n, self.k), dtype=torch.float32, device=self.device)
        else:
            a = torch.empty((self.n, (self.d + 31) // 32), dtype=torch.int32, device=self.device)
            b = torch.empty((self.n, self.M), dtype=torch.float32, device=self.device)
        status = torch.empty(self.n, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib().compams_decode(self._h, messages.data_ptr(), messages.shape[1],
                                        None if words is None else words.data_ptr(), a.data_ptr(), b.data_ptr(),
                                        status.data_ptr(), _current_stream_handle()), "compams_decode")
        return a, b, status

    # -- the two halves of a step ----------------------------------------------------------------
    def compams_worker_step(self, g: torch.Tensor):
        """The workers' lines only: compresses, updates e, leaves the messages for compams_encode."""
        assert g.dtype == torch.float32 and g.is_cuda and g.is_contiguous()
        assert g.shape == (self.n, self.ld), f"g must be {self.n} x {self.ld}, got {tuple(g.shape)}"
        with torch.cuda.device(self.device):
            _check(lib().compams_worker_step(self._h, g.data_ptr(), _current_stream_handle()), "compams_worker_step")

    def compams_server_step(self, messages: torch.Tensor, words, lr: float) -> torch.Tensor:
        """The server's lines from n packed messages; returns the per-message status words."""
        assert messages.dtype == torch.int32 and messages.is_cuda and messages.is_contiguous()
        assert messages.shape[0] == self.n
        status = torch.empty(self.n, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            _check(lib().compams_server_step(self._h, messages.data_ptr(), messages.shape[1],
                                             None if words is None else words.data_ptr(), lr, status.data_ptr(),
                                             _current_stream_handle()), "compams_server_step")
        return status

    # -- extras ----------------------------------------------------------------------------------
    def set_option(self, option: int, value: int):
        _check(lib().compams_set_option(self._h, option, value), "compams_set_option")

    def profile_enable(self, mode: int):
        """0 off, 1 every kernel, 2 only the kernel that moves most of the bytes."""
        _check(lib().compams_profile_enable(self._h, int(mode)), "compams_profile_enable")

    def profile_read(self):
        cap = 32
        names = (ctypes.c_char_p * cap)()
        ms = (ctypes.c_double * cap)()
        launches = (ctypes.c_int64 * cap)()
        cnt = ctypes.c_int()
        _check(lib().compams_profile_read(self._h, cap, names, ms, launches, ctypes.byref(cnt)),
               "compams_profile_read")
        return {names[i].decode(): (ms[i], launches[i]) for i in range(min(cnt.value, cap))}

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            lib().compams_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _tensor_from_ptr(ptr: int, count: int, dtype: torch.dtype, device, keepalive=None) -> torch.Tensor:
    """Wrap borrowed device memory as a torch tensor through the CUDA array interface."""
    itemsize = torch.empty(0, dtype=dtype).element_size()
    typestr = {torch.float32: "<f4", torch.int32: "<i4", torch.uint8: "|u1"}[dtype]

    class _Holder:
        pass

    hld = _Holder()
    hld.__cuda_array_interface__ = {"shape": (int(count),), "typestr": typestr, "data": (int(ptr), False),
                                    "version": 2, "strides": None}
    hld._keepalive = keepalive
    if count == 0:
        return torch.empty(0, dtype=dtype, device=device)
    t = torch.as_tensor(hld, device=device)
    assert t.element_size() == itemsize
    return t


def compams_step_static(n: int, d: int, k: int, theta, m, v, vhat, e, g, lr: float, idx_out=None, val_out=None,
                        beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, eps_mode: int = EPS_IN_SQRT,
                        keep_state: bool = True) -> int:
    """One whole top-k step on the caller's tensors with the library's built-in scratch array: marshals the
    arguments of the C entry point of the same name and returns its status (no exception: callers test for the
    rejection codes).  e and g are n x ld (ld = their common row stride)."""
    cfg = compams_config()
    cfg.n, cfg.d, cfg.ld, cfg.compressor, cfg.k = int(n), int(d), int(e.stride(0)), TOPK, int(k)
    cfg.beta1, cfg.beta2, cfg.eps, cfg.eps_mode = beta1, beta2, eps, eps_mode
    cfg.flags = KEEP_STATE if keep_state else 0
    cfg.theta, cfg.m, cfg.v, cfg.vhat, cfg.e = theta.data_ptr(), m.data_ptr(), v.data_ptr(), vhat.data_ptr(), e.data_ptr()
    assert g.stride(0) == e.stride(0) and g.is_cuda and g.dtype == torch.float32
    with torch.cuda.device(e.device):
        return lib().compams_step_static(ctypes.byref(cfg), g.data_ptr(), lr,
                                         None if idx_out is None else idx_out.data_ptr(),
                                         None if val_out is None else val_out.data_ptr(), _current_stream_handle())


def compams_cached_state_arrays(d: int) -> int:
    """How many of theta, m, v, vhat the server kernels keep in the memory-side cache for a problem of d coordinates."""
    count = lib().compams_cached_state_arrays(d)
    if count < 0:
        _check(count, "compams_cached_state_arrays")
    return count


def compams_inplace_probe(arrays, cached_arrays: int):
    """x += 1 on up to four separately allocated fp32 arrays of one size, in the access pattern of the server's
    lines of Algorithm 2 (the measured ceiling for the kernels that apply them); the first cached_arrays of them
    with ordinary accesses, the others with streaming ones."""
    count = arrays[0].numel()
    assert all(a.numel() == count and a.dtype == torch.float32 and a.is_cuda and a.is_contiguous() for a in arrays)
    ptrs = (ctypes.c_void_p * len(arrays))(*[a.data_ptr() for a in arrays])
    _check(lib().compams_inplace_probe(ptrs, len(arrays), count, int(cached_arrays), _current_stream_handle()),
           "compams_inplace_probe")


def compams_copy(dst: torch.Tensor, src: torch.Tensor):
    """The library's plain streaming copy kernel (bandwidth ceiling / counter calibration)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().compams_copy(dst.data_ptr(), src.data_ptr(), nbytes, _current_stream_handle()), "compams_copy")
