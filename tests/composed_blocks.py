"""A comparator for the library's top-k inside every block (COMPAMS_TOPK_BLOCKS), built by composition.

The average and the AMSGrad lines of Algorithm 2 act coordinate by coordinate, and Definition 1 applied per block
looks at one block at a time, so the step falls apart into one independent whole-row top-k step per block on the
block's slice of g, e, theta, m, v, vhat.  The class below lays one ordinary top-k context over every slice of
shared buffers and steps them one after the other: a second route to the same result that the tests compare
bit for bit with the single-context form (and with the oracle).  Test infrastructure, not part of the package."""
import ctypes
from typing import Optional

import numpy as np
import torch

from paper_2205_05632_amd import binding as B


class CompamsBlockTopk:
    """Block b keeps block_k[b] coordinates per worker: one context per block, stepped one after the other on
    the same stream.  Block offsets must be multiples of 4 (16-byte aligned slices)."""

    def __init__(self, n: int, d: int, theta0: torch.Tensor, block_offsets, block_k, beta1: float = 0.9,
                 beta2: float = 0.999, eps: float = 1e-8, eps_mode: int = B.EPS_IN_SQRT, ld: Optional[int] = None,
                 device="cuda:0"):
        self.n, self.d = int(n), int(d)
        self.off = np.ascontiguousarray(block_offsets, dtype=np.int64)
        self.kb = np.ascontiguousarray(block_k, dtype=np.int64)
        if self.off[0] != 0 or self.off[-1] != d or self.kb.size != self.off.size - 1:
            raise B.CompamsError("block offsets must run from 0 to d, with one count per block")
        if (self.off[:-1] % 4).any():
            raise B.CompamsError("block offsets must be multiples of 4 (16-byte aligned slices)")
        self.k = int(self.kb.sum())
        self.ld = B.padded_ld(d) if ld is None else int(ld)
        self.device = torch.device(device)
        f32 = dict(dtype=torch.float32, device=self.device)
        self.theta = theta0.detach().to(**f32).clone().contiguous()
        self.m = torch.empty(self.d, **f32)
        self.v = torch.empty(self.d, **f32)
        self.vhat = torch.empty(self.d, **f32)
        self.e = torch.zeros((self.n, self.ld), **f32)
        self.blocks = []
        for b in range(self.kb.size):
            lo, hi = int(self.off[b]), int(self.off[b + 1])
            views = {"theta": self.theta[lo:hi], "m": self.m[lo:hi], "v": self.v[lo:hi], "vhat": self.vhat[lo:hi],
                     "e": self.e[:, lo:hi]}
            self.blocks.append(B.Compams(n, hi - lo, None, compressor=B.TOPK, k=int(self.kb[b]), beta1=beta1, beta2=beta2,
                                       eps=eps, eps_mode=eps_mode, ld=self.ld, device=device, views=views))

    def compams_step(self, g: torch.Tensor, lr: float):
        assert g.dtype == torch.float32 and g.is_cuda and g.is_contiguous() and g.shape == (self.n, self.ld)
        with torch.cuda.device(self.device):
            stream = B._current_stream_handle()
            for b, c in enumerate(self.blocks):
                B._check(B.lib().compams_step(c._h, g.data_ptr() + 4 * int(self.off[b]), lr, stream), "compams_step")

    def compams_state(self, name: str) -> torch.Tensor:
        if name in ("theta", "m", "v", "vhat"):
            return getattr(self, name)
        if name == "e":
            for c in self.blocks:     # asking a block for its residuals applies what is pending there
                p, cnt = ctypes.c_void_p(), ctypes.c_int64()
                B._check(B.lib().compams_state(c._h, B.STATE["e"], ctypes.byref(p), ctypes.byref(cnt)), "compams_state")
            return self.e[:, : self.d]
        if name == "last_idx":
            return torch.cat([c.compams_state("last_idx") + int(self.off[b]) for b, c in enumerate(self.blocks)], dim=1)
        if name == "last_val":
            return torch.cat([c.compams_state("last_val") for c in self.blocks], dim=1)
        raise B.CompamsError(f"no such state for per-block top-k: {name}")

    def close(self):
        for c in self.blocks:
            c.close()
        self.blocks = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
