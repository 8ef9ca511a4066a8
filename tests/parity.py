"""Shared driver of the GPU-vs-oracle parity tests: runs both on the same inputs and compares."""
import numpy as np
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

RTOL = 1e-5  # the bar: |a - b| <= RTOL * |b| + RTOL * max|b|, per state tensor, after every step


def close(a, b, what, rtol=RTOL):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    nan_a, nan_b = np.isnan(a), np.isnan(b)
    assert np.array_equal(nan_a, nan_b), f"{what}: NaN pattern differs"
    fin = ~nan_b
    if not fin.any():
        return
    scale = np.max(np.abs(b[fin & np.isfinite(b)])) if (fin & np.isfinite(b)).any() else 0.0
    with np.errstate(invalid="ignore"):
        err = np.abs(a - b)
        same_inf = np.isinf(a) & np.isinf(b) & (np.sign(a) == np.sign(b))
        err[same_inf] = 0.0
        bad = fin & ~(err <= rtol * np.abs(b) + rtol * scale)
    if bad.any():
        j = np.argmax(np.where(bad, err, -1))
        raise AssertionError(f"{what}: {bad.sum()} of {a.size} outside tolerance; worst at {np.unravel_index(j, a.shape)}: "
                             f"gpu={a.flat[j]!r} oracle={b.flat[j]!r} scale={scale!r}")


def bits_equal(a, b):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


class Pair:
    """One GPU context and one oracle with identical configuration."""

    def __init__(self, n, d, theta0, compressor, k=0, block_offsets=None, eps_mode=B.EPS_IN_SQRT, ld=None,
                 beta1=0.9, beta2=0.999, eps=1e-8):
        theta0 = np.ascontiguousarray(theta0, dtype=np.float32)
        self.n, self.d, self.k, self.compressor = n, d, k, compressor
        self.gpu = B.Compams(n, d, torch.from_numpy(theta0), compressor=compressor, k=k,
                             block_offsets=block_offsets, eps_mode=eps_mode, ld=ld, beta1=beta1, beta2=beta2, eps=eps)
        self.cpu = O.Oracle(n, d, theta0, compressor=compressor, k=k, block_offsets=block_offsets,
                            eps_mode=eps_mode, beta1=beta1, beta2=beta2, eps=eps)
        self.exact = {"theta": True, "m": True, "v": True, "vhat": True, "e": True}

    def step(self, g, lr, check=True, label="", with_e=True):
        """g: numpy n x d.  Runs one step on both sides and compares everything."""
        g = np.ascontiguousarray(g, dtype=np.float32).reshape(self.n, self.d)
        gp = torch.zeros((self.n, self.gpu.ld), dtype=torch.float32)
        gp[:, : self.d] = torch.from_numpy(g)
        self.gpu.compams_step(gp.to(self.gpu.device), lr)
        self.cpu.step(g, lr)
        if check:
            self.compare(label, with_e=with_e)

    def compare(self, label="", with_e=True):
        """with_e=False leaves the residuals alone: asking for them makes the library settle its deferred
        zeroing, and the steps in between are then run in the other variant of the first pass."""
        gpu, cpu = self.gpu, self.cpu
        torch.cuda.synchronize()
        if self.compressor == B.TOPK:
            idx = gpu.compams_state("last_idx").cpu().numpy()
            val = gpu.compams_state("last_val").cpu().numpy()
            want_idx = cpu.get("idx")
            if not np.array_equal(idx, want_idx):
                rows = [i for i in range(self.n) if not np.array_equal(idx[i], want_idx[i])]
                i = rows[0]
                q = int(np.argmax(idx[i] != want_idx[i]))
                raise AssertionError(f"{label}: selected index sets differ in rows {rows}; row {i} first differs at "
                                     f"position {q}: gpu {idx[i][q:q+4]} oracle {want_idx[i][q:q+4]}")
            assert bits_equal(val, cpu.get("val")), f"{label}: selected values differ"
            # threshold key and the number of entries strictly above it, from the oracle's own selection
            keys = cpu.get("val").view(np.uint32) & 0x7FFFFFFF
            tau = keys.min(axis=1)
            assert np.array_equal(gpu.compams_state("last_threshold").cpu().numpy().view(np.uint32), tau), \
                f"{label}: threshold keys differ"
            assert np.array_equal(gpu.compams_state("last_count_gt").cpu().numpy(), (keys > tau[:, None]).sum(axis=1)), \
                f"{label}: counts above the threshold differ"
        elif self.compressor == B.BLOCKSIGN:
            bits = gpu.compams_state("last_signbits").cpu().numpy().view(np.uint32)
            assert np.array_equal(bits, cpu.get("bits")), f"{label}: sign patterns differ"
            mu = gpu.compams_state("last_scales").cpu().numpy()
            want_mu = cpu.get("mu")
            if not bits_equal(mu, want_mu):
                bad = np.argwhere(mu.view(np.uint32) != want_mu.view(np.uint32))
                raise AssertionError(f"{label}: {len(bad)} block scales differ, first (row, block) {bad[0]}: "
                                     f"gpu {mu[tuple(bad[0])]!r} oracle {want_mu[tuple(bad[0])]!r}")
        names = ["theta", "m", "v", "vhat"] + (["e"] if self.compressor != B.NONE and with_e else [])
        for name in names:
            a = gpu.compams_state(name).cpu().numpy()
            b = cpu.get(name)
            close(a, b, f"{label}: {name}")
            ok = ~np.isnan(b)       # a NaN is a NaN (close() has compared where they are): sign and payload are not part of the bar
            if not bits_equal(np.ascontiguousarray(a)[ok], b[ok]):
                self.exact[name] = False

    def close(self):
        self.gpu.close()
        self.cpu.close()
