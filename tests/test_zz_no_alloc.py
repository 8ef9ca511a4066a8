"""compams_step_static (the entry point that allocates nothing: its selection tables live in a device array inside
the library) against the existing entry points compams_init + compams_step + compams_state(E) + compams_destroy on
the same inputs: bit-identical parameters, moments, residuals and messages, on calls in a row that share the
array, the later ones with smaller inputs; and against the oracle."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

from parity import bits_equal

pytestmark = pytest.mark.gpu


def make_state(rng, n, d, ld, dev):
    """A mid-training state: nonzero moments and residuals."""
    st = {"theta": rng.standard_normal(d).astype(np.float32) * 0.1,
          "m": rng.standard_normal(d).astype(np.float32) * 1e-2,
          "v": (rng.standard_normal(d).astype(np.float32) * 1e-2) ** 2}
    st["vhat"] = np.maximum(st["v"], (rng.standard_normal(d).astype(np.float32) * 1e-2) ** 2)
    e = np.zeros((n, ld), dtype=np.float32)
    e[:, :d] = rng.standard_normal((n, d)).astype(np.float32) * 0.05
    e[:, : d : 7] = 0.0
    st["e"] = e
    return st


def grads(rng, n, d, ld):
    g = np.zeros((n, ld), dtype=np.float32)
    g[:, :d] = (rng.standard_normal((n, d)) * 10.0 ** rng.uniform(-3, 0, (1, d))).astype(np.float32)
    return g


def via_context(n, d, k, ld, st, g_list, lr, eps_mode, dev):
    """The existing entry points: one context, len(g_list) steps, everything read back at the end."""
    gpu = B.Compams(n, d, torch.from_numpy(st["theta"]), compressor=B.TOPK, k=k, ld=ld, eps_mode=eps_mode, device=dev,
                    state={"m": torch.from_numpy(st["m"]), "v": torch.from_numpy(st["v"]),
                           "vhat": torch.from_numpy(st["vhat"]), "e": torch.from_numpy(st["e"][:, :d])})
    for g in g_list:
        gpu.compams_step(torch.from_numpy(g).to(dev), lr)
    torch.cuda.synchronize()
    out = {name: np.ascontiguousarray(gpu.compams_state(name).cpu().numpy()) for name in ("theta", "m", "v", "vhat", "e")}
    out["idx"] = gpu.compams_state("last_idx").cpu().numpy()
    out["val"] = gpu.compams_state("last_val").cpu().numpy()
    gpu.close()
    return out


def via_static(n, d, k, ld, st, g_list, lr, eps_mode, dev):
    """The new entry point, once per step, on plain tensors; nothing but those tensors lives between the calls."""
    t = {name: torch.from_numpy(st[name]).to(dev) for name in ("theta", "m", "v", "vhat", "e")}
    idx = torch.full((n, k), -1, dtype=torch.int32, device=dev)
    val = torch.zeros((n, k), dtype=torch.float32, device=dev)
    for g in g_list:
        gd = torch.from_numpy(g).to(dev)
        status = B.compams_step_static(n, d, k, t["theta"], t["m"], t["v"], t["vhat"], t["e"], gd, lr, idx_out=idx,
                                       val_out=val, eps_mode=eps_mode)
        assert status == 0, B.compams_strerror(status)
    torch.cuda.synchronize()
    out = {name: t[name].cpu().numpy() for name in ("theta", "m", "v", "vhat")}
    out["e"] = np.ascontiguousarray(t["e"].cpu().numpy()[:, :d])
    out["pad"] = t["e"].cpu().numpy()[:, d:]
    out["idx"], out["val"] = idx.cpu().numpy(), val.cpu().numpy()
    return out


def via_oracle(n, d, k, st, g_list, lr, eps_mode):
    cpu = O.Oracle(n, d, st["theta"], compressor=O.TOPK, k=k, eps_mode=eps_mode)
    cpu.set_state(m=st["m"], v=st["v"], vhat=st["vhat"], e=np.ascontiguousarray(st["e"][:, :d]))
    for g in g_list:
        cpu.step(np.ascontiguousarray(g[:, :d]), lr)
    out = {name: cpu.get(name).copy() for name in ("theta", "m", "v", "vhat", "e", "idx", "val")}
    cpu.close()
    return out


# calls in a row on the one device array: a larger problem first, then smaller ones (rows of 17, 5 and 1 chunks,
# a ragged tail, ties, k = 1), then a larger one again
SHAPES = [(4, 65536 + 1234, 655, 2), (3, 20000, 37, 1), (2, 4096, 4096, 1), (5, 1000, 1, 2), (4, 70000, 700, 1)]


def test_calls_in_a_row_share_the_array_and_match_the_existing_entry_points():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(2205)
    for case, (n, d, k, steps) in enumerate(SHAPES):
        ld = B.padded_ld(d)
        st = make_state(rng, n, d, ld, dev)
        g_list = [grads(rng, n, d, ld) for _ in range(steps)]
        if case == 2:
            g_list[0][:, :d] = np.round(g_list[0][:, :d] * 4) / 4      # many equal magnitudes
        eps_mode = B.EPS_OUT_SQRT if case % 2 else B.EPS_IN_SQRT
        got = via_static(n, d, k, ld, st, g_list, 1e-3, eps_mode, dev)
        want = via_context(n, d, k, ld, st, g_list, 1e-3, eps_mode, dev)
        orc = via_oracle(n, d, k, st, g_list, 1e-3, eps_mode)
        assert not got["pad"].any(), f"case {case}: columns beyond d were touched"
        assert np.array_equal(got["idx"], want["idx"]) and np.array_equal(got["idx"], orc["idx"]), f"case {case}: index sets"
        for name in ("val", "theta", "m", "v", "vhat", "e"):
            assert bits_equal(got[name], want[name]), f"case {case}: {name} differs from the existing entry points"
            assert bits_equal(got[name], orc[name]), f"case {case}: {name} differs from the oracle"


def test_first_step_form_zeroes_the_state():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(7)
    n, d, k = 3, 30000, 300
    ld = B.padded_ld(d)
    theta0 = rng.standard_normal(d).astype(np.float32) * 0.1
    g = grads(rng, n, d, ld)
    junk = lambda *shape: torch.full(shape, 3.0, dtype=torch.float32, device=dev)
    theta, m, v, vhat, e = torch.from_numpy(theta0).to(dev), junk(d), junk(d), junk(d), junk(n, ld)
    status = B.compams_step_static(n, d, k, theta, m, v, vhat, e, torch.from_numpy(g).to(dev), 1e-3, keep_state=False)
    assert status == 0
    torch.cuda.synchronize()
    cpu = O.Oracle(n, d, theta0, compressor=O.TOPK, k=k)
    cpu.step(np.ascontiguousarray(g[:, :d]), 1e-3)
    for name, t in (("theta", theta), ("m", m), ("v", v), ("vhat", vhat)):
        assert bits_equal(t.cpu().numpy(), cpu.get(name)), name
    assert bits_equal(np.ascontiguousarray(e.cpu().numpy()[:, :d]), cpu.get("e"))
    cpu.close()


def test_sizes_beyond_the_array_and_other_compressors_are_rejected():
    dev = torch.device("cuda:0")
    L = B.lib()
    t = torch.zeros(4096, dtype=torch.float32, device=dev)
    c = B.compams_config()
    c.n, c.d, c.ld, c.compressor, c.k = 16, 11181642, 11182080, B.TOPK, 111816     # needs 156 MB of tables
    c.beta1, c.beta2, c.eps = 0.9, 0.999, 1e-8
    c.theta = c.m = c.v = c.vhat = c.e = t.data_ptr()       # never touched: the size check comes first
    assert L.compams_workspace_size(ctypes.byref(c)) > B.STATIC_SCRATCH_BYTES
    assert L.compams_step_static(ctypes.byref(c), t.data_ptr(), 1e-3, None, None, None) == -3
    c.n, c.d, c.ld, c.k = 2, 1000, 1000, 10
    assert 0 < L.compams_workspace_size(ctypes.byref(c)) <= B.STATIC_SCRATCH_BYTES
    c.compressor = B.NONE
    assert L.compams_step_static(ctypes.byref(c), t.data_ptr(), 1e-3, None, None, None) == -5
    c.compressor = B.TOPK
    assert L.compams_step_static(ctypes.byref(c), None, 1e-3, None, None, None) == -1
    assert L.compams_step_static(None, t.data_ptr(), 1e-3, None, None, None) == -1
    c.ld = 1002
    assert L.compams_step_static(ctypes.byref(c), t.data_ptr(), 1e-3, None, None, None) == -2
    torch.cuda.synchronize()
    assert not t.cpu().numpy().any()
