"""The one-launch selection (the threshold key found inside a window carried over from the last two steps) against
the oracle: every step of every case is compared bit for bit like everywhere else; on top of that the counter
COMPAMS_CNT_BAND says which route a row took, and the cases below make each way into and out of the route happen:
drifting thresholds, jumps out of the window in both directions, ties at the threshold (ranked by coordinate,
few and too many), windows that overflow, rows of one run and of eight runs, blocks, and the option that switches
the route off (same bytes either way)."""
import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

from parity import Pair
from test_gpu_topk_blocks import BlockPair, make_blocks

pytestmark = pytest.mark.gpu
BAND = 4   # COMPAMS_CNT_BAND


def band_counter(p):
    torch.cuda.synchronize()
    return p.gpu.compams_state("counters").cpu().numpy()[:, BAND].copy()


@pytest.mark.parametrize("n,d,k", [(4, 65536, 655), (3, 70 * 4096 + 100, 3000), (2, 5000, 400), (5, 300001, 30000)])
def test_stationary_gradients_settle_on_the_band_route(n, d, k):
    """Residuals build up, the threshold drifts less and less, and after a few steps every row is selected in one
    launch; rows of fewer than 64 chunks keep one run of each list, longer ones eight."""
    rng = np.random.default_rng(d + k)
    p = Pair(n, d, rng.standard_normal(d).astype(np.float32) * 0.1, B.TOPK, k=k)
    used = []
    scale = 10.0 ** rng.uniform(-2, 0, (1, d))
    for t in range(14):
        g = (rng.standard_normal((n, d)) * scale).astype(np.float32)
        p.step(g, 1e-3, label=f"stationary step {t}", with_e=(t % 5 == 4))
        used.append(band_counter(p))
    used = np.array(used)
    assert (used[:2] == 0).all(), used            # nothing to extrapolate from yet
    assert (used[-3:] > 0).all(), used            # steady state: every row, every step
    assert all(p.exact.values()), p.exact
    p.close()


def test_band_switched_off_gives_the_same_bytes():
    n, d, k = 3, 150000, 1500
    rng = np.random.default_rng(5)
    gs = [(rng.standard_normal((n, d))).astype(np.float32) for _ in range(9)]
    outs = []
    for band in (1, 0):
        p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=k)
        p.gpu.set_option(B.OPT_BAND, band)
        used = []
        for t, g in enumerate(gs):
            p.step(g, 1e-3, label=f"band={band} step {t}")
            used.append(band_counter(p))
        used = np.array(used)
        assert (used[-2:] > 0).all() if band else (used == 0).all(), used
        outs.append([p.gpu.compams_state(s).cpu().numpy().copy() for s in ("theta", "m", "v", "vhat", "e", "last_idx", "last_val")])
        p.close()
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("factor", [3.0, 1.3, 0.8, 0.3, 1e-3])
def test_threshold_jumping_out_of_the_band(factor):
    """The gradients change scale at once: the window misses (upwards: everything needed is still in the candidate
    list; downwards: it may not be), the general kernels take the step, and the route comes back."""
    n, d, k = 3, 200000, 2000
    rng = np.random.default_rng(int(factor * 1000))
    p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=k)
    used = []
    for t in range(16):
        scale = 1.0 if t < 8 else factor
        g = (rng.standard_normal((n, d)) * scale).astype(np.float32)
        if t == 8:
            p.gpu.e.zero_()                 # drop the residuals so that the threshold really moves
            p.cpu.set_state(e=np.zeros((n, d), np.float32))
        p.step(g, 1e-3, label=f"jump x{factor} step {t}", with_e=False)
        used.append(band_counter(p))
    used = np.array(used)
    assert (used[7] > 0).all() and (used[8] == 0).all() and (used[-1] > 0).all(), used
    p.compare("after the jump")
    p.close()


@pytest.mark.parametrize("levels,expect_band", [(6000, True), (3000, True), (300, False)])
def test_ties_at_the_threshold(levels, expect_band):
    """Magnitudes drawn from a fixed set of `levels` values: the threshold key is shared by d / levels coordinates,
    of which only some are kept, in coordinate order.  Up to 64 entries in the threshold's bucket are ranked
    inside the one launch; with more the general kernels rank them."""
    n, d, k = 3, 120000, 1777
    rng = np.random.default_rng(levels)
    table = np.sort(np.abs(rng.standard_normal(levels)).astype(np.float32) + 0.01)
    p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=k)
    used, ties = [], []
    for t in range(8):
        g = (table[rng.integers(0, levels, (n, d))] * rng.choice([-1.0, 1.0], (n, d))).astype(np.float32)
        p.gpu.e.zero_()                     # no residuals: x is g, with its few distinct magnitudes
        p.cpu.set_state(e=np.zeros((n, d), np.float32))
        p.step(g, 1e-3, label=f"{levels} levels step {t}", with_e=False)
        c = p.gpu.compams_state("counters").cpu().numpy()
        used.append(c[:, BAND].copy())
        ties.append(c[:, 2].copy())
    used, ties = np.array(used), np.array(ties)
    assert (ties[-1] > 1).all(), ties
    if expect_band:
        assert (used[-2:] > 0).any(), (used, ties)
    else:
        assert (ties[-1] > 64).all() and (used == 0).all(), (used, ties)
    p.close()


def test_special_values_arriving_on_the_band_route():
    """Once every row is selected in one launch, a step brings infinities, NaNs (the largest keys of all), values
    near the largest finite one and negative zeros: they lie far above the window, are kept like any other entry,
    and the rows stay on the route; the state then holds Inf and NaN at those coordinates on both sides."""
    n, d, k = 3, 33 * 4096 + 77, 1400
    rng = np.random.default_rng(77)
    p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=k)
    where = {"inf": [5, 4096 * 7 + 63, d - 1], "ninf": [4096, 4097], "nan": [64, 4096 * 20 + 1], "huge": [9, 70000],
             "nzero": [0, 1, 2, 3, 8191]}
    for t in range(12):
        g = rng.standard_normal((n, d)).astype(np.float32)
        if t == 7:
            g[:, where["inf"]] = np.inf
            g[1:, where["ninf"]] = -np.inf
            g[0, where["nan"]] = np.nan
            g[2, where["huge"]] = np.float32(-3.0e38)
            g[:, where["nzero"]] = np.float32(-0.0)
        with np.errstate(invalid="ignore", over="ignore"):
            p.step(g, 1e-3, label=f"special values step {t}", with_e=(t in (7, 11)))
        used = band_counter(p)
        if t >= 6:
            assert (used > 0).all(), (t, used)
        if t == 7:
            idx = p.gpu.compams_state("last_idx").cpu().numpy()
            assert all(np.isin(where["inf"], idx[i]).all() for i in range(n))
            assert np.isin(where["nan"], idx[0]).all() and np.isin(where["huge"], idx[2]).all()
    p.close()


def test_window_that_overflows_is_left_to_the_general_kernels():
    """Almost all magnitudes within a fraction of a per cent of each other: the window holds far more entries
    than the band list, in every step."""
    n, d, k = 2, 300000, 3000
    rng = np.random.default_rng(9)
    p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=k)
    for t in range(6):
        mag = 1.0 + 1e-3 * rng.random((n, d))
        g = (mag * rng.choice([-1.0, 1.0], (n, d))).astype(np.float32)
        p.gpu.e.zero_()
        p.cpu.set_state(e=np.zeros((n, d), np.float32))
        p.step(g, 1e-3, label=f"overflow step {t}", with_e=False)
        assert (band_counter(p) == 0).all()
    p.close()


def test_band_route_inside_blocks():
    """Top-k inside every block: each (worker, block) problem carries its own window; micro problems have none."""
    rng = np.random.default_rng(21)
    n, d = 3, 40 * 4096 + 8
    off, kb = make_blocks(d, 7, rng, frac=0.02)
    theta0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    p = BlockPair(n, d, off, kb, theta0)
    scale = 10.0 ** rng.uniform(-2, 0, (1, d))
    for t in range(12):
        p.step((rng.standard_normal((n, d)) * scale).astype(np.float32))
        p.compare(f"blocks step {t}", with_e=(t == 11))
    torch.cuda.synchronize()
    c = p.gpu.compams_state("counters").cpu().numpy()
    big = np.tile((off[1:] - off[:-1]) > 1024, n)
    assert (c[big, BAND] > 0).all() and (c[~big, BAND] == 0).all(), c[:, BAND]
    p.gpu.close(); p.cpu.close()


def test_worker_half_takes_the_band_route_too():
    n, d, k = 4, 65536, 655
    rng = np.random.default_rng(4)
    theta0 = np.zeros(d, np.float32)
    w = B.Compams(n, d, torch.from_numpy(theta0), compressor=B.TOPK, k=k)
    cpu = O.Oracle(n, d, theta0, compressor=O.TOPK, k=k)
    for t in range(10):
        g = rng.standard_normal((n, d)).astype(np.float32)
        gp = torch.zeros((n, w.ld), dtype=torch.float32)
        gp[:, :d] = torch.from_numpy(g)
        w.compams_worker_step(gp.to(w.device))
        cpu.step(g, 1e-3)
        torch.cuda.synchronize()
        assert np.array_equal(w.compams_state("last_idx").cpu().numpy(), cpu.get("idx")), f"step {t}"
    assert (w.compams_state("counters").cpu().numpy()[:, BAND] > 0).all()
    assert np.array_equal(np.ascontiguousarray(w.compams_state("e").cpu().numpy()).view(np.uint32),
                          cpu.get("e").view(np.uint32))
    w.close(); cpu.close()
