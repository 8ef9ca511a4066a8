"""Seeded random configurations: worker count, row length, row pitch, compressor, k, block layout and the kind of
gradient values are all drawn from the seed, and every step of the HIP library (through the C ABI) is compared
with the oracle to the bar of the other parity tests -- index sets, values, sign words and scales bit for bit,
floats within 1e-5.  The fixed cases elsewhere aim at known corners; this sweep is for the ones nobody thought of."""
import os

import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

from parity import Pair
from test_gpu_topk_blocks import BlockPair

pytestmark = pytest.mark.gpu

ROUTES = {"band": 0, "general": 0, "reread": 0}   # selection problems per route over the whole sweep (steps after the first)


def tally(gpu, t):
    if t == 0:
        return
    torch.cuda.synchronize()
    c = gpu.compams_state("counters").cpu().numpy()
    ROUTES["band"] += int((c[:, 4] > 0).sum())
    ROUTES["general"] += int(((c[:, 4] == 0) & (c[:, 5] > 1)).sum())
    ROUTES["reread"] += int((c[:, 0] > 0).sum())


def draw_gradients(rng, kind, n, d):
    if kind == "scaled":        # per-coordinate scales over eight decades
        g = rng.standard_normal((n, d)) * 10.0 ** rng.uniform(-6, 2, (1, d))
    elif kind == "sparse":      # half the coordinates exactly zero, in runs
        g = rng.standard_normal((n, d))
        g[:, np.repeat(rng.random((d + 63) // 64) < 0.5, 64)[:d]] = 0.0
    elif kind == "heavy":       # heavy tails
        g = rng.standard_t(2, (n, d)) * 1e-2
    elif kind == "ties":        # few distinct magnitudes, both signs and both zeros
        g = rng.integers(-3, 4, (n, d)).astype(np.float64) * 0.25
        g[:, ::5] *= -1.0
    elif kind == "denormal":    # denormals beside ordinary numbers
        g = rng.standard_normal((n, d))
        g[:, ::3] *= 1e-41
    else:                       # every other call brings a few entries that are not finite, or nearly so
        g = rng.standard_normal((n, d))
        if rng.random() < 0.5:
            pool = [np.nan, -np.nan] if kind == "nans" else [np.inf, -np.inf, np.nan, -np.nan, 3.0e38, -3.0e38]
            m = int(rng.integers(1, 7))
            g[rng.integers(0, n, m), rng.integers(0, d, m)] = rng.choice(pool, m)
    return g.astype(np.float32)


def draw_config(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16, 33]))
    d = int(10.0 ** (rng.uniform(0.0, 5.3) if rng.random() < 0.35 else rng.uniform(3.6, 5.3)))  # most span chunks
    d = max(1, min(d, 200000 // n * 4))
    if rng.random() < 0.15:     # long rows: 64 chunks and more, where the candidate list is kept as eight runs
        n = int(rng.choice([1, 2, 3, 4]))
        d = int(rng.integers(64 * 4096, 150 * 4096))
    compressor = ["topk", "blocksign", "topk_blocks", "none"][int(rng.choice(4, p=[0.35, 0.3, 0.3, 0.05]))]
    if compressor == "topk_blocks" and d < 8:
        d = 8 + 4 * int(rng.integers(0, 8))
    ld = None
    if rng.random() < 0.5:
        ld = (d + 3) // 4 * 4 + 4 * int(rng.integers(0, 6))
    kind = ["scaled", "sparse", "heavy", "ties", "denormal", "specials"][int(rng.integers(0, 6))]
    if kind == "specials" and compressor == "none":
        kind = "nans"           # an infinite entry is where the library follows Algorithm 1 and the oracle the literal
                                # error line of Algorithm 2 (a test of its own covers that)
    cfg = dict(seed=seed, n=n, d=d, ld=ld, compressor=compressor, kind=kind)
    if compressor == "topk":
        cfg["k"] = int(rng.choice([1, d, max(1, d // 100), int(rng.integers(1, d + 1))]))
    elif compressor == "blocksign":
        m = int(min(d, rng.choice([1, 2, 7, 40, 300])))
        cuts = np.sort(rng.choice(np.arange(1, d), size=m - 1, replace=False)) if m > 1 else []
        cfg["off"] = np.concatenate([[0], cuts, [d]]).astype(np.int64)
    elif compressor == "topk_blocks":
        d = d // 4 * 4          # block offsets are multiples of 4; the last block may end anywhere, here it does not
        cfg["d"] = d
        cfg["ld"] = None
        m = int(min(d // 4, rng.choice([1, 2, 5, 30, 200])))
        cuts = np.sort(rng.choice(np.arange(1, d // 4), size=m - 1, replace=False)) * 4 if m > 1 else []
        off = np.concatenate([[0], cuts, [d]]).astype(np.int64)
        size = off[1:] - off[:-1]
        frac = rng.choice([0.001, 0.01, 0.3, 1.0], size=len(size))
        cfg["off"] = off
        cfg["kb"] = np.clip((size * frac).astype(np.int64), 1, size)
    return cfg, rng


# COMPAMS_RANDOM_CONFIGS=<count> widens the sweep for an occasional longer run, COMPAMS_RANDOM_FIRST=<seed> moves it
FIRST = int(os.environ.get("COMPAMS_RANDOM_FIRST", "0"))


@pytest.mark.parametrize("seed", range(FIRST, FIRST + int(os.environ.get("COMPAMS_RANDOM_CONFIGS", "120"))))
def test_random_configuration(seed):
    cfg, rng = draw_config(seed)
    n, d = cfg["n"], cfg["d"]
    label = " ".join(f"{k}={v}" for k, v in cfg.items() if k not in ("off", "kb"))
    print(label, flush=True)
    theta0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    steps = 9 if seed % 3 == 0 else 4      # the longer ones give the one-launch selection time to settle in
    if cfg["compressor"] == "topk_blocks":
        p = BlockPair(n, d, cfg["off"], cfg["kb"], theta0)
        for t in range(steps):
            with np.errstate(invalid="ignore", over="ignore"):
                p.step(draw_gradients(rng, cfg["kind"], n, d))
            p.compare(f"{label} step {t}", with_e=(t % 2 == 1))
            tally(p.gpu, t)
    else:
        comp = {"topk": B.TOPK, "blocksign": B.BLOCKSIGN, "none": B.NONE}[cfg["compressor"]]
        p = Pair(n, d, theta0, comp, k=cfg.get("k", 0), block_offsets=cfg.get("off"), ld=cfg["ld"])
        for t in range(steps):
            with np.errstate(invalid="ignore", over="ignore"):
                p.step(draw_gradients(rng, cfg["kind"], n, d), 1e-3, label=f"{label} step {t}", with_e=(t % 2 == 1))
            if comp == B.TOPK:
                tally(p.gpu, t)
    p.close()


def test_the_sweep_took_every_route():
    """The configurations above must have exercised the one-launch selection, the general kernels with a usable
    candidate list, and the re-read of a row, many times each (else the sweep no longer tests what it is for)."""
    print(ROUTES, flush=True)
    assert ROUTES["band"] > 200 and ROUTES["general"] > 200 and ROUTES["reread"] > 100, ROUTES
