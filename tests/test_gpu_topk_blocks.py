"""Top-k inside every block (layer tensor) as one context whose launches cover all blocks of all workers
(compressor TOPK_BLOCKS), against the oracle's per-block compressor, through the C ABI: lists, values, thresholds,
parameters, moments and residuals bit for bit."""
import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B
from composed_blocks import CompamsBlockTopk

pytestmark = pytest.mark.gpu


def make_blocks(d, blocks, rng, frac=0.03):
    cuts = np.sort(rng.choice(np.arange(1, d // 4), size=blocks - 1, replace=False)) * 4 if blocks > 1 else []
    off = np.concatenate([[0], cuts, [d]]).astype(np.int64)
    kb = np.maximum(1, ((off[1:] - off[:-1]) * frac).astype(np.int64))
    return off, kb


def grads(rng, n, d):
    g = (rng.standard_normal((n, d)) * 10.0 ** rng.uniform(-3, 0, (1, d))).astype(np.float32)
    g[:, ::6] = 0.0
    return g


class BlockPair:
    def __init__(self, n, d, off, kb, theta0, **kw):
        self.n, self.d, self.off, self.kb = n, d, off, kb
        self.gpu = B.Compams(n, d, torch.from_numpy(theta0), compressor=B.TOPK_BLOCKS, block_offsets=off, block_k=kb, **kw)
        self.cpu = O.Oracle(n, d, theta0, compressor=O.TOPK_BLOCKS, block_offsets=off, block_k=kb, **kw)

    def device_g(self, g):
        gp = torch.zeros((self.n, self.gpu.ld), dtype=torch.float32)
        gp[:, : self.d] = torch.from_numpy(g)
        return gp.to(self.gpu.device)

    def step(self, g, lr=1e-3):
        self.gpu.compams_step(self.device_g(g), lr)
        self.cpu.step(g, lr)

    def compare(self, label, with_e):
        gpu, cpu = self.gpu, self.cpu
        torch.cuda.synchronize()
        idx, want = gpu.compams_state("last_idx").cpu().numpy(), cpu.get("idx")
        if not np.array_equal(idx, want):
            i, q = np.argwhere(idx != want)[0]
            b = int(np.searchsorted(np.cumsum(self.kb), q, side="right"))
            raise AssertionError(f"{label}: lists differ first at worker {i}, entry {q} (block {b}, "
                                 f"columns {self.off[b]}..{self.off[b + 1]}, k {self.kb[b]}): gpu {idx[i, q:q + 4]} "
                                 f"oracle {want[i, q:q + 4]}")
        val = gpu.compams_state("last_val").cpu().numpy()
        assert np.array_equal(val.view(np.uint32), cpu.get("val").view(np.uint32)), f"{label}: values"
        # per (worker, block): the threshold key and how many entries lie strictly above it, from the oracle's lists
        keys = cpu.get("val").view(np.uint32) & 0x7FFFFFFF
        ends = np.cumsum(self.kb)
        tau = np.stack([keys[:, e - k:e].min(axis=1) for e, k in zip(ends, self.kb)], axis=1)
        gt = np.stack([(keys[:, e - k:e] > tau[:, b:b + 1]).sum(axis=1) for b, (e, k) in enumerate(zip(ends, self.kb))],
                      axis=1)
        got_tau = gpu.compams_state("last_threshold").cpu().numpy().view(np.uint32).reshape(self.n, -1)
        assert np.array_equal(got_tau, tau), f"{label}: threshold keys"
        assert np.array_equal(gpu.compams_state("last_count_gt").cpu().numpy().reshape(self.n, -1), gt), \
            f"{label}: counts above the threshold"
        for name in ("theta", "m", "v", "vhat") + (("e",) if with_e else ()):
            got = np.ascontiguousarray(gpu.compams_state(name).cpu().numpy())
            want = cpu.get(name)
            nan = np.isnan(want)    # a NaN is a NaN: its sign and payload are not part of the bar
            assert np.array_equal(np.isnan(got), nan), f"{label}: {name}: NaN pattern"
            assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan]), f"{label}: {name}"

    def close(self):
        self.gpu.close(); self.cpu.close()


SHAPES = [(3, 40000, 7), (2, 100000, 30), (5, 8192, 2), (2, 4 * 4096, 4096), (1, 300000, 5), (4, 70001 * 4, 1),
          (17, 12288, 3), (150, 6000, 9)]


@pytest.mark.parametrize("n,d,blocks", SHAPES)
@pytest.mark.parametrize("look_at_e", ["every step", "at the end"])
def test_fused_per_block_topk(n, d, blocks, look_at_e):
    """Reading e makes the library write the deferred zeros; not reading it leaves them to the next first pass."""
    rng = np.random.default_rng(d + blocks)
    off, kb = make_blocks(d, blocks, rng)
    theta0 = rng.standard_normal(d).astype(np.float32) * 0.1
    p = BlockPair(n, d, off, kb, theta0)
    for t in range(5):
        p.step(grads(rng, n, d))
        p.compare(f"step {t}", with_e=(look_at_e == "every step" or t == 4))
    p.close()


def test_blocks_where_everything_or_one_coordinate_is_kept():
    rng = np.random.default_rng(5)
    off = np.array([0, 4, 8, 4104, 4108, 20000, 20004], dtype=np.int64)
    kb = np.array([4, 1, 4096, 1, 1, 4], dtype=np.int64)
    d = int(off[-1])
    p = BlockPair(3, d, off, kb, np.zeros(d, dtype=np.float32))
    for t in range(4):
        p.step(grads(rng, 3, d))
        p.compare(f"step {t}", with_e=t % 2 == 1)
    p.close()


def test_ties_and_zero_blocks():
    """Blocks of equal magnitudes (ties go to the lower coordinate) and a block of zeros (every key equal)."""
    rng = np.random.default_rng(11)
    d = 6 * 5000
    off = np.arange(0, d + 1, 5000, dtype=np.int64)
    kb = np.array([50, 4999, 1, 2500, 77, 5000], dtype=np.int64)
    p = BlockPair(2, d, off, kb, np.zeros(d, dtype=np.float32))
    for t in range(4):
        g = grads(rng, 2, d)
        g[:, 0:5000] = np.where(rng.random((2, 5000)) < 0.5, 1.0, -1.0) * (0.5 if t % 2 else 2.0)
        g[:, 5000:10000] = 0.0
        g[:, 15000:20000] = np.round(g[:, 15000:20000] * 4) / 4
        p.step(g)
        p.compare(f"step {t}", with_e=t == 3)
    p.close()


def test_blocks_that_one_wavefront_selects_from():
    """Blocks of at most 1024 coordinates never meet the histogram kernels: sizes around the round and size limits,
    everything kept, one kept, equal magnitudes, zeros only, non-finite entries, a ragged last block."""
    rng = np.random.default_rng(77)
    sizes = [4, 252, 256, 260, 508, 512, 516, 1020, 1024, 1028, 64, 64, 128, 1000, 4096, 8, 1023]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    kb = np.array([4, 1, 256, 3, 5, 512, 1, 1020, 7, 10, 1, 64, 2, 999, 40, 8, 11], dtype=np.int64)
    n, d = 5, int(off[-1])
    p = BlockPair(n, d, off, kb, (rng.standard_normal(d) * 0.1).astype(np.float32))
    for t in range(6):
        g = grads(rng, n, d)
        g[:, off[10]:off[11]] = np.where(rng.random((n, 64)) < 0.5, 3.0, -3.0)            # 64 equal magnitudes, one kept
        g[:, off[11]:off[12]] = 0.0                                                        # zeros only, all kept
        g[:, off[12]:off[13]] = np.round(g[:, off[12]:off[13]] * 2) / 2                    # many ties
        if t == 2:
            g[0, off[13] + 5] = np.inf; g[1, off[13] + 6] = -np.inf; g[2, off[13] + 7] = np.nan
        p.step(g)
        p.compare(f"step {t}", with_e=(t % 2 == 1) and t < 2)
    p.close()


def test_only_small_blocks():
    """Every block is one wavefront's: the sweep and counting kernels have nothing to do."""
    rng = np.random.default_rng(78)
    n, d = 7, 40 * 300
    off = np.arange(0, d + 1, 300, dtype=np.int64)
    kb = rng.integers(1, 300, size=40).astype(np.int64)
    p = BlockPair(n, d, off, kb, np.zeros(d, dtype=np.float32))
    for t in range(4):
        p.step(grads(rng, n, d))
        p.compare(f"step {t}", with_e=t == 3)
    p.close()


@pytest.mark.parametrize("route", ["dense", "no guess", "small candidate list"])
def test_routes(route):
    rng = np.random.default_rng(3)
    n, d = 3, 120000
    off, kb = make_blocks(d, 9, rng, frac=0.05)
    p = BlockPair(n, d, off, kb, rng.standard_normal(d).astype(np.float32))
    if route == "dense":
        p.gpu.set_option(B.OPT_FORCE_DENSE, 1)
    elif route == "no guess":
        p.gpu.set_option(B.OPT_PREDICT, 0)
    else:
        p.gpu.set_option(B.OPT_CANDIDATE_CAP, 64)
    for t in range(4):
        p.step(grads(rng, n, d) * (1.0 if t != 2 else 1e-3))
        p.compare(f"{route} step {t}", with_e=t == 3)
    p.close()


def test_gradient_scale_that_jumps():
    """The carried-over guess is far off after a jump in scale: the fallback has to give the same lists."""
    rng = np.random.default_rng(8)
    n, d = 2, 90000
    off, kb = make_blocks(d, 4, rng, frac=0.01)
    p = BlockPair(n, d, off, kb, np.zeros(d, dtype=np.float32))
    for t, s in enumerate([1.0, 1.0, 1e4, 1e-6, 1.0, 1.0]):
        p.step(grads(rng, n, d) * np.float32(s))
        p.compare(f"step {t}", with_e=False)
    p.compare("end", with_e=True)
    p.close()


def test_messages_and_the_two_halves():
    rng = np.random.default_rng(21)
    n, d = 4, 150000
    off, kb = make_blocks(d, 11, rng)
    off = np.concatenate([off[:-1], [d, d + 64, d + 576, d + 1600]]).astype(np.int64)   # and three small blocks
    kb = np.concatenate([kb, [1, 5, 100]]).astype(np.int64)
    d = int(off[-1])
    theta0 = rng.standard_normal(d).astype(np.float32) * 0.1
    whole = BlockPair(n, d, off, kb, theta0)
    halves = B.Compams(n, d, torch.from_numpy(theta0), compressor=B.TOPK_BLOCKS, block_offsets=off, block_k=kb)
    k = int(kb.sum())
    assert halves.compams_wire_capacity() == 3 + ((k + 255) // 256 + 3) // 4 + 2 * k
    for t in range(3):
        g = grads(rng, n, d)
        whole.step(g)
        whole.compare(f"step {t}", with_e=False)
        halves.compams_worker_step(whole.device_g(g))
        msgs, words = halves.compams_encode()
        torch.cuda.synchronize()
        want_idx, want_val = whole.cpu.get("idx"), whole.cpu.get("val")
        for i in range(n):
            ref = O.wire_encode_topk(want_idx[i], want_val[i])
            assert int(words[i]) == ref.size
            assert np.array_equal(msgs[i, : ref.size].cpu().numpy().view(np.uint32), ref), f"step {t}: message {i}"
        idx, val, status = halves.compams_decode(msgs, words)
        assert not status.cpu().numpy().any()
        assert np.array_equal(idx.cpu().numpy(), want_idx)
        assert np.array_equal(val.cpu().numpy().view(np.uint32), want_val.view(np.uint32))
        status = halves.compams_server_step(msgs, words, 1e-3)
        assert not status.cpu().numpy().any()
        for name in ("theta", "m", "v", "vhat"):
            got = halves.compams_state(name).cpu().numpy()
            assert np.array_equal(got.view(np.uint32), whole.cpu.get(name).view(np.uint32)), f"step {t}: {name} by halves"
    got = np.ascontiguousarray(halves.compams_state("e").cpu().numpy())
    assert np.array_equal(got.view(np.uint32), whole.cpu.get("e").view(np.uint32))
    whole.close(); halves.close()


def test_fused_equals_composition_and_is_deterministic():
    rng = np.random.default_rng(2)
    n, d = 3, 64000
    off, kb = make_blocks(d, 13, rng)
    theta0 = rng.standard_normal(d).astype(np.float32)
    gs = [grads(rng, n, d) for _ in range(4)]
    outs = []
    for make in (lambda: B.Compams(n, d, torch.from_numpy(theta0), compressor=B.TOPK_BLOCKS, block_offsets=off, block_k=kb),
                 lambda: B.Compams(n, d, torch.from_numpy(theta0), compressor=B.TOPK_BLOCKS, block_offsets=off, block_k=kb),
                 lambda: CompamsBlockTopk(n, d, torch.from_numpy(theta0), off, kb)):
        c = make()
        for g in gs:
            gp = torch.zeros((n, c.ld), dtype=torch.float32); gp[:, :d] = torch.from_numpy(g)
            c.compams_step(gp.cuda(), 1e-3)
        torch.cuda.synchronize()
        outs.append([np.ascontiguousarray(c.compams_state(s).cpu().numpy()) for s in
                     ("theta", "m", "v", "vhat", "e", "last_idx", "last_val")])
        c.close()
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_invalid_block_configurations_are_refused():
    t = torch.zeros(100)
    with pytest.raises(B.CompamsError):
        B.Compams(2, 100, t, compressor=B.TOPK_BLOCKS, block_offsets=[0, 50, 100], block_k=[1, 1])   # 50 % 4 != 0
    with pytest.raises(B.CompamsError):
        B.Compams(2, 100, t, compressor=B.TOPK_BLOCKS, block_offsets=[0, 48, 100], block_k=[49, 1])  # k_b > d_b
    with pytest.raises(B.CompamsError):
        B.Compams(2, 100, t, compressor=B.TOPK_BLOCKS, block_offsets=[0, 48, 100], block_k=[0, 1])   # k_b < 1
    with pytest.raises(B.CompamsError):
        B.Compams(2, 100, t, compressor=B.TOPK_BLOCKS, block_offsets=[0, 48, 96], block_k=[1, 1])    # not up to d
    with pytest.raises(B.CompamsError):
        B.Compams(2, 100, t, compressor=B.TOPK_BLOCKS, block_offsets=[0, 48, 100])                   # no counts
