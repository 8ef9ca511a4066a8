"""A step recorded into a HIP graph and replayed: compams_step only enqueues kernel launches on the caller's
stream (no allocation, no synchronisation, no memset node), so a steady-state step can be captured once and
replayed with new gradients copied into the same buffer.  Every replay is checked against the oracle, with
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

pytestmark = pytest.mark.gpu


def offsets_for(d, m, rng):
    cuts = np.sort(rng.choice(np.arange(1, d // 4), size=m - 1, replace=False)) * 4
    return np.concatenate([[0], cuts, [d]]).astype(np.int64)


CASES = {
    "topk": dict(compressor=B.TOPK, k=700),
    "topk_blocks": dict(compressor=B.TOPK_BLOCKS),
    "blocksign_layers": dict(compressor=B.BLOCKSIGN),
    "blocksign_4096": dict(compressor=B.BLOCKSIGN),
    "identity": dict(compressor=B.NONE),
}


@pytest.mark.parametrize("case", list(CASES))
def test_replayed_steps_match_the_oracle(case):
    rng = np.random.default_rng(len(case))
    n, d = 3, 5 * 4096 + 123 * 4
    kw = dict(CASES[case])
    okw = {}
    if case == "topk_blocks":
        off = offsets_for(d, 6, rng)
        kb = np.maximum(1, (off[1:] - off[:-1]) // 50)
        kw.update(block_offsets=off, block_k=kb)
        okw.update(block_k=kb)
    elif case == "blocksign_layers":
        kw.update(block_offsets=offsets_for(d, 6, rng))
    elif case == "blocksign_4096":
        kw.update(block_offsets=np.concatenate([np.arange(0, d, 4096), [d]]).astype(np.int64))
    theta0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    gpu = B.Compams(n, d, torch.from_numpy(theta0), **kw)
    cpu = O.Oracle(n, d, theta0, compressor=kw["compressor"], k=kw.get("k", 0), block_offsets=kw.get("block_offsets"), **okw)
    gbuf = torch.zeros((n, gpu.ld), dtype=torch.float32, device=gpu.device)

    def new_g():
        g = (rng.standard_normal((n, d)) * 10.0 ** rng.uniform(-3, 0, (1, d))).astype(np.float32)
        gp = torch.zeros((n, gpu.ld), dtype=torch.float32)
        gp[:, :d] = torch.from_numpy(g)
        return g, gp

    def check(label, with_e=False):
        torch.cuda.synchronize()
        for name in ("theta", "m", "v", "vhat") + (("e",) if with_e and kw["compressor"] != B.NONE else ()):
            got = np.ascontiguousarray(gpu.compams_state(name).cpu().numpy())
            assert np.array_equal(got.view(np.uint32), cpu.get(name).view(np.uint32)), f"{label}: {name}"

    for t in range(2):                      # eager: the first step differs from the later ones
        g, gp = new_g()
        gbuf.copy_(gp)
        gpu.compams_step(gbuf, 1e-3)
        cpu.step(g, 1e-3)
        check(f"eager step {t}")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):           # records the launches; nothing runs
        gpu.compams_step(gbuf, 1e-3)
    for t in range(5):
        g, gp = new_g()
        gbuf.copy_(gp)
        graph.replay()
        cpu.step(g, 1e-3)
        check(f"replay {t}")
        junk = torch.randn(1 << 16, device=gpu.device).sum().item()   # unrelated eager work between replays
        assert np.isfinite(junk)
    check("after the replays", with_e=True)  # applies what the last replay left pending
    del graph
    gpu.close(); cpu.close()
