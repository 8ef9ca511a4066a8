"""One context stepped from two streams in turn, with no host synchronisation in between: a call on another
stream than the previous one must wait, on the device, for what the context has enqueued so far (each step reads
the state, the residuals, the pending error line and the carried-over threshold guess of the one before).  Every
step is checked against the oracle afterwards.  Also the host-side answer to "is an error line pending"."""
import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

from parity import bits_equal

pytestmark = pytest.mark.gpu

N, D = 4, (1 << 20) + 4 * 123   # large enough that a step is still running when the next one is enqueued


def case_kwargs(case, rng):
    if case == "topk":
        return dict(compressor=B.TOPK, k=D // 100), {}
    if case == "identity":
        return dict(compressor=B.NONE), {}
    cuts = np.sort(rng.choice(np.arange(1, D // 4), size=11, replace=False)) * 4
    off = np.concatenate([[0], cuts, [D]]).astype(np.int64)
    if case == "blocksign":
        return dict(compressor=B.BLOCKSIGN, block_offsets=off), {}
    kb = np.maximum(1, (off[1:] - off[:-1]) // 100)
    return dict(compressor=B.TOPK_BLOCKS, block_offsets=off, block_k=kb), dict(block_k=kb)


@pytest.mark.parametrize("case", ["topk", "topk_blocks", "blocksign", "identity"])
def test_steps_alternating_between_two_streams(case):
    rng = np.random.default_rng(11)
    kw, okw = case_kwargs(case, rng)
    theta0 = (rng.standard_normal(D) * 0.1).astype(np.float32)
    gpu = B.Compams(N, D, torch.from_numpy(theta0), **kw)
    cpu = O.Oracle(N, D, theta0, compressor=kw["compressor"], k=kw.get("k", 0), block_offsets=kw.get("block_offsets"),
                   **okw)
    steps = 6
    host, dev = [], []
    for t in range(steps):
        g = (rng.standard_normal((N, D)) * 10.0 ** rng.uniform(-3, 0, (1, D))).astype(np.float32)
        gp = torch.zeros((N, gpu.ld), dtype=torch.float32)
        gp[:, :D] = torch.from_numpy(g)
        host.append(g)
        dev.append(gp.to(gpu.device))
    torch.cuda.synchronize()            # the inputs are the caller's to order: all resident before the first step
    streams = [torch.cuda.Stream(device=gpu.device), torch.cuda.Stream(device=gpu.device)]
    snaps = []
    for t in range(steps):
        with torch.cuda.stream(streams[t % 2]):
            gpu.compams_step(dev[t], 1e-3)
            # a copy on the step's own stream, ordered after it: what the parameters were after step t
            snaps.append(gpu.compams_state("theta").clone())
    has_e = kw["compressor"] != B.NONE
    assert gpu.compams_state("pending") == has_e
    torch.cuda.synchronize()
    for t in range(steps):
        cpu.step(host[t], 1e-3)
        assert bits_equal(snaps[t].cpu().numpy(), cpu.get("theta")), f"{case}: theta after step {t}"
    for name in ("m", "v", "vhat") + (("e",) if has_e else ()):
        got = np.ascontiguousarray(gpu.compams_state(name).cpu().numpy())
        assert bits_equal(got, cpu.get(name)), f"{case}: {name} after {steps} steps"
    assert gpu.compams_state("pending") is False      # asking for e applied it
    if kw["compressor"] == B.TOPK:
        assert np.array_equal(gpu.compams_state("last_idx").cpu().numpy(), cpu.get("idx"))
    gpu.close(); cpu.close()


def test_messages_packed_on_another_stream_than_the_step():
    rng = np.random.default_rng(12)
    theta0 = (rng.standard_normal(D) * 0.1).astype(np.float32)
    k = D // 100
    gpu = B.Compams(N, D, torch.from_numpy(theta0), compressor=B.TOPK, k=k)
    cpu = O.Oracle(N, D, theta0, compressor=O.TOPK, k=k)
    g = rng.standard_normal((N, D)).astype(np.float32)
    gp = torch.zeros((N, gpu.ld), dtype=torch.float32)
    gp[:, :D] = torch.from_numpy(g)
    gd = gp.to(gpu.device)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(device=gpu.device), torch.cuda.Stream(device=gpu.device)
    with torch.cuda.stream(s1):
        gpu.compams_step(gd, 1e-3)
    with torch.cuda.stream(s2):
        msgs, words = gpu.compams_encode()      # the library orders s2 behind the step on s1
    torch.cuda.synchronize()
    cpu.step(g, 1e-3)
    m, wn = msgs.cpu().numpy().view(np.uint32), words.cpu().numpy()
    for i in range(N):
        want = O.wire_encode_topk(cpu.get("idx")[i], cpu.get("val")[i])
        assert wn[i] == want.size and np.array_equal(m[i, : wn[i]], want), f"message of worker {i}"
    gpu.close(); cpu.close()
