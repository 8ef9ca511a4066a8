"""GPU parity of the wire codec: compams_encode / compams_decode, through the C ABI, against the oracle's codec.

Bar: every word of every message identical; decoded coordinates, values, sign words and scales identical."""
import numpy as np
import pytest
import torch

from oracle import compams_oracle as O
from paper_2205_05632_amd import binding as B

from parity import Pair

pytestmark = pytest.mark.gpu


def check_topk_messages(p, label):
    """p: a Pair that has taken at least one step."""
    msgs, words = p.gpu.compams_encode()
    torch.cuda.synchronize()
    m = msgs.cpu().numpy().view(np.uint32)
    wn = words.cpu().numpy()
    idx, val = p.cpu.get("idx"), p.cpu.get("val")
    for i in range(p.n):
        want = O.wire_encode_topk(idx[i], val[i])
        assert wn[i] == want.size, f"{label}: worker {i} message length {wn[i]} != {want.size}"
        assert np.array_equal(m[i, : wn[i]], want), f"{label}: worker {i} message differs"
    a, b, status = p.gpu.compams_decode(msgs, words)
    torch.cuda.synchronize()
    assert not status.cpu().numpy().any(), f"{label}: status {status.cpu().numpy()}"
    assert np.array_equal(a.cpu().numpy(), idx), f"{label}: decoded coordinates"
    assert np.array_equal(b.cpu().numpy().view(np.uint32), val.view(np.uint32)), f"{label}: decoded values"
    return m, wn


def check_blocksign_messages(p, label):
    msgs, words = p.gpu.compams_encode()
    torch.cuda.synchronize()
    m = msgs.cpu().numpy().view(np.uint32)
    wn = words.cpu().numpy()
    bits, mu = p.cpu.get("bits"), p.cpu.get("mu")
    for i in range(p.n):
        want = O.wire_encode_blocksign(p.d, bits[i], mu[i])
        assert wn[i] == want.size and np.array_equal(m[i, : wn[i]], want), f"{label}: worker {i} message differs"
    a, b, status = p.gpu.compams_decode(msgs, words)
    torch.cuda.synchronize()
    assert not status.cpu().numpy().any()
    assert np.array_equal(a.cpu().numpy().view(np.uint32), bits), f"{label}: decoded sign words"
    assert np.array_equal(b.cpu().numpy().view(np.uint32), mu.view(np.uint32)), f"{label}: decoded scales"


@pytest.mark.parametrize("n,d,k", [(4, 65536, 655), (3, 100003, 1000), (2, 8191, 8191), (1, 1, 1), (2, 20000, 1),
                                   (2, 300000, 7), (3, 70001, 35000), (5, 4097, 4096)])
def test_topk_messages_match_the_oracle_word_for_word(n, d, k):
    rng = np.random.default_rng(d + k)
    p = Pair(n, d, rng.standard_normal(d).astype(np.float32) * 0.1, B.TOPK, k=k)
    for t in range(2):
        g = rng.standard_normal((n, d)).astype(np.float32)
        if t == 1:
            g[:, : d // 2] *= 1e-3      # the kept coordinates crowd into one half: small gaps after one large one
        p.step(g, 1e-3, label=f"wire step {t}")
        check_topk_messages(p, f"top-k n={n} d={d} k={k} step {t}")
    p.close()


def test_topk_message_with_the_widest_gaps():
    """k = 2 with the kept coordinates at both ends of a long row: the gap needs more than 20 bits."""
    n, d = 2, 3_000_000
    p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=2)
    g = np.full((n, d), 1e-3, np.float32)
    g[0, 0], g[0, d - 1] = 5.0, -7.0
    g[1, 1], g[1, d - 2] = -3.0, 2.0
    p.step(g, 1e-3, label="wide gaps")
    m, wn = check_topk_messages(p, "wide gaps")
    # gap d - 2 = 2 999 998 needs 22 bits; one tile of 2 gaps: 44 bits = 2 words after the one width word
    assert m[0, 2] == 256 and m[0, 3] == 22 and wn[0] == 3 + 1 + 2 + 2
    p.close()


@pytest.mark.parametrize("n,d,offsets", [(3, 5000, [0, 1, 11, 500, 2548, 5000]), (4, 70000, "fixed4096"),
                                         (2, 9000, "unit"), (2, 33, [0, 33])])
def test_blocksign_messages_match_the_oracle_word_for_word(n, d, offsets):
    rng = np.random.default_rng(d)
    if offsets == "fixed4096":
        off = np.concatenate([np.arange(0, d, 4096), [d]]).astype(np.int64)
    elif offsets == "unit":
        off = np.arange(d + 1, dtype=np.int64)
    else:
        off = np.array(offsets, dtype=np.int64)
    p = Pair(n, d, rng.standard_normal(d).astype(np.float32) * 0.1, B.BLOCKSIGN, block_offsets=off)
    for t in range(2):
        p.step(rng.standard_normal((n, d)).astype(np.float32), 1e-3, label=f"wire step {t}")
        check_blocksign_messages(p, f"block-sign d={d} step {t}")
    p.close()


def test_decode_flags_malformed_messages_and_stays_in_bounds():
    n, d, k = 4, 50000, 500
    rng = np.random.default_rng(9)
    p = Pair(n, d, np.zeros(d, np.float32), B.TOPK, k=k)
    p.step(rng.standard_normal((n, d)).astype(np.float32), 1e-3)
    msgs, words = p.gpu.compams_encode()
    torch.cuda.synchronize()
    bad = msgs.clone()
    bad[0, 0] = 7                       # not a top-k message
    bad[1, 3] = 0x2000                  # first tile: width 0, second tile: width 32
    bad[2, 4:12] = -1                   # gaps of all ones in the first tile: coordinates run past d
    wrong_words = words.clone()
    wrong_words[3] += 1                 # a length that does not fit the header
    a, b, status = p.gpu.compams_decode(bad, wrong_words)
    torch.cuda.synchronize()
    st = status.cpu().numpy()
    assert st[0] & 1 and st[1] & 1 and st[2] == 4 and st[3] == 2, st
    # the untouched message still decodes to what was sent
    assert np.array_equal(a[3].cpu().numpy(), p.cpu.get("idx")[3])
    p.close()


def test_encode_needs_a_step_and_a_compressor():
    d = 1000
    c = B.Compams(2, d, torch.zeros(d), compressor=B.TOPK, k=10)
    with pytest.raises(B.CompamsError):
        c.compams_encode()
    c.close()
    c = B.Compams(2, d, torch.zeros(d), compressor=B.NONE)
    c.compams_step(torch.zeros((2, c.ld), device=c.device), 1e-3)
    assert c.compams_wire_capacity() == 0
    with pytest.raises(B.CompamsError):
        c.compams_encode(stride_words=8)
    c.close()
