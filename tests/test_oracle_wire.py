"""Pins of the oracle's wire codec (CPU only).

The format is the library's own (stated in include/compams.h); the paper fixes only the accounting of the
experiments section: 32 bits per transmitted float, top-k at 1 % about 100 times and block-sign about 30 times
fewer bits than the full gradient.  The codec is pinned against a word sequence worked out by hand, against an
independent formulation of the gap stream as one big integer, by round trips and by the paper's ratios.
"""
import numpy as np
import pytest

from oracle import compams_oracle as O
from paper_2205_05632_amd import workloads as W


def f32_words(values):
    return np.asarray(values, dtype=np.float32).view(np.uint32).tolist()


def test_topk_message_worked_out_by_hand():
    # coordinates 5, 6, 100, 101: gaps 5, 0, 93, 0; one tile; its widest gap 93 needs 7 bits (width word 0x07);
    # stream = 5 + 0 * 2^7 + 93 * 2^14 + 0 * 2^21 = 1 523 717 = 0x174005, one word
    msg = O.wire_encode_topk([5, 6, 100, 101], [1.0, 2.0, 3.0, 4.0])
    assert msg.tolist() == [1, 4, 256, 0x07, 0x174005] + f32_words([1.0, 2.0, 3.0, 4.0])


def test_topk_message_of_two_tiles_worked_out_by_hand():
    # 258 coordinates: 0 .. 255 (a full tile of zero gaps: width 1, 256 bits = 8 zero words), then 1255 and 1258
    # (gaps 999 and 2: width 10; stream word 999 + 2 * 2^10 = 3047).  Width word: 0x0a01.
    idx = list(range(256)) + [1255, 1258]
    msg = O.wire_encode_topk(idx, np.ones(258))
    assert msg[:4].tolist() == [1, 258, 256, 0x0A01]
    assert msg[4:13].tolist() == [0] * 8 + [3047]
    assert msg.size == 4 + 9 + 258


def test_topk_message_of_consecutive_coordinates_uses_one_bit_per_gap():
    # gaps are all zero: width 1 (never 0), stream of ceil(40 / 32) = 2 zero words
    msg = O.wire_encode_topk(np.arange(40), np.ones(40))
    assert msg[:6].tolist() == [1, 40, 256, 1, 0, 0] and msg.size == 3 + 1 + 2 + 40


def test_topk_gap_stream_is_the_little_endian_big_integer_of_each_tile():
    rng = np.random.default_rng(5)
    for d, k in [(1000, 37), (1 << 20, 5000), (70000, 70000), (50, 1), ((1 << 31) - 1, 300), (1 << 22, 1025)]:
        idx = np.sort(rng.choice(d, size=k, replace=False)) if d <= (1 << 22) else \
            np.unique(rng.integers(0, d, size=2 * k))[:k]
        if k == 300:
            idx[-1] = d - 1  # the largest coordinate the library admits
        val = rng.standard_normal(k).astype(np.float32)
        msg = O.wire_encode_topk(idx, val)
        gaps = [int(idx[0])] + [int(idx[q]) - int(idx[q - 1]) - 1 for q in range(1, k)]
        tiles = [gaps[i:i + 256] for i in range(0, k, 256)]
        width_words = [0] * ((len(tiles) + 3) // 4)
        stream = []
        for t, tile in enumerate(tiles):
            b = max(1, max(tile).bit_length())
            width_words[t // 4] |= b << (8 * (t % 4))
            big = 0
            for i, gap in enumerate(tile):
                big |= gap << (i * b)
            stream += [(big >> (32 * w)) & 0xFFFFFFFF for w in range((len(tile) * b + 31) // 32)]
        want = [1, k, 256] + width_words + stream + f32_words(val)
        assert msg.tolist() == want
        i2, v2 = O.wire_decode_topk(msg, k, d)
        assert np.array_equal(i2, idx) and np.array_equal(v2.view(np.uint32), val.view(np.uint32))


def test_topk_decode_rejects_what_is_not_a_message():
    msg = O.wire_encode_topk([5, 6, 100, 101], [1.0, 2.0, 3.0, 4.0])
    O.wire_decode_topk(msg, 4, 102)
    with pytest.raises(ValueError):
        O.wire_decode_topk(msg, 4, 101)       # coordinate 101 does not exist for d = 101
    with pytest.raises(ValueError):
        O.wire_decode_topk(msg, 5, 102)       # another k
    with pytest.raises(ValueError):
        O.wire_decode_topk(msg[:-1], 4, 102)  # truncated
    bad = msg.copy(); bad[0] = 2
    with pytest.raises(ValueError):
        O.wire_decode_topk(bad, 4, 102)
    bad = msg.copy(); bad[2] = 128      # another tile size
    with pytest.raises(ValueError):
        O.wire_decode_topk(bad, 4, 102)
    bad = msg.copy(); bad[3] = 0        # a width of zero bits
    with pytest.raises(ValueError):
        O.wire_decode_topk(bad, 4, 102)
    bad = msg.copy(); bad[3] = 32       # a width no coordinate gap can need
    with pytest.raises(ValueError):
        O.wire_decode_topk(bad, 4, 102)


def test_blocksign_message_by_hand_and_round_trip():
    mu = np.array([0.5, 2.0], dtype=np.float32)
    bits = np.array([0x80000001, 0x3], dtype=np.uint32)   # d = 34: coordinates 0, 31, 32, 33 negative
    msg = O.wire_encode_blocksign(34, bits, mu)
    assert msg.tolist() == [2, 34, 2, 0x80000001, 0x3] + f32_words(mu)
    b2, m2 = O.wire_decode_blocksign(msg, 34, 2)
    assert np.array_equal(b2, bits) and np.array_equal(m2, mu)
    with pytest.raises(ValueError):
        O.wire_decode_blocksign(msg, 35, 2)
    with pytest.raises(ValueError):
        O.wire_decode_blocksign(msg[:-1], 34, 2)


def test_messages_of_a_step_round_trip_and_match_the_papers_accounting():
    """Encode what the oracle's workers send in a step; decode; the server's inputs are recovered bit for bit.
    Sizes: 32 bits per float (experiments section).  Top-k at 1 %: the values alone are 100 times fewer bits
    than the full gradient, the whole message (values, gap stream, header) stays between the two obvious
    bounds; block-sign with layer blocks is just under 32 times ("about 30")."""
    w = W.get("tiny")
    rng = np.random.default_rng(3)
    o = O.Oracle(w.n, w.d, np.zeros(w.d, np.float32), compressor=O.TOPK, k=w.k)
    o.step(rng.standard_normal((w.n, w.d)).astype(np.float32), 1e-3)
    idx, val = o.get("idx"), o.get("val")
    for i in range(w.n):
        msg = O.wire_encode_topk(idx[i], val[i])
        i2, v2 = O.wire_decode_topk(msg, w.k, w.d)
        assert np.array_equal(i2, idx[i]) and np.array_equal(v2.view(np.uint32), val[i].view(np.uint32))
        assert 32 * w.k < 32 * msg.size < 64 * w.k + 128
    o.close()
    assert 32 * w.d / (32 * w.k) == pytest.approx(100.0, rel=0.01)

    r18 = W.get("r18_blocksign")
    M = len(r18.block_offsets()) - 1
    bits_msg = 32 * (3 + (r18.d + 31) // 32 + M)
    assert 30.0 < 32 * r18.d / bits_msg < 32.0

    tb = W.get("tiny_blocksign")
    o = O.Oracle(tb.n, tb.d, np.zeros(tb.d, np.float32), compressor=O.BLOCKSIGN, block_offsets=tb.block_offsets())
    o.step(rng.standard_normal((tb.n, tb.d)).astype(np.float32), 1e-3)
    bits, mu = o.get("bits"), o.get("mu")
    for i in range(tb.n):
        msg = O.wire_encode_blocksign(tb.d, bits[i], mu[i])
        b2, m2 = O.wire_decode_blocksign(msg, tb.d, mu.shape[1])
        assert np.array_equal(b2, bits[i]) and np.array_equal(m2.view(np.uint32), mu[i].view(np.uint32))
    o.close()
