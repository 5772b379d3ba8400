"""Pins of the oracle's wire format (block-wise delta coding of the indices; the paper leaves the
encoding open, so the definition in include/adacomp.h is the authority): a hand-worked stream, an
independent big-integer formulation, closed-form sizes, round trips, and rejection of bad streams."""
import json
import os

import numpy as np
import pytest

import oracle
import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MAGIC = 0x31434441


def bigint_pack(off, idx, val):
    """The same definition through Python integers: the deltas of a block form one big number,
    sum d_i << ((i-1) * w), which is then cut into 32-bit words."""
    off = [int(x) for x in off]
    L = len(off) - 1
    firsts, widths, streams = [], [], []
    for l in range(L):
        for e0 in range(off[l], off[l + 1], 64):
            blk = [int(x) for x in idx[e0:min(e0 + 64, off[l + 1])]]
            d = [b - a - 1 for a, b in zip(blk, blk[1:])]
            w = max(d).bit_length() if d else 0
            big = sum(x << (i * w) for i, x in enumerate(d))
            nwords = (len(d) * w + 31) // 32
            firsts.append(blk[0])
            widths.append(w)
            streams += [(big >> (32 * j)) & 0xFFFFFFFF for j in range(nwords)]
    wbytes = bytes(widths) + b"\0" * (-len(widths) % 4)
    words = [MAGIC, L, off[L] & 0xFFFFFFFF, off[L] >> 32] + [off[l + 1] - off[l] for l in range(L)] + firsts
    words += list(np.frombuffer(wbytes, dtype="<u4")) + streams
    words += list(np.asarray(val, dtype=np.float32).view(np.uint32))
    return np.array(words, dtype=np.uint32)


def random_update(rng, sizes, counts):
    off, idx = [0], []
    for n, k in zip(sizes, counts):
        idx.append(np.sort(rng.choice(n, size=k, replace=False)).astype(np.uint32) if k else np.empty(0, np.uint32))
        off.append(off[-1] + k)
    idx = np.concatenate(idx) if idx else np.empty(0, np.uint32)
    return np.array(off, dtype=np.uint64), idx, rng.standard_normal(idx.size).astype(np.float32)


def test_hand_worked_stream():
    with open(os.path.join(GOLD, "wire_hand_example.json")) as f:
        g = json.load(f)
    want = np.array([int(x, 16) for x in g["words_hex"]], dtype=np.uint32)
    got = oracle.wire_pack(g["layer_off"], g["idx"], np.array(g["val"], dtype=np.float32))
    assert got.tolist() == want.tolist()
    off, idx, val = oracle.wire_unpack(want, 3)
    assert off.tolist() == g["layer_off"] and idx.tolist() == g["idx"]
    assert val.view(np.uint32).tolist() == np.array(g["val"], dtype=np.float32).view(np.uint32).tolist()


@pytest.mark.parametrize("seed", range(6))
def test_against_bigint_formulation_and_round_trip(seed):
    rng = np.random.default_rng(seed)
    sizes = [1, 64, 65, 5000, 1 << 20, 0xFFFFFFFF, 300]
    counts = [1, 64, 65, int(rng.integers(0, 700)), int(rng.integers(1, 3000)), 130, 0]
    off, idx, val = random_update(rng, sizes, counts)
    words = oracle.wire_pack(off, idx, val)
    assert words.tolist() == bigint_pack(off, idx, val).tolist()
    assert words.size <= oracle.wire_bound(off)
    o2, i2, v2 = oracle.wire_unpack(words, len(sizes))
    assert o2.tolist() == off.tolist() and np.array_equal(i2, idx)
    assert np.array_equal(v2.view(np.uint32), val.view(np.uint32))


def test_extreme_widths():
    """Consecutive indices need no delta bits; the two ends of the index range need all 32."""
    off = np.array([0, 200, 202], dtype=np.uint64)
    idx = np.concatenate([np.arange(1000, 1200), [0, 0xFFFFFFFF]]).astype(np.uint32)
    val = np.ones(202, dtype=np.float32)
    words = oracle.wire_pack(off, idx, val)
    # blocks: 64 + 64 + 64 + 8 of tensor 0 (width 0, no delta words), 1 of tensor 1 (width 32, one word)
    nblocks = 5
    assert words.size == 4 + 2 + nblocks + 2 + 1 + 202
    assert words[4 + 2 + nblocks:4 + 2 + nblocks + 2].tolist() == [0, 32]          # width bytes 0,0,0,0 | 32,0,0,0
    assert words[4 + 2 + nblocks + 2] == 0xFFFFFFFE                                # the one delta: 2^32 - 1 - 0 - 1
    assert words.tolist() == bigint_pack(off, idx, val).tolist()
    o2, i2, _ = oracle.wire_unpack(words, 2)
    assert np.array_equal(i2, idx)


@pytest.mark.parametrize("step", [1, 2, 3, 200, 1024, 1025])
def test_size_of_an_arithmetic_progression(step):
    """idx = a + i * step: every delta is step - 1, so every full block takes ceil(63 * w / 32) words
    with w = bit length of step - 1."""
    k = 64 * 7 + 10
    idx = (5 + step * np.arange(k)).astype(np.uint32)
    off = np.array([0, k], dtype=np.uint64)
    words = oracle.wire_pack(off, idx, np.zeros(k, dtype=np.float32))
    w = (step - 1).bit_length()
    want = 4 + 1 + 8 + 2 + 7 * ((63 * w + 31) // 32) + (9 * w + 31) // 32 + k
    assert words.size == want


def test_selected_updates_round_trip_and_beat_raw_pairs():
    """Updates as SELECT_GRAD makes them (1% of a CNN-shaped gradient): exact round trip, and fewer
    bytes than 8 per entry but more than the 4 per entry of the paper's traffic model (Sec. 3.2)."""
    g = [x.numpy() for x in workloads.gradient("cnn_select", 0)]
    off, idx, val = oracle.select(g, 0.01)
    words = oracle.wire_pack(off, idx, val)
    o2, i2, v2 = oracle.wire_unpack(words, len(g))
    assert o2.tolist() == off.tolist() and np.array_equal(i2, idx) and np.array_equal(v2.view(np.uint32), val.view(np.uint32))
    per_entry = 4.0 * words.size / idx.size
    assert 4.0 < per_entry < 6.0


def test_bad_streams_are_rejected():
    rng = np.random.default_rng(9)
    off, idx, val = random_update(rng, [1000, 50], [100, 10])
    good = oracle.wire_pack(off, idx, val)
    oracle.wire_unpack(good, 2)
    bad = good.copy(); bad[0] ^= 1
    with pytest.raises(ValueError): oracle.wire_unpack(bad, 2)                 # magic
    with pytest.raises(ValueError): oracle.wire_unpack(good, 3)                # tensor count
    with pytest.raises(ValueError): oracle.wire_unpack(good[:-1], 2)           # truncated
    with pytest.raises(ValueError): oracle.wire_unpack(np.append(good, 0), 2)  # trailing word
    bad = good.copy(); bad[2] += 1
    with pytest.raises(ValueError): oracle.wire_unpack(bad, 2)                 # total != sum of counts
    bad = good.copy(); bad[4 + 2 + 3] = 33                                     # first width byte
    with pytest.raises(ValueError): oracle.wire_unpack(bad, 2)
    with pytest.raises(ValueError): oracle.wire_unpack(good, 2, cap=50)        # output too small
    with pytest.raises(ValueError): oracle.wire_pack([0, 2], [5, 5], [1.0, 1.0])   # not strictly ascending
