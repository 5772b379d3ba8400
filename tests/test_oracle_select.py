"""Pins for the select half of the CPU oracle (Alg. 1, SELECT_GRAD).

None of these re-type the oracle's own formula: they use hand-worked fixtures,
brute-force sorts, library routines (numpy stable argsort, torch.topk) and
invariances that the definition implies.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def key(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def check_valid_selection(g, k, idx, val):
    """What any correct AdaComp selection must satisfy, whatever the tie rule."""
    g = np.asarray(g, dtype=np.float32)
    assert idx.dtype == np.uint32 and val.dtype == np.float32
    assert idx.size == k and val.size == k
    if k == 0:
        return
    assert np.all(np.diff(idx.astype(np.int64)) > 0), "indices strictly ascending"
    assert int(idx[-1]) < g.size
    assert np.array_equal(val.view(np.uint32), g[idx].view(np.uint32)), "values copied bit for bit"
    mask = np.zeros(g.size, dtype=bool)
    mask[idx] = True
    keys = key(g)
    if k < g.size:
        assert keys[mask].min() >= keys[~mask].max(), "dominance"
        # brute force: the k-th largest magnitude of the sorted tensor is the smallest selected one
        assert np.sort(keys)[::-1][k - 1] == keys[mask].min()


def check_tie_rule(g, idx):
    """Lower index first among entries whose magnitude equals the threshold."""
    keys = key(g)
    mask = np.zeros(keys.size, dtype=bool)
    mask[idx] = True
    if mask.all() or not mask.any():
        return
    T = keys[mask].min()
    eq = np.flatnonzero(keys == T)
    sel_eq, unsel_eq = eq[mask[eq]], eq[~mask[eq]]
    if sel_eq.size and unsel_eq.size:
        assert sel_eq.max() < unsel_eq.min()


def test_count_table():
    with open(os.path.join(GOLD, "count_table.json")) as f:
        rows = json.load(f)["rows"]
    for n, c, k in rows:
        assert oracle.count(n, c) == k, (n, c)


def test_count_one_over_n_and_bounds():
    rng = np.random.default_rng(7)
    ns = list(range(1, 3000)) + rng.integers(1, 5_000_000, 3000).tolist()
    for n in ns:
        assert oracle.count(n, 1.0 / n) == 1, n
        assert oracle.count(n, 1.0) == n
        assert oracle.count(n, 0.0) == 0
    for n in rng.integers(1, 1 << 32, 2000).tolist():
        for c in (1e-9, 1e-4, 0.013, 0.5, 0.999999):
            k = oracle.count(n, c)
            assert 1 <= k <= n
            # sent fraction is at least c (up to the 2^-40 guard) and less than one entry above it
            assert k >= c * n * (1 - 2.0 ** -39) and (k - 1 < c * n or k == 1)


def test_hand_example():
    with open(os.path.join(GOLD, "select_hand_example.json")) as f:
        ex = json.load(f)
    g = np.array([float(s) for s in ex["g"]], dtype=np.float32)
    assert g[5] != 0 and key(g)[5] < 0x00800000, "1e-40 must stay an fp32 denormal"
    assert np.signbit(g[6]) and g[6] == 0
    for ks, want in ex["selected_idx_by_k"].items():
        idx, val = oracle.select_layer(g, int(ks))
        assert idx.tolist() == want, ks
        assert np.array_equal(val.view(np.uint32), g[want].view(np.uint32))


@pytest.mark.parametrize("seed", range(12))
def test_dominance_ties_and_stable_argsort(seed):
    """Random tiny tensors with many repeated magnitudes: brute-force checks, and
    the exact index set against numpy's stable argsort on the negated key."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 400))
    pool = rng.standard_normal(max(2, n // 8)).astype(np.float32)
    g = pool[rng.integers(0, pool.size, n)] * rng.choice([-1.0, 1.0], n).astype(np.float32)
    g[rng.random(n) < 0.2] = 0.0
    g[rng.random(n) < 0.1] = -0.0
    for k in sorted({0, 1, n // 7, n // 2, n - 1, n} & set(range(n + 1))):
        idx, val = oracle.select_layer(g, k)
        check_valid_selection(g, k, idx, val)
        check_tie_rule(g, idx)
        order = np.argsort(-(key(g).astype(np.int64)), kind="stable")
        assert np.array_equal(np.sort(order[:k]).astype(np.uint32), idx)


@pytest.mark.parametrize("cfg", ["cnn_select", "adversarial"])
def test_topk_library_crosscheck(cfg):
    """The multiset of selected magnitudes equals torch.topk(|g|, k) on the workload's
    own distributions (indices may differ among ties; values may not)."""
    sizes = workloads.sizes_of(cfg)
    for layer, n in enumerate(sizes):
        if n > 600_000:
            continue
        g = workloads.gradient_layer(cfg, 0, layer, n)
        for rate in (0.01, 0.3):
            k = oracle.count(n, rate)
            idx, val = oracle.select_layer(g.numpy(), k)
            check_valid_selection(g.numpy(), k, idx, val)
            check_tie_rule(g.numpy(), idx)
            top = torch.topk(g.abs(), k).values.numpy()
            assert np.array_equal(np.sort(np.abs(val)), np.sort(top))


def test_keep_all_is_identity():
    g = workloads.gradient_layer("adversarial", 0, 0, 5003).numpy()
    idx, val = oracle.select_layer(g, g.size)
    assert np.array_equal(idx, np.arange(g.size, dtype=np.uint32))
    assert np.array_equal(val.view(np.uint32), g.view(np.uint32))


def test_invariance_negation_and_power_of_two_scaling():
    g = workloads.gradient_layer("cnn_select", 0, 2).numpy()
    k = oracle.count(g.size, 0.01)
    idx, val = oracle.select_layer(g, k)
    idx_n, val_n = oracle.select_layer(-g, k)
    assert np.array_equal(idx, idx_n) and np.array_equal(val_n, -val)
    idx_s, val_s = oracle.select_layer(g * np.float32(8.0), k)
    assert np.array_equal(idx, idx_s) and np.array_equal(val_s, val * np.float32(8.0))


def test_special_values_order():
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    g = np.array([1.0, -inf, 3e38, nan, 0.0, inf, 1e-45], dtype=np.float32)
    # magnitude order by bit pattern: nan > inf (index 1 before 5) > 3e38 > 1 > 1e-45 > 0
    want_order = [3, 1, 5, 2, 0, 6, 4]
    for k in range(g.size + 1):
        idx, _ = oracle.select_layer(g, k)
        assert idx.tolist() == sorted(want_order[:k])


def test_multi_layer_layout_and_per_layer_independence():
    """Every tensor is its own selection domain (Sec. 4 'Selection method'): the
    joint call equals per-tensor calls laid end to end; a bias vector of 10 entries
    still sends one entry at 1%."""
    layers = [g.numpy() for g in workloads.gradient("cnn_select", 0)]
    small = [layers[i] for i in (0, 1, 3, 5, 6, 7)]
    off, idx, val = oracle.select(small, 0.01)
    assert off.tolist() == np.cumsum([0] + [oracle.count(g.size, 0.01) for g in small]).tolist()
    assert int(off[-1] - off[-2]) == 1
    for l, g in enumerate(small):
        i1, v1 = oracle.select_layer(g, int(off[l + 1] - off[l]))
        assert np.array_equal(idx[off[l]:off[l + 1]], i1)
        assert np.array_equal(val[off[l]:off[l + 1]].view(np.uint32), v1.view(np.uint32))
    # whole-model selection (the competitors' rule) picks a different set
    flat = np.concatenate(small)
    fi, _ = oracle.select_layer(flat, int(off[-1]))
    per_layer_global = np.concatenate([idx[off[l]:off[l + 1]].astype(np.int64) + s
                                       for l, s in enumerate(np.cumsum([0] + [g.size for g in small[:-1]]))])
    assert not np.array_equal(fi.astype(np.int64), per_layer_global)


def test_k_override_and_errors():
    g = [np.arange(5, dtype=np.float32), np.arange(3, dtype=np.float32)]
    off, idx, val = oracle.select(g, 0.5, k_override=[2, 0])
    assert off.tolist() == [0, 2, 2] and idx.tolist() == [3, 4]
    with pytest.raises(RuntimeError):
        oracle.select(g, 0.5, k_override=[6, 0])
