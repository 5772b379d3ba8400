"""Pins for the parameter-server half of the CPU oracle (Alg. 2, eqs. 3-5).

Closed forms, the hand-worked chronology fixture, reductions to plain SGD and to
dense staleness-aware ASGD, and a dense brute force on tiny inputs.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")
METHODS = [oracle.HISTORY_LISTS, oracle.HISTORY_BITMAP]


def upd(L_sizes, per_layer):
    """per_layer: list (one per tensor) of dict index -> value."""
    off, idx, val = [0], [], []
    for d in per_layer:
        for k in sorted(d):
            idx.append(k)
            val.append(d[k])
        off.append(len(idx))
    return (np.array(off, dtype=np.uint64), np.array(idx, dtype=np.uint32),
            np.array(val, dtype=np.float32))


@pytest.mark.parametrize("method", METHODS)
def test_chronology_fixture(method):
    with open(os.path.join(GOLD, "apply_chronology.json")) as f:
        ex = json.load(f)
    for mode, want in ((oracle.PER_PARAMETER, ex["theta_per_parameter"]),
                       (oracle.GLOBAL, ex["theta_global_staleness"])):
        theta = [np.zeros(ex["n"], dtype=np.float32)]
        ps = oracle.ParameterServer(theta, method)
        for u, want_sigma in zip(ex["updates"], ex["sigma_per_parameter"]):
            off, idx, val = upd([ex["n"]], [dict(zip(u["idx"], u["val"]))])
            sig = ps.apply(off, idx, val, u["pull_ts"], ex["lr"], mode, want_sigma=True)
            if mode == oracle.PER_PARAMETER:
                assert sig.tolist() == want_sigma
        assert ps.t == 3
        assert theta[0].tolist() == want
    assert ex["theta_per_parameter"] != ex["theta_global_staleness"]


@pytest.mark.parametrize("method", METHODS)
@pytest.mark.parametrize("f64", [False, True])
def test_harmonic_closed_form(method, f64):
    """One parameter, Q updates of value v all pulled at time 0: update q sees
    sigma = q, so theta_Q = theta_0 - lr*v*(1 + sum_{q=1}^{Q-1} 1/q)."""
    Q, lr, v = 40, 0.5, 3.0
    theta = [np.zeros(1, dtype=np.float64 if f64 else np.float32)]
    ps = oracle.ParameterServer(theta, method, f64=f64)
    exact = Fraction(0)
    for q in range(Q):
        off, idx, val = upd([1], [{0: v}])
        sig = ps.apply(off, idx, val, 0, lr, want_sigma=True)
        assert sig.tolist() == [q]
        exact -= Fraction(lr) * Fraction(v) * (Fraction(1, q) if q else 1)
        tol = 1e-14 if f64 else (q + 1) * 2.0 ** -23
        assert abs(float(theta[0][0]) - float(exact)) <= tol * abs(float(exact))
    # the first four values of the sequence with lr = v = 1, by hand: -1, -2, -2.5, -17/6
    theta = [np.zeros(1, dtype=np.float32)]
    ps = oracle.ParameterServer(theta, method)
    seen = []
    for q in range(4):
        ps.apply(*upd([1], [{0: 1.0}]), 0, 1.0)
        seen.append(float(theta[0][0]))
    assert seen[:3] == [-1.0, -2.0, -2.5] and abs(seen[3] + 17 / 6) < 3e-7


@pytest.mark.parametrize("method", METHODS)
def test_window_is_j_to_i_minus_1(method):
    """Three touches of one parameter; the third was pulled at time 1, so only the
    update applied at time 1 counts (sigma = 1), not the one at time 0."""
    theta = [np.zeros(2, dtype=np.float32)]
    ps = oracle.ParameterServer(theta, method)
    ps.apply(*upd([2], [{0: 1.0}]), 0, 1.0)
    ps.apply(*upd([2], [{0: 1.0}]), 1, 1.0)
    s = ps.apply(*upd([2], [{0: 1.0, 1: 1.0}]), 1, 1.0, want_sigma=True)
    assert s.tolist() == [1, 0]
    s = ps.apply(*upd([2], [{0: 4.0}]), 0, 1.0, want_sigma=True)      # pulled at 0, applied at 3
    assert s.tolist() == [3]
    assert theta[0][0] == np.float32(-3.0) - np.float32(np.float32(1.0) / np.float32(3.0)) * np.float32(4.0)
    s = ps.apply(*upd([2], [{0: 1.0}]), 4, 1.0, want_sigma=True)      # fresh pull
    assert s.tolist() == [0]
    with pytest.raises(RuntimeError):
        ps.apply(*upd([2], [{0: 1.0}]), 6, 1.0)                        # pull from the future


def plain_sgd(theta, updates, lr):
    out = [t.copy() for t in theta]
    for off, idx, val in updates:
        for l in range(len(out)):
            for e in range(int(off[l]), int(off[l + 1])):
                out[l][idx[e]] = np.float32(out[l][idx[e]] - np.float32(np.float32(lr) * val[e]))
    return out


def small_queue(seed, sizes, Q, density, zero_frac=0.0):
    rng = np.random.default_rng(seed)
    ups = []
    for _ in range(Q):
        per = []
        for n in sizes:
            k = max(0, int(round(density * n)))
            ids = rng.choice(n, size=min(n, k), replace=False)
            d = {int(i): float(np.float32(rng.standard_normal())) for i in ids}
            for i in list(d):
                if rng.random() < zero_frac:
                    d[i] = 0.0 if rng.random() < 0.5 else -0.0
            per.append(d)
        ups.append(upd(sizes, per))
    return ups


@pytest.mark.parametrize("method", METHODS)
def test_unit_staleness_is_plain_sgd(method):
    sizes = [37, 5, 64]
    theta0 = [np.random.default_rng(l).standard_normal(n).astype(np.float32) for l, n in enumerate(sizes)]
    ups = small_queue(1, sizes, 20, 0.4)
    theta = [t.copy() for t in theta0]
    ps = oracle.ParameterServer(theta, method)
    for q, u in enumerate(ups):
        ps.apply(*u, max(0, q - (q % 2)), 0.01)          # staleness 0 or 1
    want = plain_sgd(theta0, ups, 0.01)
    for a, b in zip(theta, want):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("method", METHODS)
def test_disjoint_supports_are_plain_sgd_whatever_the_pull_times(method):
    n, Q = 64, 8
    theta0 = [np.linspace(-1, 1, n).astype(np.float32)]
    ups = [upd([n], [{q * 8 + r: 0.25 * (r + 1) for r in range(8)}]) for q in range(Q)]
    theta = [theta0[0].copy()]
    ps = oracle.ParameterServer(theta, method)
    for q, u in enumerate(ups):
        sig = ps.apply(*u, 0, 0.1, want_sigma=True)
        assert not sig.any()
    assert np.array_equal(theta[0], plain_sgd(theta0, ups, 0.1)[0])


@pytest.mark.parametrize("method", METHODS)
def test_keep_all_is_dense_staleness_aware_asgd(method):
    """c = 1 with no exact zero in any gradient: every sigma_k equals i - j, which is
    the competitors' rule of Sec. 5.2: theta -= (lr / max(1, i - j)) * g, densely."""
    sizes = [50, 7]
    rng = np.random.default_rng(3)
    Q = 12
    stale = rng.integers(0, 6, Q).tolist()
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    theta = [t.copy() for t in theta0]
    dense = [t.copy() for t in theta0]
    ps = oracle.ParameterServer(theta, method)
    theta_g = [t.copy() for t in theta0]
    ps_g = oracle.ParameterServer(theta_g, method)
    for q in range(Q):
        grads = [(rng.standard_normal(n).astype(np.float32) + np.float32(3.0)) for n in sizes]
        j = max(0, q - stale[q])
        off = np.cumsum([0] + sizes).astype(np.uint64)
        idx = np.concatenate([np.arange(n, dtype=np.uint32) for n in sizes])
        val = np.concatenate(grads)
        sig = ps.apply(off, idx, val, j, 0.05, want_sigma=True)
        assert np.all(sig == q - j)
        ps_g.apply(off, idx, val, j, 0.05, oracle.GLOBAL)
        a = np.float32(0.05) / np.float32(max(1, q - j))
        for l in range(len(sizes)):
            dense[l] = (dense[l] - a * grads[l]).astype(np.float32)
    for a, b, c in zip(theta, dense, theta_g):
        assert np.array_equal(a, b) and np.array_equal(a, c)


@pytest.mark.parametrize("seed", range(6))
def test_dense_brute_force(seed):
    """Tiny random queues: staleness counted on dense update vectors kept for the whole
    trace, both history structures, fp32 and fp64 parameters."""
    rng = np.random.default_rng(100 + seed)
    sizes = [int(rng.integers(1, 40)) for _ in range(3)]
    Q = int(rng.integers(1, 33))
    ups = small_queue(seed, sizes, Q, 0.35, zero_frac=0.15)
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    lr = 0.125
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    runs = {}
    for method in METHODS:
        theta = [t.copy() for t in theta0]
        theta64 = [t.astype(np.float64) for t in theta0]
        ps, ps64 = oracle.ParameterServer(theta, method), oracle.ParameterServer(theta64, method, f64=True)
        sigs = []
        for u, j in zip(ups, pulls):
            sigs.append(ps.apply(*u, j, lr, want_sigma=True))
            assert np.array_equal(sigs[-1], ps64.apply(*u, j, lr, want_sigma=True))
        runs[method] = (theta, theta64, sigs)
    # brute force with dense vectors
    dense_hist = []
    ref = [t.astype(np.float64) for t in theta0]
    for q, ((off, idx, val), j) in enumerate(zip(ups, pulls)):
        dense = [np.zeros(n, dtype=np.float32) for n in sizes]
        for l in range(len(sizes)):
            for e in range(int(off[l]), int(off[l + 1])):
                k = int(idx[e])
                sigma = sum(int(dense_hist[u][l][k] != 0) for u in range(j, q))
                assert sigma == int(runs[METHODS[0]][2][q][e])
                ref[l][k] -= (lr / sigma if sigma else lr) * float(val[e])
                dense[l][k] = val[e]
        dense_hist.append(dense)
    for l in range(len(sizes)):
        assert np.array_equal(runs[METHODS[0]][0][l], runs[METHODS[1]][0][l])
        assert np.array_equal(runs[METHODS[0]][1][l], runs[METHODS[1]][1][l])
        assert np.allclose(runs[METHODS[0]][1][l], ref[l], rtol=1e-13, atol=1e-15)
        assert np.allclose(runs[METHODS[0]][0][l], ref[l], rtol=0, atol=Q * 2.0 ** -22 * 4)


@pytest.mark.parametrize("method", METHODS)
def test_transmitted_zeros_do_not_count(method):
    """An entry whose value is +-0 is in the index list but is not 'Delta Theta_k != 0'
    (eq. 3): it leaves later staleness alone; a denormal does count."""
    theta = [np.ones(3, dtype=np.float32)]
    ps = oracle.ParameterServer(theta, method)
    ps.apply(*upd([3], [{0: 0.0, 1: -0.0, 2: 1e-40}]), 0, 1.0)
    assert theta[0][0] == 1.0 and theta[0][1] == 1.0
    s = ps.apply(*upd([3], [{0: 1.0, 1: 1.0, 2: 1.0}]), 0, 1.0, want_sigma=True)
    assert s.tolist() == [0, 0, 1]


def test_empty_update_advances_time_only():
    theta = [np.ones(4, dtype=np.float32)]
    ps = oracle.ParameterServer(theta)
    ps.apply(*upd([4], [{1: 1.0}]), 0, 1.0)
    ps.apply(*upd([4], [{}]), 0, 1.0)
    assert ps.t == 2
    s = ps.apply(*upd([4], [{1: 1.0}]), 0, 1.0, want_sigma=True)
    assert s.tolist() == [1] and ps.t == 3


def test_splitting_a_tensor_changes_nothing():
    """Parameters are independent: one 60-entry tensor or the same split 25 + 35."""
    rng = np.random.default_rng(5)
    Q = 15
    whole = small_queue(9, [60], Q, 0.3)
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    t_whole = [np.zeros(60, dtype=np.float32)]
    t_split = [np.zeros(25, dtype=np.float32), np.zeros(35, dtype=np.float32)]
    ps_w, ps_s = oracle.ParameterServer(t_whole), oracle.ParameterServer(t_split)
    for (off, idx, val), j in zip(whole, pulls):
        ps_w.apply(off, idx, val, j, 0.3)
        cut = int(np.searchsorted(idx, 25))
        idx2 = idx.copy()
        idx2[cut:] -= 25
        ps_s.apply(np.array([0, cut, idx.size], dtype=np.uint64), idx2, val, j, 0.3)
    assert np.array_equal(t_whole[0], np.concatenate(t_split))


def test_lr_power_of_two_scaling_single_touch():
    ups = [upd([32], [{k: 0.1 * (k + 1)}]) for k in range(32)]
    res = []
    for lr in (0.25, 1.0):
        theta = [np.zeros(32, dtype=np.float32)]
        ps = oracle.ParameterServer(theta)
        for u in ups:
            ps.apply(*u, 0, lr)
        res.append(theta[0])
    assert np.array_equal(res[0] * np.float32(4.0), res[1])


def test_workload_shaped_queue_lists_vs_bitmap():
    """A queue with the cnn configuration's staleness draw on its small tensors."""
    cfg = "cnn_apply"
    layers = [0, 1, 3, 5, 6, 7]
    Q = 30
    stale = workloads.staleness(cfg, Q)
    pulls = workloads.pull_timestamps(stale)
    assert all(1 <= s <= 200 for s in stale) and all(0 <= p <= q for q, p in enumerate(pulls))
    t0 = [t.numpy().copy() for t in workloads.theta0(cfg, layers=layers)]
    ta, tb = [t.copy() for t in t0], [t.copy() for t in t0]
    pa, pb = oracle.ParameterServer(ta, oracle.HISTORY_LISTS), oracle.ParameterServer(tb, oracle.HISTORY_BITMAP)
    for q in range(Q):
        g = [x.numpy() for x in workloads.gradient(cfg, q, layers=layers)]
        off, idx, val = oracle.select(g, 0.05)
        sa = pa.apply(off, idx, val, pulls[q], 0.01, want_sigma=True)
        sb = pb.apply(off, idx, val, pulls[q], 0.01, want_sigma=True)
        assert np.array_equal(sa, sb) and sa.max() <= q - pulls[q]
    for a, b in zip(ta, tb):
        assert np.array_equal(a, b)
