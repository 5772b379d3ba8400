"""GPU parity: adacomp_apply (HIP, through the C ABI) against the CPU oracle's parameter server.

Contract: parameters within 1e-6 relative of the fp32 oracle (|a-b| <= 1e-6 * max(|a|,|b|,1e-30)).
Both sides evaluate eqs. 5 and 4 as divide, multiply, subtract in fp32, so in practice the
results are expected to be identical; the tests report the number of differing entries.
Against the fp64 oracle the bound is the accumulated fp32 rounding: with m touches of a
parameter, |err| <= 3 * m * 2^-24 * max|intermediate value|.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import gpu_select, oracle_select_parallel, rel_err, update_to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ac():
    import paper_1702_04683_amd as pkg
    pkg.load_library()
    return pkg


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda:0")


def run_gpu(ac, theta_host, updates_host, pulls, lr, dev, chunks=None, state=None, history=0):
    """updates_host: list of (off, idx, val).  Returns (theta list of numpy, counters, state)."""
    theta = [torch.from_numpy(t.copy()).to(dev) for t in theta_host]
    L = len(theta)
    ups = [ac.Update.from_host(o, i, v, dev, pull_ts=p) for (o, i, v), p in zip(updates_host, pulls)]
    st = ac.State(theta, history=history) if state is None else state
    chunks = chunks or [len(ups)]
    pos = 0
    for c in chunks:
        part = ups[pos:pos + c]
        ws = torch.empty(max(ac.adacomp_apply_workspace([t.numel() for t in theta], part, st), 256), dtype=torch.uint8, device=dev)
        ac.adacomp_apply(theta, st, part, lr, ws)
        pos += c
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in theta], [c.cpu().numpy() for c in st.cnt], st


def run_oracle(theta_host, updates_host, pulls, lr, method=oracle.HISTORY_LISTS, f64=False):
    theta = [t.astype(np.float64) if f64 else t.copy() for t in theta_host]
    ps = oracle.ParameterServer(theta, method, f64=f64)
    for (o, i, v), p in zip(updates_host, pulls):
        ps.apply(o, i, v, p, lr)
    return theta


def run_oracle_per_tensor(theta_host, updates_host, pulls, lr, method=oracle.HISTORY_LISTS, threads=16):
    """The oracle's server, one instance per tensor, in parallel threads (the C call releases the
    GIL).  Every instance sees the whole queue restricted to its tensor, so its timestamps are the
    queue's; eqs. 3-5 couple nothing across parameters (pinned on the CPU by the oracle's
    split-a-tensor test)."""
    from concurrent.futures import ThreadPoolExecutor

    def one(l):
        ups = []
        for o, i, v in updates_host:
            a, b = int(o[l]), int(o[l + 1])
            ups.append((np.array([0, b - a], dtype=np.uint64), i[a:b], v[a:b]))
        return run_oracle([theta_host[l]], ups, pulls, lr, method=method)[0]

    order = sorted(range(len(theta_host)), key=lambda l: -theta_host[l].size)   # largest first
    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = dict(zip(order, ex.map(one, order)))
    return [res[l] for l in range(len(theta_host))]


def compare(got, want, what):
    worst, differing = 0.0, 0
    for l, (a, b) in enumerate(zip(got, want)):
        worst = max(worst, rel_err(a, b))
        differing += int(np.count_nonzero(a.view(np.uint32) != b.view(np.uint32)))
    print(f"[apply] {what}: max rel err {worst:.3e}, entries not bit-identical: {differing}", flush=True)
    assert worst <= 1e-6, what
    return differing


def random_updates(rng, sizes, Q, density, pool=None, zero_frac=0.0):
    ups = []
    for _ in range(Q):
        off, idx, val = [0], [], []
        for n in sizes:
            k = min(n, max(0, int(round(density * n)))) if n else 0
            if pool is not None:
                cand = np.unique(rng.integers(0, min(n, pool), size=k)) if k else np.empty(0, np.int64)
            else:
                cand = np.sort(rng.choice(n, size=k, replace=False)) if k else np.empty(0, np.int64)
            v = rng.standard_normal(cand.size).astype(np.float32)
            if zero_frac:
                z = rng.random(cand.size) < zero_frac
                v[z] = np.where(rng.random(int(z.sum())) < 0.5, 0.0, -0.0).astype(np.float32)
            idx.append(cand.astype(np.uint32))
            val.append(v)
            off.append(off[-1] + cand.size)
        ups.append((np.array(off, dtype=np.uint64), np.concatenate(idx) if idx else np.empty(0, np.uint32),
                    np.concatenate(val) if val else np.empty(0, np.float32)))
    return ups


def test_small_random_queues_bit_exact(ac, dev):
    """Dense overlap, zero-valued entries, empty tensors and empty updates, random pull times."""
    rng = np.random.default_rng(42)
    for trial in range(6):
        sizes = [int(rng.integers(1, 3000)) for _ in range(5)] + [0, 1]
        Q = int(rng.integers(1, 50))
        ups = random_updates(rng, sizes, Q, 0.2, zero_frac=0.1)
        if Q > 3:
            ups[2] = (np.zeros(len(sizes) + 1, dtype=np.uint64), np.empty(0, np.uint32), np.empty(0, np.float32))
        pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
        theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
        got, cnt, st = run_gpu(ac, theta0, ups, pulls, 0.05, dev)
        want = run_oracle(theta0, ups, pulls, 0.05)
        assert st.t == Q
        assert compare(got, want, f"random queue {trial}") == 0


def test_split_calls_equal_one_call_when_pulls_stay_inside(ac, dev):
    """State carries over between calls (timestamp and counters); a pull before the current call is refused."""
    rng = np.random.default_rng(8)
    sizes = [500, 77]
    Q = 24
    ups = random_updates(rng, sizes, Q, 0.3)
    pulls = [max(q - int(rng.integers(0, 4)), (q // 8) * 8) for q in range(Q)]   # never before the chunk start
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    one, _, _ = run_gpu(ac, theta0, ups, pulls, 0.1, dev)
    three, _, st = run_gpu(ac, theta0, ups, pulls, 0.1, dev, chunks=[8, 8, 8])
    want = run_oracle(theta0, ups, pulls, 0.1)
    assert st.t == Q
    assert compare(one, want, "one call") == 0 and compare(three, want, "three calls") == 0
    theta = [torch.from_numpy(t.copy()).to(dev) for t in theta0]
    u = ac.Update.from_host(*ups[0], dev, pull_ts=3)
    ws = torch.empty(4096, dtype=torch.uint8, device=dev)
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_apply(theta, st, [u], 0.1, ws)
    assert e.value.code == -9 and st.t == Q


def test_closed_forms_on_gpu(ac, dev):
    """Harmonic sum, the three-worker chronology, unit staleness = plain SGD, keep-all = dense ASGD."""
    one = (np.array([0, 1], dtype=np.uint64), np.array([0], dtype=np.uint32), np.array([1.0], dtype=np.float32))
    got, _, _ = run_gpu(ac, [np.zeros(1, np.float32)], [one] * 4, [0] * 4, 1.0, dev)
    assert abs(float(got[0][0]) + 17 / 6) < 3e-7
    mk = lambda d: (np.array([0, len(d)], dtype=np.uint64), np.array(sorted(d), dtype=np.uint32),
                    np.array([d[k] for k in sorted(d)], dtype=np.float32))
    ups = [mk({0: 1, 1: 1}), mk({1: 1, 2: 1}), mk({1: 1, 2: 1, 3: 1})]
    got, _, _ = run_gpu(ac, [np.zeros(4, np.float32)], ups, [0, 0, 0], 1.0, dev)
    assert got[0].tolist() == [-1.0, -2.5, -2.0, -1.0]
    rng = np.random.default_rng(1)
    sizes = [1000, 10]
    ups = random_updates(rng, sizes, 20, 0.5)
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    got, _, _ = run_gpu(ac, theta0, ups, [max(0, q - 1) for q in range(20)], 0.01, dev)
    sgd = [t.copy() for t in theta0]
    for o, i, v in ups:
        for l in range(2):
            sl = slice(int(o[l]), int(o[l + 1]))
            sgd[l][i[sl]] = sgd[l][i[sl]] - np.float32(0.01) * v[sl]
    assert all(np.array_equal(a, b) for a, b in zip(got, sgd))
    dense = random_updates(rng, sizes, 12, 1.0)
    dense = [(o, i, v + np.float32(3.0)) for o, i, v in dense]
    stale = rng.integers(0, 6, 12).tolist()
    pulls = [max(0, q - s) for q, s in enumerate(stale)]
    got, _, _ = run_gpu(ac, theta0, dense, pulls, 0.05, dev)
    ref = [t.copy() for t in theta0]
    for q, (o, i, v) in enumerate(dense):
        a = np.float32(0.05) / np.float32(max(1, q - pulls[q]))
        for l in range(2):
            ref[l] = (ref[l] - a * v[int(o[l]):int(o[l + 1])]).astype(np.float32)
    assert all(np.array_equal(a, b) for a, b in zip(got, ref))


def test_cnn_apply_config(ac, dev):
    """Config 'PS apply for the small CNN': 200 queued 1% updates made by the oracle's own
    selection from 200 seeded gradients, staleness uniform in [1, 200], lr 0.01."""
    cfg, rate = "cnn_apply", 0.01
    Q = workloads.CONFIGS[cfg]["Q"]
    lr = workloads.CONFIGS[cfg]["lr"]
    stale = workloads.staleness(cfg)
    pulls = workloads.pull_timestamps(stale)
    print("[apply] cnn: oracle selects 200 gradients", flush=True)
    grads = [[x.numpy() for x in workloads.gradient(cfg, q)] for q in range(Q)]
    ups = oracle_select_parallel(grads, rate, threads=12)
    del grads
    theta0 = [t.numpy() for t in workloads.theta0(cfg)]
    print("[apply] cnn: gpu apply", flush=True)
    got, _, st = run_gpu(ac, theta0, ups, pulls, lr, dev)
    assert st.t == Q
    print("[apply] cnn: oracle apply", flush=True)
    want = run_oracle(theta0, ups, pulls, lr, method=oracle.HISTORY_BITMAP)
    assert compare(got, want, "cnn_apply vs fp32 oracle") == 0
    want64 = run_oracle(theta0, ups, pulls, lr, method=oracle.HISTORY_BITMAP, f64=True)
    for a, b in zip(got, want64):
        assert np.all(np.abs(a - b) <= 3 * Q * 2.0 ** -24 * np.maximum(np.abs(b), 0.2))


@pytest.mark.parametrize("rate", [0.001, 0.01, 0.1])
def test_mid_apply_config(ac, dev, rate):
    """Config 'mid-size CNN' at 0.1%, 1% and 10% (at 10% every parameter is touched 6 times on
    average): 64 queued updates, staleness uniform in [1, 64].  The whole model, all 8 tensors
    including the 37.7M- and 16.8M-parameter ones, is checked entry by entry against the oracle;
    the updates come from the oracle's own selection from the seeded gradients."""
    cfg = "mid"
    sizes = workloads.sizes_of(cfg)
    Q, lr = 64, workloads.CONFIGS[cfg]["lr"]
    pulls = workloads.pull_timestamps(workloads.staleness(cfg))
    print(f"[apply] mid at {rate}: oracle selects 64 gradients of {sum(sizes)} entries", flush=True)
    grads = [[x.cpu().numpy() for x in workloads.gradient(cfg, q, device=dev)] for q in range(Q)]
    ups = oracle_select_parallel(grads, rate, threads=16)
    del grads
    theta0 = [t.numpy() for t in workloads.theta0(cfg)]
    print(f"[apply] mid at {rate}: gpu, {int(ups[0][0][-1])} entries per update", flush=True)
    got, _, st = run_gpu(ac, theta0, ups, pulls, lr, dev)
    assert st.t == Q
    print(f"[apply] mid at {rate}: oracle", flush=True)
    want = run_oracle_per_tensor(theta0, ups, pulls, lr, method=oracle.HISTORY_BITMAP)
    assert compare(got, want, f"mid apply at {rate}, whole model") == 0


def test_extreme_staleness_long_queue(ac, dev):
    """Staleness 1 and 10^4 side by side: 10,050 queued updates of one entry per tensor (rate 1/N),
    drawn from a handful of parameters per tensor so that sigma_k reaches the thousands."""
    rng = np.random.default_rng(77)
    sizes = workloads.sizes_of("adversarial")[:12]
    Q = 10_050
    ups = []
    for q in range(Q):
        idx = np.array([rng.integers(0, min(n, 3)) for n in sizes], dtype=np.uint32)
        val = rng.standard_normal(len(sizes)).astype(np.float32)
        ups.append((np.arange(len(sizes) + 1, dtype=np.uint64), idx, val))
    stale = [1 if q % 2 else 10_000 for q in range(Q)]
    pulls = workloads.pull_timestamps(stale)
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    print("[apply] long queue: gpu", flush=True)
    got, cnt, st = run_gpu(ac, theta0, ups, pulls, 0.01, dev)
    assert st.t == Q
    print("[apply] long queue: oracle", flush=True)
    want = run_oracle(theta0, ups, pulls, 0.01)
    assert compare(got, want, "long queue") == 0
    assert max(int(c.max()) for c in cnt) > 3000      # this queue runs update by update: counters reach the thousands


@pytest.mark.parametrize("plan", ["auto", "sweep"])
def test_extreme_staleness_all_adversarial_tensors(ac, dev, plan, monkeypatch):
    """The same 10,050-update queue (staleness 1 and 10^4 alternating) on all 40 adversarial tensors,
    every update taking its one entry per tensor from a pool of up to 64 parameters spread over
    the whole tensor, 5% of the values exact zeros.  Run as the library chooses and with the sweep
    forced: there the general sorting kernel stages the queue 256 updates at a time in 40,000 tiles,
    and the tiles of the small tensors, which collect up to 10,050 entries, go to the kernel that
    replays a tile from global memory."""
    if plan != "auto":
        monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
    rng = np.random.default_rng(78)
    sizes = workloads.sizes_of("adversarial")
    assert len(sizes) == 40
    Q = 10_050
    pools = [np.sort(rng.choice(n, size=min(n, 64), replace=False)) for n in sizes]
    ups = []
    for q in range(Q):
        idx = np.array([p[rng.integers(0, p.size)] for p in pools], dtype=np.uint32)
        val = rng.standard_normal(len(sizes)).astype(np.float32)
        val[rng.random(len(sizes)) < 0.05] = 0.0
        ups.append((np.arange(len(sizes) + 1, dtype=np.uint64), idx, val))
    stale = [1 if q % 2 else 10_000 for q in range(Q)]
    pulls = workloads.pull_timestamps(stale)
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    print(f"[apply] long queue, 40 tensors, plan {plan}: gpu", flush=True)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.01, dev)
    assert st.t == Q
    print(f"[apply] long queue, 40 tensors, plan {plan}: oracle", flush=True)
    want = run_oracle(theta0, ups, pulls, 0.01)
    assert compare(got, want, f"long queue, 40 tensors, plan {plan}") == 0


@pytest.mark.parametrize("Q", [300, 1000])
def test_long_spread_queues_through_the_general_sweep(ac, dev, monkeypatch, Q):
    """Queues longer than the kernels for short and dense queues take (more than 256 updates), with
    the sweep forced: entries spread over ragged tensors of several tiles each, a stretch that every
    update hits (its tile overflows and is replayed from global memory), zero-valued entries,
    random pulls; in one call and in three calls with a trace."""
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "sweep")
    rng = np.random.default_rng(600 + Q)
    sizes = [2048 * 9 + 5, 1, 0, 50_001, 777]
    ups = random_updates(rng, sizes, Q, 0.003, zero_frac=0.1)
    hot = np.arange(30_000, 30_003, dtype=np.uint32)
    for q in range(Q):
        off, idx, val = ups[q]
        a, b = int(off[3]), int(off[4])
        merged = np.union1d(idx[a:b], hot).astype(np.uint32)
        v = rng.standard_normal(merged.size).astype(np.float32)
        shift = merged.size - (b - a)
        ups[q] = (np.concatenate([off[:4], off[4:] + shift]).astype(np.uint64),
                  np.concatenate([idx[:a], merged, idx[b:]]), np.concatenate([val[:a], v, val[b:]]))
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    want = run_oracle(theta0, ups, pulls, 0.02)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev)
    assert st.t == Q
    assert compare(got, want, f"general sweep, Q={Q}, one call") == 0
    a = Q // 3
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev, chunks=[a, 2, Q - a - 2], history=Q)
    assert compare(got, want, f"general sweep, Q={Q}, three calls with a trace") == 0


def test_flat_config_full_size_sampled(ac, dev):
    """The roofline configuration in the launch shapes bench.py times: 16 seeded 1B-element worker
    gradients (100 tensors of 10M each) go through ONE adacomp_select call over the 1600 tensors
    at 0.5%; its output is viewed as 16 updates (staleness uniform in [1, 16]) and applied by one
    adacomp_apply call to 100 tensors of 10M parameters.  The oracle replays ten tensors
    chosen by seed (its own selection from the same bits, its own apply); properties that hold at any size are
    checked on many more."""
    cfg, rate = "flat", 0.005
    sizes = workloads.sizes_of(cfg)
    L, Q, lr = len(sizes), 16, workloads.CONFIGS[cfg]["lr"]
    pulls = workloads.pull_timestamps(workloads.staleness(cfg))
    sample = sorted(int(l) for l in np.random.default_rng(4004).choice(L, size=10, replace=False))
    theta = workloads.theta0(cfg, device=dev)
    theta0 = {l: theta[l].cpu().numpy().copy() for l in sample}
    print("[apply] flat: generating 16 gradients (64 GB)", flush=True)
    grads = [workloads.gradient(cfg, q, device=dev) for q in range(Q)]
    host_g = {l: [grads[q][l].cpu().numpy() for q in range(Q)] for l in sample}
    k = ac.adacomp_count(sizes[0], rate)
    print("[apply] flat: one select call over 1600 tensors", flush=True)
    big = gpu_select(ac, [t for g in grads for t in g], rate)
    assert big.offsets == [k * i for i in range(L * Q + 1)]
    # select, any size: per tensor the threshold is the k-th largest magnitude, everything above it is
    # there, ties go to the lowest indices, values are the tensor's own bits (every 8th tensor)
    for t in range(0, L * Q, 8):
        g = grads[t // L][t % L]
        idx = big.idx[t * k:(t + 1) * k].to(torch.int64)
        val = big.val[t * k:(t + 1) * k]
        assert bool((idx[1:] > idx[:-1]).all()) and 0 <= int(idx[0]) and int(idx[-1]) < sizes[t % L]
        assert torch.equal(g[idx].view(torch.int32), val.view(torch.int32))
        key = g.view(torch.int32) & 0x7FFFFFFF
        T = int((val.view(torch.int32) & 0x7FFFFFFF).min())
        n_gt = int((key > T).sum())
        assert n_gt < k <= int((key >= T).sum()), f"tensor {t}: threshold"
        assert int((key[idx] > T).sum()) == n_gt, f"tensor {t}: an entry above the threshold is missing"
        assert torch.equal(idx[key[idx] == T], torch.nonzero(key == T).flatten()[:k - n_gt]), f"tensor {t}: ties"
    del grads
    ups = [big.view(q * L, (q + 1) * L, pull_ts=pulls[q]) for q in range(Q)]
    st = ac.State(theta)
    aws = torch.empty(ac.adacomp_apply_workspace(sizes, ups, st), dtype=torch.uint8, device=dev)
    print("[apply] flat: gpu apply", flush=True)
    ac.adacomp_apply(theta, st, ups, lr, aws)
    torch.cuda.synchronize()
    assert st.t == Q
    # apply, any size: parameters no update names are untouched, the others moved
    theta_before = workloads.theta0(cfg, device=dev)
    for l in range(L):
        touched = torch.zeros(sizes[l], dtype=torch.bool, device=dev)
        for u in ups:
            touched[u.idx[l * k:(l + 1) * k].to(torch.int64)] = True
        same = theta[l] == theta_before[l]
        assert bool(same[~touched].all()), f"tensor {l}: an unnamed parameter changed"
        assert float(same[touched].float().mean()) < 0.01, f"tensor {l}: named parameters did not move"
    del theta_before
    print(f"[apply] flat: oracle on sampled tensors {sample}", flush=True)
    jobs = [[host_g[l][q]] for l in sample for q in range(Q)]
    sel = oracle_select_parallel(jobs, rate, threads=16)
    del jobs, host_g
    o_ups = {l: sel[n * Q:(n + 1) * Q] for n, l in enumerate(sample)}
    for l in sample:
        for q, (o, i, v) in enumerate(o_ups[l]):    # the batched select against the oracle, entry by entry
            assert np.array_equal(ups[q].idx[l * k:(l + 1) * k].cpu().numpy().view(np.uint32), i), (q, l)
            assert np.array_equal(ups[q].val[l * k:(l + 1) * k].cpu().numpy().view(np.uint32), v.view(np.uint32))
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=10) as ex:
        wants = list(ex.map(lambda l: run_oracle([theta0[l]], o_ups[l], pulls, lr)[0], sample))
    for l, want in zip(sample, wants):
        assert compare([theta[l].cpu().numpy()], [want], f"flat tensor {l}") == 0


@pytest.mark.parametrize("plan", ["scatter", "sweep"])
def test_both_plans_on_the_same_queues(ac, dev, plan, monkeypatch):
    """The execution plan is an internal choice; forced either way the result is the oracle's.
    Includes queues that overflow a tile's LDS lists (hot coordinates, dense updates), which the
    sweep hands to its per-tile fallback kernel."""
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
    rng = np.random.default_rng(2024)
    cases = []
    # sparse, many tensors, ragged sizes, several tiles per tensor
    sizes = [70_001, 5, 0, 12_345, 1, 300_000]
    cases.append(("sparse", sizes, random_updates(rng, sizes, 40, 0.01, zero_frac=0.05)))
    # dense: every update touches 60% of every tensor -> tiles overflow the stage
    sizes = [5_000, 777]
    cases.append(("dense", sizes, random_updates(rng, sizes, 30, 0.6)))
    # hot coordinates: 400 updates all hitting the same few parameters -> lists longer than a tile can stage
    sizes = [10_000, 3]
    hot = []
    for q in range(400):
        i0 = np.unique(np.concatenate([[7, 4099, 9999], rng.integers(0, 10_000, 20)])).astype(np.uint32)
        i1 = np.array([0, 2], dtype=np.uint32)
        v = rng.standard_normal(i0.size + 2).astype(np.float32)
        hot.append((np.array([0, i0.size, i0.size + 2], dtype=np.uint64), np.concatenate([i0, i1]), v))
    cases.append(("hot", sizes, hot))
    for name, sizes, ups in cases:
        Q = len(ups)
        pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
        theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
        got, cnt, st = run_gpu(ac, theta0, ups, pulls, 0.03, dev)
        want = run_oracle(theta0, ups, pulls, 0.03)
        assert st.t == Q
        assert compare(got, want, f"{plan}/{name}") == 0
        if plan == "scatter":   # this plan's scratch counters: at most one increment per applied non-zero entry
            for l, n in enumerate(sizes):  # (the last updates of a call, which no later one looks back on, are not counted)
                ref = np.zeros(max(n, 1), dtype=np.int64)
                for o, i, v in ups:
                    sl = slice(int(o[l]), int(o[l + 1]))
                    np.add.at(ref, i[sl][v[sl] != 0], 1)
                assert np.all(cnt[l].astype(np.int64) <= ref), f"{plan}/{name} counters tensor {l}"


def test_sweep_and_scatter_agree_on_cnn_queue_bitwise(ac, dev, monkeypatch):
    """Same seeded queue (updates built with torch.topk here, not by either implementation under
    test), both plans: identical parameters and counters."""
    cfg = "cnn_apply"
    sizes = workloads.sizes_of(cfg)
    Q = 40
    pulls = workloads.pull_timestamps(workloads.staleness(cfg, Q))
    ups = []
    for q in range(Q):
        off, idx, val = [0], [], []
        for g in workloads.gradient(cfg, q, device=dev):
            k = max(1, g.numel() // 100)
            i = torch.topk(g.abs(), k).indices.sort().values
            idx.append(i.cpu().numpy().astype(np.uint32))
            val.append(g[i].cpu().numpy())
            off.append(off[-1] + k)
        ups.append((np.array(off, dtype=np.uint64), np.concatenate(idx), np.concatenate(val)))
    theta0 = [t.numpy() for t in workloads.theta0(cfg)]
    res = {}
    for plan in ("scatter", "sweep"):
        monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
        res[plan] = run_gpu(ac, theta0, ups, pulls, 0.01, dev)
    for a, b in zip(res["scatter"][0], res["sweep"][0]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    want = run_oracle(theta0, ups, pulls, 0.01, method=oracle.HISTORY_BITMAP)
    assert compare(res["sweep"][0], want, "cnn queue, sweep") == 0


@pytest.mark.parametrize("plan", ["scatter", "sweep", "auto"])
def test_pulls_reaching_back_across_calls(ac, dev, plan, monkeypatch):
    """The parameter server of Alg. 2 receives updates a few at a time; a worker may have pulled
    long before the current call.  With a trace of the last d updates the earlier part of the
    window of eq. 3 is searched in the remembered index lists; the result must be the oracle's,
    whatever the split into calls."""
    if plan != "auto":
        monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
    rng = np.random.default_rng(31)
    d = 16
    for trial, (sizes, Q, density) in enumerate([([4000, 37, 1], 70, 0.05), ([700], 50, 0.4), ([30_000, 5], 40, 0.01)]):
        ups = random_updates(rng, sizes, Q, density, zero_frac=0.1)
        ups[5] = (np.zeros(len(sizes) + 1, dtype=np.uint64), np.empty(0, np.uint32), np.empty(0, np.float32))
        pulls = [int(rng.integers(max(0, q - d), q + 1)) for q in range(Q)]
        chunks = []
        while sum(chunks) < Q:
            chunks.append(min(int(rng.integers(1, 8)), Q - sum(chunks)))
        theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
        got, cnt, st = run_gpu(ac, theta0, ups, pulls, 0.07, dev, chunks=chunks, history=d)
        want = run_oracle(theta0, ups, pulls, 0.07)
        assert st.t == Q
        assert compare(got, want, f"{plan}/history trial {trial}, calls {chunks[:6]}...") == 0


def test_one_update_per_call_is_the_server_loop_of_the_paper(ac, dev):
    """Q = 1 per call: Alg. 2 literally.  Staleness up to the whole trace."""
    rng = np.random.default_rng(32)
    sizes, Q, d = [2500, 64], 120, 40
    ups = random_updates(rng, sizes, Q, 0.1)
    pulls = [int(rng.integers(max(0, q - d), q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.05, dev, chunks=[1] * Q, history=d)
    want = run_oracle(theta0, ups, pulls, 0.05)
    assert compare(got, want, "one update per call") == 0
    # a pull older than the trace is refused and changes nothing
    theta = [torch.from_numpy(t.copy()).to(dev) for t in theta0]
    u = ac.Update.from_host(*ups[0], dev, pull_ts=Q - d - 1)
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_apply_workspace(sizes, [u], st)
    assert e.value.code == -9
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_apply(theta, st, [u], 0.05, ws)
    assert e.value.code == -9 and st.t == Q
    u.pull_ts = Q - d                                    # the oldest remembered update: accepted
    assert ac.adacomp_apply_workspace(sizes, [u], st) > 0


def test_cnn_queue_in_calls_of_eight_with_history(ac, dev):
    """cnn tensors, 48 updates (1%, chosen with torch.topk here), staleness uniform in [1, 48],
    applied eight per call with a 48-deep trace."""
    cfg = "cnn_apply"
    Q, d = 48, 48
    rng = np.random.default_rng(33)
    stale = rng.integers(1, d + 1, Q).tolist()
    pulls = workloads.pull_timestamps(stale)
    ups = []
    for q in range(Q):
        off, idx, val = [0], [], []
        for g in workloads.gradient(cfg, 300 + q, device=dev):
            k = max(1, g.numel() // 100)
            i = torch.topk(g.abs(), k).indices.sort().values
            idx.append(i.cpu().numpy().astype(np.uint32))
            val.append(g[i].cpu().numpy())
            off.append(off[-1] + k)
        ups.append((np.array(off, dtype=np.uint64), np.concatenate(idx), np.concatenate(val)))
    theta0 = [t.numpy() for t in workloads.theta0(cfg)]
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.01, dev, chunks=[8] * 6, history=d)
    want = run_oracle(theta0, ups, pulls, 0.01, method=oracle.HISTORY_BITMAP)
    assert compare(got, want, "cnn queue, calls of 8, history 48") == 0


def test_global_staleness_rule_of_the_competitors(ac, dev):
    """adacomp_apply_global_staleness against the oracle's GLOBAL mode (Sec. 5.2: one learning rate
    per update, divided by its global staleness), and the hand-worked chronology, where the
    per-parameter and the global rule differ."""
    mk = lambda d: (np.array([0, len(d)], dtype=np.uint64), np.array(sorted(d), dtype=np.uint32),
                    np.array([d[k] for k in sorted(d)], dtype=np.float32))
    ups = [mk({0: 1, 1: 1}), mk({1: 1, 2: 1}), mk({1: 1, 2: 1, 3: 1})]

    def run_global(theta_host, updates_host, pulls, lr):
        theta = [torch.from_numpy(t.copy()).to(dev) for t in theta_host]
        us = [ac.Update.from_host(o, i, v, dev, pull_ts=p) for (o, i, v), p in zip(updates_host, pulls)]
        st = ac.State(theta)
        ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
        ac.adacomp_apply_global_staleness(theta, st, us, lr, ws)
        torch.cuda.synchronize()
        assert st.t == len(us)
        return [t.cpu().numpy() for t in theta]

    got = run_global([np.zeros(4, np.float32)], ups, [0, 0, 0], 1.0)
    assert got[0].tolist() == [-1.0, -2.5, -1.5, -0.5]            # tests/golden/apply_chronology.json
    rng = np.random.default_rng(51)
    sizes = [5000, 3, 0, 777]
    Q = 30
    ups = random_updates(rng, sizes, Q, 0.2, zero_frac=0.1)
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    got = run_global(theta0, ups, pulls, 0.05)
    want = [t.copy() for t in theta0]
    ps = oracle.ParameterServer(want)
    for (o, i, v), p in zip(ups, pulls):
        ps.apply(o, i, v, p, 0.05, mode=oracle.GLOBAL)
    assert compare(got, want, "global staleness") == 0
    per_param = run_oracle(theta0, ups, pulls, 0.05)
    assert any(not np.array_equal(a, b) for a, b in zip(want, per_param)), "the two rules must differ here"


def test_global_and_per_parameter_calls_mixed_on_one_state(ac, dev):
    """Calls under the competitors' rule enter their updates into the trace like any other, so a later
    per-parameter call that looks back across them counts them (eq. 3 asks which updates touched
    the parameter, not which rule set their step)."""
    rng = np.random.default_rng(53)
    sizes, Q, d = [4000, 9, 300], 36, 12
    ups = random_updates(rng, sizes, Q, 0.15, zero_frac=0.1)
    pulls = [int(rng.integers(max(0, q - d), q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    calls = [(0, 5, "per"), (5, 9, "global"), (9, 10, "per"), (10, 20, "global"), (20, 27, "per"), (27, 36, "per")]
    theta = [torch.from_numpy(t.copy()).to(dev) for t in theta0]
    us = [ac.Update.from_host(o, i, v, dev, pull_ts=p) for (o, i, v), p in zip(ups, pulls)]
    st = ac.State(theta, history=d)
    want = [t.copy() for t in theta0]
    ps = oracle.ParameterServer(want)
    for a, b, rule in calls:
        part = us[a:b]
        if rule == "per":
            ws = torch.empty(max(ac.adacomp_apply_workspace(sizes, part, st), 256), dtype=torch.uint8, device=dev)
            ac.adacomp_apply(theta, st, part, 0.04, ws)
        else:
            ws = torch.empty(1 << 12, dtype=torch.uint8, device=dev)
            ac.adacomp_apply_global_staleness(theta, st, part, 0.04, ws)
        for q in range(a, b):
            ps.apply(*ups[q], pulls[q], 0.04, mode=oracle.PER_PARAMETER if rule == "per" else oracle.GLOBAL)
    torch.cuda.synchronize()
    assert st.t == Q
    assert compare([t.cpu().numpy() for t in theta], want, "global and per-parameter calls mixed") == 0


def test_update_validate_and_malformed_entries_are_skipped(ac, dev, monkeypatch):
    rng = np.random.default_rng(52)
    sizes = [3000, 40]
    sizes_dev = torch.tensor(sizes, dtype=torch.int64, device=dev)
    flags = torch.zeros(1, dtype=torch.int32, device=dev)
    good = random_updates(rng, sizes, 1, 0.1)[0]

    def check(o, i, v):
        u = ac.Update.from_host(o, i, v, dev)
        ac.adacomp_update_validate(u, sizes_dev, flags)
        torch.cuda.synchronize()
        return int(flags.item())

    assert check(*good) == 0
    o, i, v = good
    bad = i.copy(); bad[5] = 3000                    # outside tensor 0
    assert check(o, bad, v) & 1
    bad = i.copy(); bad[7], bad[8] = i[8], i[7]      # not ascending
    assert check(o, bad, v) == 2
    bad = i.copy(); bad[8] = bad[7]                  # duplicate
    assert check(o, bad, v) == 2
    bad = i.copy(); bad[int(o[1])] = 40              # outside tensor 1
    assert check(o, bad, v) & 1
    # apply skips an out-of-range entry and treats all others as the oracle does
    Q = 6
    ups = random_updates(rng, sizes, Q, 0.1)
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    broken = [(o.copy(), i.copy(), v.copy()) for o, i, v in ups]
    oo, ii, vv = broken[3]
    last = int(oo[1]) - 1                             # last entry of tensor 0 of update 3
    ii[last] = 3000 + 17
    cleaned = list(ups)
    keep = np.ones(ups[3][1].size, dtype=bool); keep[last] = False
    cleaned[3] = (np.array([0, int(oo[1]) - 1, int(oo[2]) - 1], dtype=np.uint64), ups[3][1][keep], ups[3][2][keep])
    want = run_oracle(theta0, cleaned, pulls, 0.05)
    for plan in ("scatter", "sweep"):
        monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
        got, _, _ = run_gpu(ac, theta0, broken, pulls, 0.05, dev)
        assert compare(got, want, f"{plan}: out-of-range entry skipped") == 0


@pytest.mark.parametrize("kernel,tpb", [("short", "1"), ("short", "2"), ("short", "4"), ("long", "1"), ("long", "2"), ("long", "4"),
                                        ("dense", "1"), ("sparse", "1"), ("sparse", "2"), ("sparse", "4")])
def test_sweep_kernels_and_tiles_per_workgroup(ac, dev, monkeypatch, kernel, tpb):
    """The sweep has a kernel for queues of up to 64 updates (all loads of a workgroup's tiles
    requested ahead) and a general one, each working through 1, 2 or 4 tiles per workgroup; forced
    each way on queues with ragged tile counts, empty tiles, tiles that overflow into the fallback
    kernel, zero-valued entries and pulls that reach back across calls: always the oracle's result."""
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "sweep")
    monkeypatch.setenv("ADACOMP_TPB", tpb)
    monkeypatch.setenv("ADACOMP_SWEEP_KERNEL", {"short": "tiled", "long": "long", "dense": "dense", "sparse": "sparse"}[kernel])
    rng = np.random.default_rng(7 + int(tpb))
    sizes = [2048 * 5 + 3, 1, 0, 2048 * 2, 70_001]            # 6 + 1 + 0 + 2 + 35 tiles of 2048
    Q = 20
    ups = random_updates(rng, sizes, Q, 0.004, zero_frac=0.1)
    # a hot stretch: every update hits the same 40 parameters of one tile -> that tile overflows its stage
    hot = np.arange(4100, 4140, dtype=np.uint32)
    for q in range(Q):
        off, idx, val = ups[q]
        a, b = int(off[0]), int(off[1])
        merged = np.union1d(idx[a:b], hot).astype(np.uint32)
        v = rng.standard_normal(merged.size).astype(np.float32)
        shift = merged.size - (b - a)
        ups[q] = (np.concatenate([off[:1], off[1:] + shift]).astype(np.uint64),
                  np.concatenate([merged, idx[b:]]), np.concatenate([v, val[b:]]))
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    want = run_oracle(theta0, ups, pulls, 0.02)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev)
    assert st.t == Q
    assert compare(got, want, f"{kernel} kernel, {tpb} tiles per workgroup, one call") == 0
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev, chunks=[7, 1, 12], history=Q)
    assert compare(got, want, f"{kernel} kernel, {tpb} tiles per workgroup, three calls with history") == 0


@pytest.mark.parametrize("seed", range(6))
def test_random_queues_shapes_and_call_splits(ac, dev, seed):
    """Seeded random queues: tensor sizes from 0 to 300K, 2 to 60 updates of random density (so short
    and long queues, large and one-parameter tiles), zero-valued entries, random pulls, applied in
    one call and in random splits with a trace; the plan is whatever the library chooses."""
    rng = np.random.default_rng(3000 + seed)
    L = int(rng.integers(1, 7))
    sizes = [int(rng.choice([0, 1, 5, 2048, 2049, int(rng.integers(1, 300_000)), int(rng.integers(1, 5_000))])) for _ in range(L)]
    Q = int(rng.integers(2, 61))
    density = float(rng.choice([0.0005, 0.004, 0.03, 0.3]))
    ups = random_updates(rng, sizes, Q, density, zero_frac=float(rng.choice([0.0, 0.2])))
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    want = run_oracle(theta0, ups, pulls, 0.01)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.01, dev)
    assert st.t == Q
    assert compare(got, want, f"random queue {seed}: Q={Q} density={density} sizes={sizes}") == 0
    chunks, left = [], Q
    while left:
        c = int(rng.integers(1, left + 1))
        chunks.append(c)
        left -= c
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.01, dev, chunks=chunks, history=Q)
    assert compare(got, want, f"random queue {seed} in calls of {chunks}") == 0


def test_calls_longer_than_the_trace(ac, dev):
    """A call that applies more updates than the trace can remember keeps the last `d` of them; the
    next call may reach back exactly that far and no further."""
    rng = np.random.default_rng(35)
    sizes, d = [3000, 9], 4
    Q = 10 + 3 + 12 + 1
    ups = random_updates(rng, sizes, Q, 0.05, zero_frac=0.1)
    call_start = [0] * 10 + [10] * 3 + [13] * 12 + [25]
    pulls = [int(rng.integers(max(0, call_start[q] - d), q + 1)) for q in range(Q)]
    pulls[10] = 10 - d                                   # the oldest remembered update, exactly
    pulls[25] = 25 - d
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.05, dev, chunks=[10, 3, 12, 1], history=d)
    want = run_oracle(theta0, ups, pulls, 0.05)
    assert st.t == Q
    assert compare(got, want, "calls longer than the trace") == 0
    u = ac.Update.from_host(*ups[0], dev, pull_ts=Q - d - 1)
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_apply_workspace(sizes, [u], st)
    assert e.value.code == -9


def test_queue_longer_than_the_sweep_can_number(ac, dev):
    """More than 32767 updates in one call: the sweep's 15-bit update numbers do not suffice, the call
    runs update by update (two launches each); staleness up to 50."""
    rng = np.random.default_rng(36)
    sizes = [40, 3]
    Q = 33_000
    ups = []
    for q in range(Q):
        i0 = np.unique(rng.integers(0, 40, 3)).astype(np.uint32)
        i1 = np.array([int(rng.integers(0, 3))], dtype=np.uint32)
        v = rng.standard_normal(i0.size + 1).astype(np.float32)
        ups.append((np.array([0, i0.size, i0.size + 1], dtype=np.uint64), np.concatenate([i0, i1]), v))
    pulls = [max(0, q - int(rng.integers(0, 51))) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    print("[apply] 33000 updates: gpu", flush=True)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 1e-3, dev)
    assert st.t == Q
    print("[apply] 33000 updates: oracle", flush=True)
    want = run_oracle(theta0, ups, pulls, 1e-3)
    assert compare(got, want, "33000 updates") == 0


def test_degenerate_calls(ac, dev):
    """No tensors, no updates, empty updates only, tensors of zero size only: legal, nothing but the
    timestamp changes."""
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=dev)
    none = ac.Update(0, 0, dev)
    ac.adacomp_select([], 0.5, none, ws)
    assert none.offsets == [0]
    st = ac.State([])
    ac.adacomp_apply([], st, [none, none], 0.1, ws)          # two pushes to a model without parameters
    assert st.t == 2
    ac.adacomp_apply([], st, [], 0.1, ws)
    assert st.t == 2
    theta = [torch.arange(10, dtype=torch.float32, device=dev), torch.empty(0, device=dev)]
    before = theta[0].clone()
    st = ac.State(theta)
    empty = ac.Update.from_host(np.zeros(3, dtype=np.uint64), np.empty(0, np.uint32), np.empty(0, np.float32), dev)
    for plan_q in (1, 5):
        ac.adacomp_apply(theta, st, [empty] * plan_q, 0.1, ws)
    torch.cuda.synchronize()
    assert st.t == 6 and torch.equal(theta[0], before)
    # empty updates carry pull_ts 0 throughout: without entries there is no staleness to look up;
    # a fresh update after the six empty pushes takes the full step
    u = ac.Update.from_host(np.array([0, 2, 2], dtype=np.uint64), np.array([1, 9], dtype=np.uint32),
                            np.array([1.0, -1.0], dtype=np.float32), dev, pull_ts=6)
    ac.adacomp_apply(theta, st, [u], 0.5, ws)
    torch.cuda.synchronize()
    assert theta[0].tolist() == [0.0, 0.5, 2.0, 3.0, 4.0, 5.0, 6.0, 7.0, 8.0, 9.5]
    zero_size = [torch.empty(0, device=dev), torch.empty(0, device=dev)]
    out = ac.Update(2, 0, dev)
    ac.adacomp_select(zero_size, 0.3, out, ws)
    st0 = ac.State(zero_size)
    ac.adacomp_apply(zero_size, st0, [out], 0.1, ws)
    torch.cuda.synchronize()
    assert out.offsets == [0, 0, 0] and st0.t == 1


@pytest.mark.parametrize("Q,density", [(2, 1.0), (17, 0.05), (33, 0.6), (64, 0.3), (64, 1.0), (65, 0.2), (130, 1.0), (200, 0.1),
                                       (256, 0.4)])
@pytest.mark.parametrize("kernel", ["dense", "tiled", "sparse"])
def test_dense_queues_one_thread_per_coordinate(ac, dev, monkeypatch, Q, density, kernel):
    """Queues with about one entry per parameter or more go through a sweep kernel of their own (a
    thread per coordinate, the non-zero touches of a coordinate as a bit mask over the queue) for
    up to 256 updates.  Forced on and off here, on ragged tensors (sizes 0, 1, 255, 256, 257), with
    slices longer than a wavefront (density 1), zero-valued entries and pulls that reach back
    across calls: the oracle's result either way."""
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "sweep")
    monkeypatch.setenv("ADACOMP_SWEEP_KERNEL", kernel)
    rng = np.random.default_rng(9000 + Q)
    sizes = [1000, 1, 0, 255, 256, 257, 3 * 256 + 100]
    ups = random_updates(rng, sizes, Q, density, zero_frac=0.15)
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    want = run_oracle(theta0, ups, pulls, 0.03)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.03, dev)
    assert st.t == Q
    assert compare(got, want, f"{kernel}: Q={Q} density={density}, one call") == 0
    if Q >= 3:
        a = Q // 3
        got, _, st = run_gpu(ac, theta0, ups, pulls, 0.03, dev, chunks=[a, 1, Q - a - 1], history=Q)
        assert compare(got, want, f"{kernel}: Q={Q} density={density}, three calls with a trace") == 0


@pytest.mark.parametrize("kernel", ["tiled", "sparse"])
@pytest.mark.parametrize("Q", [10, 64, 70])
def test_tiles_that_every_update_fills(ac, dev, monkeypatch, Q, kernel):
    """A sparse queue (large tiles) in which every update also carries one whole stretch of 3000
    consecutive parameters, as when the same rows are large in every worker's gradient: those tiles
    hold thousands of queued entries, slices of up to 2048 entries per update, and are replayed by
    the kernels for tiles that the sort declines (out of LDS up to 64 updates, from global memory
    beyond), in one call and in calls with a trace."""
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "sweep")
    monkeypatch.setenv("ADACOMP_SWEEP_KERNEL", kernel)
    rng = np.random.default_rng(500 + Q)
    sizes = [2048 * 12 + 77, 9]
    ups = random_updates(rng, sizes, Q, 0.002, zero_frac=0.1)
    hot = np.arange(5000, 8000, dtype=np.uint32)
    for q in range(Q):
        off, idx, val = ups[q]
        a, b = int(off[0]), int(off[1])
        merged = np.union1d(idx[a:b], hot).astype(np.uint32)
        v = rng.standard_normal(merged.size).astype(np.float32)
        v[rng.random(merged.size) < 0.05] = 0.0
        shift = merged.size - (b - a)
        ups[q] = (np.concatenate([off[:1], off[1:] + shift]).astype(np.uint64),
                  np.concatenate([merged, idx[b:]]), np.concatenate([v, val[b:]]))
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    want = run_oracle(theta0, ups, pulls, 0.02)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev)
    assert st.t == Q
    assert compare(got, want, f"filled tiles, Q={Q}, one call") == 0
    a = Q // 3
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev, chunks=[a, 2, Q - a - 2], history=Q)
    assert compare(got, want, f"filled tiles, Q={Q}, three calls with a trace") == 0


@pytest.mark.parametrize("tpb", ["1", "4"])
@pytest.mark.parametrize("Q,density", [(16, 0.005), (2, 0.05), (40, 0.002), (64, 0.004), (16, 0.06)])
def test_sparse_queues_lone_touches_need_no_list(ac, dev, monkeypatch, Q, density, tpb):
    """The sweep for sparse queues applies a touch that is alone on its coordinate straight from
    registers and groups only the touches of shared coordinates.  Forced here on ragged tensors of
    several tiles with: a stretch of 200 coordinates that a third of the updates hit (a few hundred
    entries on shared coordinates in one tile), a stretch of 400 coordinates that every update hits
    (more shared entries than the kernel lists: the tile must be left untouched for the kernel for
    overflowing tiles), a tile that collects more entries than the kernel stages at all,
    zero-valued entries, and pulls that reach back across calls (lone touches then carry the
    staleness accumulated before the call)."""
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "sweep")
    monkeypatch.setenv("ADACOMP_SWEEP_KERNEL", "sparse")
    monkeypatch.setenv("ADACOMP_TPB", tpb)
    rng = np.random.default_rng(7000 + Q)
    sizes = [4096 * 6 + 11, 1, 0, 4096 * 2, 90_001, 4097]
    ups = random_updates(rng, sizes, Q, density, zero_frac=0.1)
    some = np.arange(9000, 9200, dtype=np.uint32)        # tensor 0, tile 2
    every = np.arange(17000, 17400, dtype=np.uint32)     # tensor 0, tile 4
    full = np.arange(41000, 41000 + 1100, dtype=np.uint32)   # tensor 4, tile 10: 1100 entries from one update alone
    for q in range(Q):
        off, idx, val = ups[q]
        parts_i, parts_v, new_off = [], [], [0]
        for l in range(len(sizes)):
            a, b = int(off[l]), int(off[l + 1])
            ii = idx[a:b]
            if l == 0:
                ii = np.union1d(ii, every)
                if q % 3 == 0:
                    ii = np.union1d(ii, some)
            if l == 4 and q == Q // 2:
                ii = np.union1d(ii, full)
            ii = ii.astype(np.uint32)
            vv = rng.standard_normal(ii.size).astype(np.float32)
            vv[rng.random(ii.size) < 0.1] = 0.0
            parts_i.append(ii)
            parts_v.append(vv)
            new_off.append(new_off[-1] + ii.size)
        ups[q] = (np.array(new_off, dtype=np.uint64), np.concatenate(parts_i), np.concatenate(parts_v))
    pulls = [int(rng.integers(0, q + 1)) for q in range(Q)]
    theta0 = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    want = run_oracle(theta0, ups, pulls, 0.02)
    got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev)
    assert st.t == Q
    assert compare(got, want, f"sparse sweep, Q={Q} density={density}, one call") == 0
    if Q >= 3:
        a = Q // 3
        got, _, st = run_gpu(ac, theta0, ups, pulls, 0.02, dev, chunks=[a, 1, Q - a - 1], history=Q)
        assert compare(got, want, f"sparse sweep, Q={Q} density={density}, three calls with a trace") == 0
