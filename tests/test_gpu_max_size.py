"""The largest tensor the boundary accepts: 2^32 - 1 elements (17 GB).  No oracle can sort that in a test,
so the inputs are built to have a known answer: the k entries of largest magnitude are planted by hand
(everything else is far smaller), among them the first and the last element and both sides of 2^31.
Apply: coordinates are independent, so the oracle replays the touched coordinates as a small problem of
their own, and the untouched parameters must keep their bits."""
import numpy as np
import pytest
import torch

import oracle
from helpers import gpu_select

pytestmark = pytest.mark.gpu

N = (1 << 32) - 1


def planted_indices(rng, k):
    special = np.array([0, 1, 8191, 8192, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, N - 8193, N - 2, N - 1], dtype=np.int64)
    rest = rng.choice(N, size=k - special.size, replace=False).astype(np.int64)
    idx = np.unique(np.concatenate([special, rest]))
    assert idx.size == k
    return idx


def test_select_on_a_tensor_of_2_to_the_32_minus_1_elements():
    import paper_1702_04683_amd as ac
    ac.load_library()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(41)
    k = 1000
    print(f"[max size] generating {N} elements", flush=True)
    g = torch.empty(N, dtype=torch.float32, device=dev)
    gen = torch.Generator(device=dev).manual_seed(7)
    step = 1 << 28
    for a in range(0, N, step):                          # in pieces: no second 17 GB temporary
        g[a:a + step].normal_(0.0, 1e-3, generator=gen)
    where = planted_indices(rng, k)
    values = (rng.permutation(k).astype(np.float32) + 10.0) * rng.choice([-1.0, 1.0], size=k).astype(np.float32)
    g[torch.from_numpy(where).to(dev)] = torch.from_numpy(values).to(dev)
    print("[max size] select", flush=True)
    u = gpu_select(ac, [g], 0.5, k_override=[k])
    assert u.offsets == [0, k]
    idx = u.idx[:k].cpu().numpy().view(np.uint32).astype(np.int64)
    val = u.val[:k].cpu().numpy()
    assert np.array_equal(idx, where)
    assert np.array_equal(val.view(np.uint32), values.view(np.uint32))
    # one more than planted: the largest of the rest joins, wherever it is
    rest_max = None
    u = gpu_select(ac, [g], 0.5, k_override=[k + 1])
    idx1 = u.idx[:k + 1].cpu().numpy().view(np.uint32).astype(np.int64)
    extra = np.setdiff1d(idx1, where)
    assert extra.size == 1
    g[torch.from_numpy(where).to(dev)] = 0.0
    best = 0.0
    for a in range(0, N, step):
        best = max(best, float(g[a:a + step].abs().max()))
    assert abs(float(u.val[:k + 1].cpu().numpy()[np.searchsorted(idx1, extra[0])])) == best


def test_keep_all_and_a_quarter_of_a_tensor_of_2_to_the_32_minus_1_elements():
    """k = n (identity copy) and k = n / 4 (the descent reads the tensor itself, no candidate filter) at the
    largest size: checked piece by piece on the device against the definition of the selection."""
    import paper_1702_04683_amd as ac
    ac.load_library()
    dev = torch.device("cuda:0")
    g = torch.empty(N, dtype=torch.float32, device=dev)
    gen = torch.Generator(device=dev).manual_seed(11)
    step = 1 << 28
    for a in range(0, N, step):
        g[a:a + step].normal_(0.0, 1.0, generator=gen)
    print("[max size] keep all", flush=True)
    u = gpu_select(ac, [g], 1.0)
    assert u.offsets == [0, N]
    for a in range(0, N, step):
        b = min(a + step, N)
        want = torch.arange(a, b, device=dev, dtype=torch.int64)
        assert torch.equal(u.idx[a:b].to(torch.int64) & 0xFFFFFFFF, want)
        assert torch.equal(u.val[a:b].view(torch.int32), g[a:b].view(torch.int32))
    del u
    k = N // 4
    print(f"[max size] k = {k}", flush=True)
    u = gpu_select(ac, [g], 0.5, k_override=[k])
    assert u.offsets == [0, k]
    T = None
    for a in range(0, k, step):                           # threshold = smallest selected magnitude
        m = int((u.val[a:a + step].view(torch.int32) & 0x7FFFFFFF).min())
        T = m if T is None else min(T, m)
    n_gt = n_ge = sel_gt = 0
    for a in range(0, N, step):
        key = g[a:a + step].view(torch.int32) & 0x7FFFFFFF
        n_gt += int((key > T).sum())
        n_ge += int((key >= T).sum())
    assert n_gt < k <= n_ge, "threshold is not the k-th largest magnitude"
    last = -1
    for a in range(0, k, step):
        idx = u.idx[a:a + step].to(torch.int64) & 0xFFFFFFFF
        assert int(idx[0]) > last and bool((idx[1:] > idx[:-1]).all())          # strictly ascending
        last = int(idx[-1])
        assert torch.equal(g[idx].view(torch.int32), u.val[a:a + step].view(torch.int32))
        sel_gt += int(((u.val[a:a + step].view(torch.int32) & 0x7FFFFFFF) > T).sum())
    assert last < N and sel_gt == n_gt, "an entry above the threshold is missing"


def test_apply_on_a_tensor_of_2_to_the_32_minus_1_parameters(monkeypatch):
    import paper_1702_04683_amd as ac
    ac.load_library()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(43)
    k, Q = 600, 5
    where = planted_indices(rng, k)
    print(f"[max size] parameters: {N}", flush=True)
    theta = torch.empty(N, dtype=torch.float32, device=dev)
    gen = torch.Generator(device=dev).manual_seed(9)
    step = 1 << 28
    for a in range(0, N, step):
        theta[a:a + step].normal_(0.0, 0.05, generator=gen)
    touched_before = theta[torch.from_numpy(where).to(dev)].cpu().numpy()
    checksum_before = [int(theta[a:a + step].view(torch.int32).to(torch.int64).sum()) for a in range(0, N, step)]
    # every update takes a random 70 % of the planted coordinates
    ups_small, ups_big = [], []
    for q in range(Q):
        pick = np.sort(rng.choice(k, size=int(0.7 * k), replace=False))
        v = rng.standard_normal(pick.size).astype(np.float32)
        v[rng.random(pick.size) < 0.1] = 0.0
        off = np.array([0, pick.size], dtype=np.uint64)
        ups_small.append((off, pick.astype(np.uint32), v))
        ups_big.append((off, where[pick].astype(np.uint32), v))
    pulls = [0, 0, 1, 0, 3]
    small = [touched_before.copy()]
    ps = oracle.ParameterServer(small)
    for (o, i, v), p in zip(ups_small, pulls):
        ps.apply(o, i, v, p, 0.05)
    for plan in ("sweep", "scatter"):
        monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
        print(f"[max size] apply, plan {plan}", flush=True)
        theta[torch.from_numpy(where).to(dev)] = torch.from_numpy(touched_before).to(dev)
        us = [ac.Update.from_host(o, i, v, dev, pull_ts=p) for (o, i, v), p in zip(ups_big, pulls)]
        st = ac.State([theta])
        ws = torch.empty(max(256, ac.adacomp_apply_workspace([N], us, st)), dtype=torch.uint8, device=dev)
        ac.adacomp_apply([theta], st, us, 0.05, ws)
        torch.cuda.synchronize()
        got = theta[torch.from_numpy(where).to(dev)].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), small[0].view(np.uint32)), plan
        # everything else untouched: restore the touched ones and compare the piecewise bit sums
        theta[torch.from_numpy(where).to(dev)] = torch.from_numpy(touched_before).to(dev)
        after = [int(theta[a:a + step].view(torch.int32).to(torch.int64).sum()) for a in range(0, N, step)]
        assert after == checksum_before, plan
        del st, ws, us


def test_twenty_thousand_tensors(monkeypatch):
    """Many tensors in one call (descriptor tables of megabytes, one workgroup or more per tensor in every
    kernel): select through the one-workgroup path and through the streaming pipeline, then apply."""
    import paper_1702_04683_amd as ac
    from helpers import assert_update_equal, update_to_host
    ac.load_library()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(47)
    L = 20_000
    sizes = rng.integers(0, 300, size=L).tolist()
    sizes[5], sizes[L - 1] = 9000, 70_000
    flat = torch.randn(sum(sizes) + L, generator=torch.Generator(device=dev).manual_seed(3), device=dev)
    tensors, at = [], 0
    for n in sizes:
        tensors.append(flat[at:at + n])
        at += n + 1                                       # most tensors start off a 16-byte boundary
    host = [t.cpu().numpy() for t in tensors]
    want = oracle.select(host, 0.05)
    print("[many tensors] select, one workgroup per tensor", flush=True)
    u = gpu_select(ac, tensors, 0.05)
    assert_update_equal(update_to_host(u), want, "20000 tensors")
    print("[many tensors] select, streaming pipeline", flush=True)
    monkeypatch.setenv("ADACOMP_SELECT_SMALL", "0")
    assert_update_equal(update_to_host(gpu_select(ac, tensors, 0.05)), want, "20000 tensors, pipeline")
    monkeypatch.delenv("ADACOMP_SELECT_SMALL")
    print("[many tensors] apply", flush=True)
    theta_host = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    ref = [t.copy() for t in theta_host]
    ps = oracle.ParameterServer(ref)
    ups = []
    for q in range(3):
        g = [rng.standard_normal(n).astype(np.float32) for n in sizes]
        off, idx, val = oracle.select(g, 0.05)
        ps.apply(off, idx, val, 0, 0.1)
        ups.append(ac.Update.from_host(off, idx, val, dev, pull_ts=0))
    theta = [torch.from_numpy(t).to(dev) for t in theta_host]
    st = ac.State(theta)
    ws = torch.empty(max(256, ac.adacomp_apply_workspace(sizes, ups, st)), dtype=torch.uint8, device=dev)
    ac.adacomp_apply(theta, st, ups, 0.1, ws)
    torch.cuda.synchronize()
    for l in range(L):
        if sizes[l]:
            assert np.array_equal(theta[l].cpu().numpy().view(np.uint32), ref[l].view(np.uint32)), f"tensor {l}"


def test_keep_all_update_of_the_largest_tensor_applied_three_times():
    """An update with 2^32 - 1 entries (every parameter, rate 1) goes through the update-by-update plan
    with 64-bit entry numbers.  Applied three times with all pulls at time 0 the third application
    sees every parameter changed twice: theta - lr g - lr g - (lr / 2) g, each step rounded as eqs. 4-5
    say (keep-all selection = dense staleness-aware ASGD); torch evaluates that on the device."""
    import paper_1702_04683_amd as ac
    ac.load_library()
    dev = torch.device("cuda:0")
    step = 1 << 28
    g = torch.empty(N, dtype=torch.float32, device=dev)
    theta = torch.empty(N, dtype=torch.float32, device=dev)
    gen = torch.Generator(device=dev).manual_seed(13)
    for a in range(0, N, step):
        g[a:a + step].normal_(0.0, 1e-2, generator=gen)
        theta[a:a + step].normal_(0.0, 0.05, generator=gen)
    g[12345] = 0.0                                        # one exact zero: it never counts in eq. 3
    want = theta.clone()
    lr = 0.1
    for alpha in (lr, lr, np.float32(lr) / np.float32(2.0)):
        for a in range(0, N, step):
            want[a:a + step] -= g[a:a + step] * float(alpha)
    want[12345] = theta[12345]
    print("[max size] keep-all select", flush=True)
    u = gpu_select(ac, [g], 1.0)
    del g
    ups = [u.view(0, 1, pull_ts=0) for _ in range(3)]
    st = ac.State([theta])
    ws = torch.empty(max(256, ac.adacomp_apply_workspace([N], ups, st)), dtype=torch.uint8, device=dev)
    print(f"[max size] apply three times, workspace {ws.numel() / 1e9:.1f} GB", flush=True)
    ac.adacomp_apply([theta], st, ups, lr, ws)
    torch.cuda.synchronize()
    assert st.t == 3
    for a in range(0, N, step):
        assert torch.equal(theta[a:a + step].view(torch.int32), want[a:a + step].view(torch.int32)), f"piece at {a}"
