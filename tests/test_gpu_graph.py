"""One step of the path (select over a batch of worker gradients, then the queue apply) recorded in a
HIP graph and replayed: every replay, with eager work and synchronisations in between, must give what
the oracle gives for the gradients that are in the buffers at that moment.

What a recorded step fixes: buffer addresses, sizes, rate, learning rate, and every update's pull
time RELATIVE to the start of the queue (so all pulls must lie inside the queue, history off).  The
host-side timestamp of the state is advanced by the recording call only; a caller who replays adds Q
per replay himself if he needs it.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import assert_update_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("plan", ["sweep", "scatter"])
def test_recorded_step_replays_exactly(plan, monkeypatch):
    import paper_1702_04683_amd as ac
    ac.load_library()
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", plan)
    dev = torch.device("cuda:0")
    cfg, rate, lr, Q = "cnn_select", 0.01, 0.05, 4
    sizes = workloads.sizes_of(cfg)
    L = len(sizes)
    rel_pull = [0, 0, 1, 1]                      # update q was pulled after rel_pull[q] updates of its queue
    grads = [[torch.zeros(n, device=dev) for n in sizes] for _ in range(Q)]       # static input buffers
    theta = workloads.theta0(cfg, device=dev)
    theta_ref = [t.cpu().numpy().copy() for t in theta]
    ps = oracle.ParameterServer(theta_ref)
    all_tensors = [t for g in grads for t in g]
    cap = sum(ac.adacomp_count(n, rate) for n in sizes)
    big = ac.Update(L * Q, cap * Q, dev)
    sel_ws = torch.empty(ac.adacomp_select_workspace(sizes * Q, rate), dtype=torch.uint8, device=dev)
    state = ac.State(theta)

    def load(r):
        fresh = [workloads.gradient(cfg, 100 + r * Q + q, device=dev) for q in range(Q)]
        for q in range(Q):
            for dst, src in zip(grads[q], fresh[q]):
                dst.copy_(src)
        return [[t.cpu().numpy() for t in g] for g in fresh]

    def step():
        ac.adacomp_select(all_tensors, rate, big, sel_ws)
        for q in range(Q):
            views[q].pull_ts = state.t + rel_pull[q]
        ac.adacomp_apply(theta, state, views, lr, app_ws)

    # sizes of the selection do not depend on the data: fill layer_off once, make the 16 views (they
    # upload their offset tables, which a recording must not contain) and size the apply workspace
    ac.adacomp_select(all_tensors, rate, big, sel_ws)
    views = [big.view(q * L, (q + 1) * L, pull_ts=rel_pull[q]) for q in range(Q)]
    app_ws = torch.empty(max(256, ac.adacomp_apply_workspace(sizes, views)), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def expect(host_grads, r):
        for q in range(Q):
            off, idx, val = oracle.select(host_grads[q], rate)
            ps.apply(off, idx, val, r * Q + rel_pull[q], lr)
            yield off, idx, val

    def verify(host_grads, r, what):
        torch.cuda.synchronize()
        idx_all = big.idx.cpu().numpy().view(np.uint32)
        val_all = big.val.cpu().numpy()
        for q, want in enumerate(expect(host_grads, r)):
            a = q * cap
            got = (want[0], idx_all[a:a + cap], val_all[a:a + cap])
            assert big.offsets[q * L:(q + 1) * L + 1] == [a + int(o) for o in want[0]]
            assert_update_equal(got, want, f"{what}, update {q}")
        for l in range(L):
            assert np.array_equal(theta[l].cpu().numpy().view(np.uint32), theta_ref[l].view(np.uint32)), \
                f"{what}: parameters of tensor {l}"

    # replay 0 is the eager run (also the warm-up that recording wants)
    print(f"[graph] plan={plan} eager step", flush=True)
    hg = load(0)
    step()
    verify(hg, 0, "eager")

    print("[graph] recording", flush=True)
    graph = torch.cuda.CUDAGraph()
    hg = load(1)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()                                   # recorded, not run
    for r in range(1, 5):
        if r > 1:
            hg = load(r)
        junk = torch.randn(1 << 20, device=dev).sum()      # the program's own eager work between replays
        torch.cuda.synchronize()
        print(f"[graph] replay {r}", flush=True)
        graph.replay()
        verify(hg, r, f"replay {r}")
        assert torch.isfinite(junk)
