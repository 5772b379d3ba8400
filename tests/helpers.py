"""Shared test plumbing: run the HIP path through the C ABI binding and bring results to the host."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle


def gpu_select(ac, tensors, rate, k_override=None, pull_ts=0, ws=None):
    dev = tensors[0].device if tensors else torch.device("cuda:0")
    sizes = [t.numel() for t in tensors]
    need = ac.adacomp_select_workspace(sizes, rate, k_override)
    if ws is None or ws.numel() < need:
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
    ks = k_override if k_override is not None else [ac.adacomp_count(n, rate) for n in sizes]
    u = ac.Update(len(tensors), sum(ks), dev, pull_ts=pull_ts)
    # poison the outputs so that an entry the kernels fail to write is seen
    u.idx.fill_(-1)
    u.val.fill_(float("nan"))
    ac.adacomp_select(tensors, rate, u, ws, k_override=k_override)
    torch.cuda.synchronize()
    return u


def update_to_host(u):
    total = u.total
    off_dev = u.layer_off_dev.cpu().numpy().astype(np.uint64)
    assert off_dev.tolist() == u.offsets, "device and host copies of layer_off differ"
    idx = u.idx[:total].cpu().numpy().view(np.uint32)
    val = u.val[:total].cpu().numpy()
    return np.array(u.offsets, dtype=np.uint64), idx, val


def assert_update_equal(got, want, what=""):
    off_g, idx_g, val_g = got
    off_w, idx_w, val_w = want
    assert off_g.tolist() == off_w.tolist(), f"{what}: layer offsets differ"
    for l in range(len(off_w) - 1):
        a, b = int(off_w[l]), int(off_w[l + 1])
        if not np.array_equal(idx_g[a:b], idx_w[a:b]):
            bad = np.flatnonzero(idx_g[a:b] != idx_w[a:b])
            raise AssertionError(f"{what}: tensor {l}: {bad.size} of {b - a} indices differ, first at entry "
                                 f"{bad[0]}: got {idx_g[a + bad[0]]} want {idx_w[a + bad[0]]}")
        assert np.array_equal(val_g[a:b].view(np.uint32), val_w[a:b].view(np.uint32)), \
            f"{what}: tensor {l}: values differ"


def oracle_select_parallel(grad_lists, rate, k_override=None, threads=8):
    """oracle.select for several gradients at once (the C call releases the GIL)."""
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda g: oracle.select(g, rate, k_override), grad_lists))


def rel_err(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.maximum(np.maximum(np.abs(a), np.abs(b)), 1e-30)
    return float(np.max(np.abs(a - b) / den)) if a.size else 0.0
