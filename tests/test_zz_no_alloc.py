"""GPU: adacomp_select_noalloc (the library's built-in scratch buffer instead of a caller's
workspace) gives what adacomp_select gives, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

import workloads
from helpers import gpu_select, update_to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ac():
    import paper_1702_04683_amd as ac
    ac.load_library()
    return ac


def _noalloc(ac, tensors, rate, k_override=None):
    dev = tensors[0].device
    sizes = [t.numel() for t in tensors]
    ks = k_override if k_override is not None else [ac.adacomp_count(n, rate) for n in sizes]
    u = ac.Update(len(tensors), sum(ks), dev)
    u.idx.fill_(-1)
    u.val.fill_(float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
    ac.adacomp_select_noalloc(tensors, rate, u, k_override=k_override)
    assert torch.cuda.memory_stats(dev)["allocation.all.allocated"] == before
    torch.cuda.synchronize()
    return u


def _same(a, b):
    off_a, idx_a, val_a = update_to_host(a)
    off_b, idx_b, val_b = update_to_host(b)
    assert off_a.tolist() == off_b.tolist()
    assert np.array_equal(idx_a, idx_b), "indices differ"
    assert np.array_equal(val_a.view(np.uint32), val_b.view(np.uint32)), "values differ"


def test_two_calls_in_a_row_second_one_smaller(ac):
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # first: the small CNN (one 3.2M tensor through the streaming pipeline, the rest in one workgroup each)
    big = workloads.gradient("cnn_select", 0, device=dev)
    assert ac.adacomp_select_workspace([t.numel() for t in big], 0.01) <= ac.SELECT_NOALLOC_SCRATCH_BYTES
    print("noalloc: cnn_select sizes", [t.numel() for t in big], flush=True)
    _same(_noalloc(ac, big, 0.01), gpu_select(ac, big, 0.01))
    # second, smaller: ragged tensors of the same pipeline (fewer segments, other thresholds), ties included
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    small = [torch.randn(n, generator=g, device=dev) * 1e-3 for n in (700_001, 300_007, 129, 1)]
    small[1][1000:3000] = 0.5
    print("noalloc: second call sizes", [t.numel() for t in small], flush=True)
    _same(_noalloc(ac, small, 0.003), gpu_select(ac, small, 0.003))
    # and the first input once more: what the second call left in the buffer does not matter
    _same(_noalloc(ac, big, 0.01), gpu_select(ac, big, 0.01))


def test_refused_beyond_the_limit(ac):
    dev = torch.device("cuda:0")
    t = [torch.zeros(40_000_000, device=dev)]
    u = ac.Update(1, 400_000, dev)
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_select_noalloc(t, 0.01, u)
    assert e.value.code == -13
