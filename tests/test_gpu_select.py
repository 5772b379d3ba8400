"""GPU parity: adacomp_select (HIP, through the C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import assert_update_equal, gpu_select, oracle_select_parallel, update_to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ac():
    import paper_1702_04683_amd as pkg
    pkg.load_library()
    return pkg


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda:0")


@pytest.fixture(autouse=True, params=["finish kernel", "multi-launch"])
def finish_mode(request, monkeypatch):
    """Every test of this file runs twice: with tensors finished by one workgroup each right after
    their filter (the default), and with that kernel switched off (check, gather, descent, count,
    scan and emit launches for every tensor).  Tests marked fused_only skip the second run."""
    if request.param == "multi-launch":
        if request.node.get_closest_marker("fused_only"):
            pytest.skip("run with the finish kernel only")
        monkeypatch.setenv("ADACOMP_SELECT_FUSED", "0")
    return request.param


def host(tensors):
    return [t.cpu().numpy() for t in tensors]


def check(ac, tensors, rate, k_override=None, what=""):
    print(f"[select] {what} rate={rate} k_override={'yes' if k_override else 'no'} "
          f"sizes={[t.numel() for t in tensors][:8]}...", flush=True)
    u = gpu_select(ac, tensors, rate, k_override)
    want = oracle.select(host(tensors), rate, k_override)
    assert_update_equal(update_to_host(u), want, what)
    return u


@pytest.mark.parametrize("rate", [0.01, 0.001, 0.1, 0.3, 1.0, 0.0])
def test_cnn_config(ac, dev, rate):
    """Config 'small CNN, one worker update': 8 tensors, heavy-tailed gradients."""
    g = workloads.gradient("cnn_select", 0, device=dev)
    check(ac, g, rate, what="cnn")


def test_cnn_repeatable_and_workspace_reuse(ac, dev):
    g = workloads.gradient("cnn_select", 1, device=dev)
    ws = torch.empty(ac.adacomp_select_workspace([t.numel() for t in g], 0.01), dtype=torch.uint8, device=dev)
    ws.fill_(0xAB)   # the workspace may hold anything on entry
    runs = [update_to_host(gpu_select(ac, g, 0.01, ws=ws)) for _ in range(3)]
    want = oracle.select(host(g), 0.01)
    for r in runs:
        assert_update_equal(r, want, "repeat")


@pytest.mark.fused_only
@pytest.mark.parametrize("rate", [0.001, 0.01, 0.1])
def test_mid_config(ac, dev, rate):
    """Config 'mid-size CNN': 57M Laplace gradients in 8 tensors."""
    g = workloads.gradient("mid", 0, device=dev)
    print(f"[select] mid rate={rate}", flush=True)
    u = gpu_select(ac, g, rate)
    want = oracle_select_parallel([[x] for x in host(g)], rate)
    off, idx, val = update_to_host(u)
    for l, (o, i, v) in enumerate(want):
        a, b = int(off[l]), int(off[l + 1])
        assert b - a == int(o[1])
        assert np.array_equal(idx[a:b], i), f"tensor {l} indices"
        assert np.array_equal(val[a:b].view(np.uint32), v.view(np.uint32)), f"tensor {l} values"


def test_adversarial_config_k1_rate1_rate0(ac, dev):
    """Config 'adversarial': 40 ragged tensors (two of one element), zeros, ties, +-duplicates,
    denormals; rates 0, 1/N (as k_override = 1 and as rate = 1/N on single tensors) and 100%."""
    g = workloads.gradient("adversarial", 0, device=dev)
    sizes = [t.numel() for t in g]
    assert sizes.count(1) >= 2 and all(n % 64 for n in sizes)
    L = len(g)
    # rate 0: nothing selected
    u = gpu_select(ac, g, 0.0)
    assert u.total == 0 and u.offsets == [0] * (L + 1)
    # k = 1 per tensor through k_override
    print("[select] adversarial k_override=1", flush=True)
    u = gpu_select(ac, g, 0.5, k_override=[1] * L)
    hg = host(g)
    want = oracle_select_parallel([[x] for x in hg], 0.5, k_override=[1])
    off, idx, val = update_to_host(u)
    for l, (o, i, v) in enumerate(want):
        assert idx[l] == i[0] and val[l:l + 1].view(np.uint32)[0] == v.view(np.uint32)[0], f"tensor {l}"
    # rate = 1/N on single tensors
    for l in (0, 3, 7, L - 2):
        check(ac, [g[l]], 1.0 / sizes[l], what=f"adversarial 1/N tensor {l}")
    # rate 1: identity; the oracle is consulted on the tensors below 1M entries, the definition on all
    print("[select] adversarial rate=1", flush=True)
    u = gpu_select(ac, g, 1.0)
    off, idx, val = update_to_host(u)
    assert off.tolist() == np.cumsum([0] + sizes).tolist()
    for l in range(L):
        a, b = int(off[l]), int(off[l + 1])
        assert np.array_equal(idx[a:b], np.arange(sizes[l], dtype=np.uint32))
        assert np.array_equal(val[a:b].view(np.uint32), hg[l].view(np.uint32))
        if sizes[l] < 1_000_000:
            i, v = oracle.select_layer(hg[l], sizes[l])
            assert np.array_equal(idx[a:b], i)


@pytest.mark.parametrize("rate", [0.01, 0.3, 0.0007, 0.6])
def test_adversarial_ties_at_threshold(ac, dev, rate):
    """Runs of identical magnitudes planted at the 1% and 30% quantiles: the threshold falls
    inside a run and the lower indices must win."""
    sizes = workloads.sizes_of("adversarial")
    pick = [l for l, n in enumerate(sizes) if n < 2_000_000][:10]
    g = [workloads.gradient_layer("adversarial", 0, l, sizes[l], dev) for l in pick]
    check(ac, g, rate, what="adversarial ties")


@pytest.mark.parametrize("n", [300_007, 70_001, 4_099])
def test_degenerate_tensors(ac, dev, n):
    """Constant magnitudes, all zeros, strictly monotone ramps, two levels, special values: at a size
    that goes through the streaming pipeline and at sizes one workgroup selects on its own."""
    ones = torch.ones(n, device=dev)
    ones[::3] = -1.0
    zeros = torch.zeros(n, device=dev)
    zeros[1::2] = -0.0
    ramp = torch.arange(n, device=dev, dtype=torch.float32)
    two_level = torch.where(torch.arange(n, device=dev) % 7 == 0, 2.0, 1.0)
    one = torch.tensor([-3.5], device=dev)
    empty = torch.empty(0, device=dev)
    tiny = torch.tensor([1e-45, -1e-45, 0.0, 3e-39, -3e-39], device=dev)
    special = torch.tensor([1.0, float("-inf"), 3e38, float("nan"), 0.0, float("inf"), 1e-45], device=dev)
    tensors = [ones, zeros, ramp, two_level, one, empty, tiny, special, ramp.flip(0).contiguous()]
    for rate in (0.01, 0.2, 0.5, 0.9):
        check(ac, tensors, rate, what="degenerate")
    check(ac, tensors, 0.5, k_override=[1, 2, 3, n - 1, 1, 0, 4, 3, n // 2], what="degenerate k_override")


def test_clustered_large_values_overflow_their_regions(ac, dev):
    """All large entries sit in one contiguous stretch, so wave segments there overflow their
    candidate regions (the gather filters those segments again) while a strided sample misjudges
    the threshold (too few candidates: the tensor itself is read instead): the result must stay exact."""
    n = 2_000_003
    gen = torch.Generator(device=dev).manual_seed(11)
    g = torch.randn(n, generator=gen, device=dev) * 1e-3
    g[700_001:700_001 + 30_000] = torch.randn(30_000, generator=gen, device=dev)
    h = torch.randn(n, generator=gen, device=dev) * 1e-3
    h[::8192] *= 1000.0      # large entries only where a strided sample rarely looks
    for rate in (0.01, 0.002):
        check(ac, [g, h], rate, what="clustered")
    # every fourth segment dense with large entries, ragged end inside such a segment, unaligned start
    n = 8192 * 41 + 1234
    base = torch.randn(n + 1, generator=gen, device=dev) * 1e-3
    for s0 in range(0, n, 4 * 8192):
        base[s0 + 100:s0 + 8000] = torch.randn(7900, generator=gen, device=dev)
    base[8192 * 40:] = torch.randn(base.numel() - 8192 * 40, generator=gen, device=dev) * 3.0
    for rate in (0.02, 0.1, 0.2):
        check(ac, [base[:n], base[1:]], rate, what="overflowing segments")


def test_unaligned_tensor_views(ac, dev):
    """Tensors that start 4, 8 or 12 bytes past a 16-byte boundary: only the elements in front of the
    first boundary are read singly."""
    base = workloads.gradient_layer("cnn_select", 2, 4, 3211264, dev)
    views = [base[1:1_000_000], base[2:777_779], base[3:50_001], base[5:6]]
    assert all(v.data_ptr() % 16 != 0 for v in views)
    check(ac, [v for v in views], 0.01, what="unaligned")
    check(ac, [v for v in views], 0.4, what="unaligned dense")


def test_views_at_any_offset_with_sizes_around_segment_borders(ac, dev):
    """The borders between a tensor's 8192-element segments lie on 128-byte boundaries of its memory:
    views that start 1 to 33 elements into a buffer, with sizes that leave the last segment empty,
    nearly empty or full, selected by the filter pipeline (too large for the one-workgroup kernel)."""
    base = workloads.gradient_layer("cnn_select", 2, 4, 3211264, dev)
    whole = 40 * 8192
    cases = [(1, 0), (1, 1), (3, 2), (3, 3), (4, 28), (8, 31), (31, 32), (33, 33), (2, 8191), (31, 1), (33, 30), (5, 8160)]
    views = [base[o:o + whole + d] for o, d in cases]
    assert all(v.numel() > (1 << 18) for v in views)
    check(ac, views, 0.005, what="views around segment borders")
    check(ac, views, 0.08, what="views around segment borders, dense")


def test_negation_and_scaling_invariance_on_gpu(ac, dev):
    g = workloads.gradient("cnn_select", 2, device=dev)
    a = update_to_host(gpu_select(ac, g, 0.01))
    b = update_to_host(gpu_select(ac, [-x for x in g], 0.01))
    c = update_to_host(gpu_select(ac, [x * 4.0 for x in g], 0.01))
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], -b[2])
    assert np.array_equal(a[1], c[1]) and np.array_equal(a[2] * np.float32(4.0), c[2])


@pytest.mark.fused_only
def test_flat_config_full_size(ac, dev):
    """The roofline configuration in the launch shape bench.py times: 100 tensors of 10M entries,
    rate 0.5%, one call.  The oracle checks sampled tensors entry by entry; on all 100 the
    properties that define a correct selection are evaluated with torch on the device."""
    cfg, rate = "flat", 0.005
    sizes = workloads.sizes_of(cfg)
    g = workloads.gradient(cfg, 0, device=dev)
    print("[select] flat full size, 1e9 elements", flush=True)
    u = gpu_select(ac, g, rate)
    k = ac.adacomp_count(sizes[0], rate)
    assert u.offsets == [k * l for l in range(len(sizes) + 1)] and k == 50_000
    for l in (0, 37, 99):
        i, v = oracle.select_layer(g[l].cpu().numpy(), k)
        assert np.array_equal(u.idx[l * k:(l + 1) * k].cpu().numpy().view(np.uint32), i), f"tensor {l}"
        assert np.array_equal(u.val[l * k:(l + 1) * k].cpu().numpy().view(np.uint32), v.view(np.uint32))
    for l in range(len(sizes)):
        idx = u.idx[l * k:(l + 1) * k].to(torch.int64)
        val = u.val[l * k:(l + 1) * k]
        assert bool((idx[1:] > idx[:-1]).all()) and int(idx[-1]) < sizes[l] and int(idx[0]) >= 0
        assert torch.equal(g[l][idx].view(torch.int32), val.view(torch.int32))
        key = g[l].view(torch.int32) & 0x7FFFFFFF
        T = int((val.view(torch.int32) & 0x7FFFFFFF).min())
        n_gt, n_ge = int((key > T).sum()), int((key >= T).sum())
        assert n_gt < k <= n_ge, f"tensor {l}: threshold is not the k-th largest magnitude"
        sel_key = key[idx]
        assert int((sel_key > T).sum()) == n_gt, f"tensor {l}: an entry above the threshold is missing"
        eq_all = torch.nonzero(key == T).flatten()[:k - n_gt]
        assert torch.equal(idx[sel_key == T], eq_all), f"tensor {l}: tie rule"


def test_whole_model_selection_is_select_on_one_tensor(ac, dev):
    """The competitors' selection (Sec. 4 'Selection method': the largest entries across the whole
    model) is the same call on the model passed as a single tensor; it differs from the per-tensor rule."""
    g = workloads.gradient("cnn_select", 3, device=dev)
    flat = torch.cat([x.view(-1) for x in g])
    u = check(ac, [flat], 0.01, what="whole model")
    per = gpu_select(ac, g, 0.01)
    base = np.cumsum([0] + [x.numel() for x in g])
    per_global = np.concatenate([per.idx[per.offsets[l]:per.offsets[l + 1]].cpu().numpy().view(np.uint32).astype(np.int64) + base[l]
                                 for l in range(len(g))])
    whole = u.idx[:u.total].cpu().numpy().view(np.uint32).astype(np.int64)
    assert whole.size != per_global.size or not np.array_equal(whole, per_global)


def test_small_tensors_through_the_streaming_pipeline(ac, dev, monkeypatch):
    """With the one-workgroup path switched off, small tensors take the pipeline built for large
    ones; both must give the oracle's selection."""
    monkeypatch.setenv("ADACOMP_SELECT_SMALL", "0")
    g = workloads.gradient("paper_cnn", 1, device=dev)
    for rate in (0.1, 0.01, 0.0001):
        check(ac, g, rate, what="paper_cnn, pipeline")
    sizes = workloads.sizes_of("adversarial")
    pick = [l for l, n in enumerate(sizes) if n < 300_000][:6]
    check(ac, [workloads.gradient_layer("adversarial", 0, l, sizes[l], dev) for l in pick], 0.02, what="adversarial, pipeline")
    monkeypatch.delenv("ADACOMP_SELECT_SMALL")
    check(ac, g, 0.01, what="paper_cnn, one workgroup per tensor")


def test_many_small_tensors_ties_and_unaligned(ac, dev):
    """600 small tensors of ragged sizes cut out of one buffer (most start off a 16-byte boundary),
    values quantised to a few levels so that every threshold falls inside a run of equal magnitudes."""
    gen = torch.Generator(device=dev).manual_seed(23)
    base = (torch.randn(3_000_000, generator=gen, device=dev) * 4).round() / 4       # multiples of 0.25
    sizes = torch.randint(1, 9000, (600,), generator=torch.Generator().manual_seed(5)).tolist()
    sizes[17], sizes[18] = 262_144, 262_143
    tensors, at = [], 1
    for n in sizes:
        tensors.append(base[at:at + n])
        at += n + 1
    for rate in (0.003, 0.05, 0.5):
        check(ac, tensors, rate, what="many small")


def test_small_tensor_with_clustered_large_values(ac, dev):
    """One workgroup per tensor: all large entries sit in a stretch that belongs to one or two waves,
    whose candidate slots in LDS overflow; the workgroup must then finish from the tensor itself."""
    gen = torch.Generator(device=dev).manual_seed(31)
    n = 200_003
    g = torch.randn(n, generator=gen, device=dev) * 1e-3
    g[60_001:60_001 + 3_000] = torch.randn(3_000, generator=gen, device=dev)
    h = torch.randn(n, generator=gen, device=dev) * 1e-3
    h[::4096] *= 1000.0
    for rate in (0.01, 0.002, 0.0001):
        check(ac, [g, h, g[1:70_000]], rate, what="small, clustered")


def test_groups_of_tensors_reuse_the_candidate_regions(ac, dev, monkeypatch):
    """With the region size forced down to 1 MB the 8 tensors of the mid-size configuration split into
    several groups that reuse one set of candidate regions (a tensor larger than the limit forms a
    group of its own); the selection must not change."""
    g = workloads.gradient("cnn_select", 5, device=dev) + [workloads.gradient_layer("mid", 0, 2, 884736, dev),
                                                           workloads.gradient_layer("mid", 0, 3, 663552, dev)]
    want = [update_to_host(gpu_select(ac, g, r)) for r in (0.01, 0.002)]
    for mb in ("1", "3", "0"):
        monkeypatch.setenv("ADACOMP_SELECT_GROUP_MB", mb)
        for r, w in zip((0.01, 0.002), want):
            assert_update_equal(update_to_host(gpu_select(ac, g, r)), w, f"group size {mb} MB")
    monkeypatch.delenv("ADACOMP_SELECT_GROUP_MB")
    check(ac, g, 0.01, what="groups, default size")


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_rates_and_counts(ac, dev, seed):
    """Seeded random mixes of tensor sizes (1 .. 600K, so both the one-workgroup path and the streaming
    pipeline run in one call), value distributions, rates and per-tensor counts, including 0 and n."""
    rng = np.random.default_rng(1000 + seed)
    gen = torch.Generator(device=dev).manual_seed(2000 + seed)
    L = int(rng.integers(1, 24))
    sizes = [int(rng.choice([1, 2, 63, 64, 65, 255, 257, 4096, int(rng.integers(1, 600_000)), int(rng.integers(1, 40_000))]))
             for _ in range(L)]
    tensors = []
    for n in sizes:
        kind = int(rng.integers(0, 4))
        x = torch.randn(n, generator=gen, device=dev)
        if kind == 1:
            x = (x * 3).round() / 3                      # few levels: ties everywhere
        elif kind == 2:
            x = x * (torch.rand(n, generator=gen, device=dev) < 0.1)      # 90 % zeros
        elif kind == 3:
            x = x.abs().pow(8.0) * 1e-20                 # wide dynamic range, denormals
        tensors.append(x.contiguous())
    rate = float(rng.choice([0.0003, 0.004, 0.03, 0.2, 0.7]))
    check(ac, tensors, rate, what=f"random {seed}")
    ks = [int(rng.choice([0, 1, n, n // 2, min(n, 7), int(rng.integers(0, n + 1))])) for n in sizes]
    check(ac, tensors, rate, k_override=ks, what=f"random {seed}, counts given")


@pytest.mark.parametrize("small", ["0", "1"])
def test_sizes_around_every_internal_boundary(ac, dev, monkeypatch, small):
    """Tensor sizes at and next to the sizes the kernels are built around (4-element loads, 256-element
    pieces, the 512 elements up to which a tensor is ranked by all-pairs comparison, 8192-element wave
    segments, 2048-candidate chunks, the 2^18 limit of the one-workgroup path), each with k = 1, k = n - 1 and two rates, through the pipeline and through the one-workgroup path."""
    monkeypatch.setenv("ADACOMP_SELECT_SMALL", small)
    gen = torch.Generator(device=dev).manual_seed(77)
    sizes = [1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2048, 2049, 8191, 8192, 8193, 16383, 16384, 16385,
             65535, 65537, 262143, 262144, 262145, 262144 + 8192, 524287, 524288, 524289]
    tensors = [(torch.randn(n, generator=gen, device=dev) * 7).round() / 7 for n in sizes]    # ties are common
    for rate in (0.01, 0.2):
        check(ac, tensors, rate, what=f"boundary sizes, small={small}")
    check(ac, tensors, 0.5, k_override=[1] * len(sizes), what="boundary sizes, k = 1")
    check(ac, tensors, 0.5, k_override=[max(n - 1, 0) for n in sizes], what="boundary sizes, k = n - 1")


def test_counts_around_the_switch_between_filter_and_direct_descent(ac, dev):
    """k just below, at and above n / 8 (above it the descent reads the tensor directly), a quarter, all
    but one; on Gaussian data, on a tensor of NaNs with different payloads, and on one of infinities."""
    gen = torch.Generator(device=dev).manual_seed(91)
    n = 1_000_003
    x = torch.randn(n, generator=gen, device=dev)
    payload = torch.randint(0, 1 << 22, (n,), generator=gen, device=dev, dtype=torch.int32)
    nans = (payload | 0x7FC00000 | (torch.randint(0, 2, (n,), generator=gen, device=dev, dtype=torch.int32) << 31)).view(torch.float32)
    infs = torch.where(torch.rand(n, generator=gen, device=dev) < 0.5, float("inf"), float("-inf")).to(torch.float32)
    for k in (n // 8 - 1, n // 8, n // 8 + 1, n // 4, n - 1, 3):
        check(ac, [x, nans.contiguous(), infs.contiguous()], 0.5, k_override=[k, k, k], what=f"k = {k}")


def test_two_streams_at_once(ac, dev):
    """The library keeps no state between calls: two selects enqueued on two streams, each with its own
    workspace and outputs, run side by side and both give the oracle's result."""
    g = [workloads.gradient("cnn_select", 7, device=dev), workloads.gradient("cnn_select", 8, device=dev)]
    sizes = [t.numel() for t in g[0]]
    streams = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]
    cap = sum(ac.adacomp_count(n, 0.01) for n in sizes)
    outs = [ac.Update(len(sizes), cap, dev) for _ in range(2)]
    wss = [torch.empty(ac.adacomp_select_workspace(sizes, 0.01), dtype=torch.uint8, device=dev) for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(3):
        for i in range(2):
            ac.adacomp_select(g[i], 0.01, outs[i], wss[i], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        assert_update_equal(update_to_host(outs[i]), oracle.select(host(g[i]), 0.01), f"stream {i}")


def _sampled_pieces(n):
    """The 1 KB pieces (256 elements) of an n-element tensor that the sample histogram reads: a
    white-box copy of the library's choice, so that a test can bias exactly what the sample sees."""
    npieces = (n + 255) // 256
    stride = 64
    while stride > 1 and npieces // stride < 512:
        stride >>= 1
    slots = (npieces + stride - 1) // stride
    p = np.arange(slots, dtype=np.uint64)
    jit = ((p * 2654435761) & 0xffffffff) >> 16 & (stride - 1)
    return np.minimum(p * stride + jit, npieces - 1), stride


@pytest.mark.fused_only
@pytest.mark.parametrize("bias,what", [(1.12, "the reserve threshold takes over"), (1.6, "the tensor itself is read"),
                                       (0.8, "more candidates than needed")])
def test_sample_that_misjudges_the_threshold(ac, dev, bias, what):
    """Everything the sample reads is scaled by `bias`, nothing else: above 1 the sampled threshold
    is too high and the filter finds fewer than k candidates (slightly: the lower threshold it
    counted against has enough; grossly: the descent reads the tensor itself), below 1 too low.
    Row-scaled gradients (large entries clustered in rows) produce the same situations by chance."""
    n = 4_000_037
    gen = torch.Generator(device=dev).manual_seed(77)
    g = torch.randn(n, generator=gen, device=dev) * 1e-3
    pieces, stride = _sampled_pieces(n)
    assert stride > 1
    idx = (torch.from_numpy(pieces.astype(np.int64)).to(dev)[:, None] * 256 + torch.arange(256, device=dev)[None, :]).flatten()
    idx = idx[idx < n]
    g[idx] *= bias
    check(ac, [g], 0.005, what=what)
    rows = workloads.gradient("mid", 3, device=dev, layers=[5, 6], row_spread=1.5)
    check(ac, rows, 0.005, what="row-scaled gradient")


def test_tiny_tensors_special_values_and_ties(ac, dev):
    """Tensors of at most 512 elements are ranked by all-pairs comparison in one workgroup: ties
    (lower index first), signed zeros, denormals, infinities and NaNs with payloads must come
    out as the oracle orders them, at every count from 0 to n."""
    gen = torch.Generator(device=dev).manual_seed(123)
    n = 300
    x = (torch.randn(n, generator=gen, device=dev) * 3).round() / 3          # many equal magnitudes, +x and -x
    bits = x.view(torch.int32).clone()
    bits[5] = 0x7FC00001; bits[6] = -0x00400000 + 7; bits[7] = 0x7F800000; bits[8] = -0x00800000   # NaNs, +inf, -inf
    bits[9] = 1; bits[10] = -0x7FFFFFFF; bits[11] = 0; bits[12] = -0x80000000                     # denormals, +0, -0
    special = bits.view(torch.float32).contiguous()
    zeros = torch.zeros(37, device=dev)
    zeros[::2] = -0.0
    one = torch.tensor([-2.5], device=dev)
    for k in (0, 1, 2, 13, 150, 299, 300):
        check(ac, [special, zeros, one, x[:64].contiguous(), x[:65].contiguous()], 0.5,
              k_override=[k, min(k, 37), min(k, 1), min(k, 64), min(k, 65)], what=f"tiny tensors, k = {k}")


@pytest.mark.parametrize("group_mb", ["2", None])
def test_row_scaled_gradients_in_many_groups(ac, dev, monkeypatch, group_mb):
    """Tensors of 300K to 3M elements whose rows are scaled log-normally (large entries cluster),
    in one call, with the candidate regions forced down to 2 MB (a dozen groups that reuse them)
    and at their default size: regions that overflow, thresholds that fall short and tensors that
    are read directly all occur side by side; every tensor must come out as the oracle orders it."""
    if group_mb:
        monkeypatch.setenv("ADACOMP_SELECT_GROUP_MB", group_mb)
    gen = torch.Generator(device=dev).manual_seed(31)
    rng = np.random.default_rng(31)
    tensors = []
    for i in range(10):
        n = int(rng.integers(300_000, 3_000_000))
        row = int(rng.choice([256, 1000, 4096]))
        x = torch.randn(n, generator=gen, device=dev) * 1e-3
        scale = torch.exp(float(rng.choice([0.7, 1.5, 2.5])) * torch.randn((n + row - 1) // row, generator=gen, device=dev))
        tensors.append(x * scale.repeat_interleave(row)[:n])
    for rate in (0.002, 0.02, 0.1):
        check(ac, tensors, rate, what=f"row-scaled, groups of {group_mb} MB, rate {rate}")


def test_finish_kernel_hands_back_what_it_cannot_resolve(ac, dev):
    """One workgroup finishes a tensor only if the threshold lies less than a factor two above the
    filter threshold and few regions overflowed; otherwise the tensor goes back to the launches
    that work for anything.  Forced here: (a) values whose k-th largest lies far above the
    threshold the sample suggests (every sampled piece is small, the large values sit elsewhere);
    (b) ties: thousands of equal magnitudes at the threshold, more than a wave can keep in LDS,
    so that its counts come from one more pass; (c) many overflowing regions next to tensors that
    are finished normally, in one call, several groups."""
    gen = torch.Generator(device=dev).manual_seed(2718)
    n = 3_000_001
    a = torch.randn(n, generator=gen, device=dev) * 1e-3
    a[5::97] = torch.randn(a[5::97].numel(), generator=gen, device=dev) * 50.0      # 1% of the entries, 4 orders larger
    b = torch.randn(n, generator=gen, device=dev) * 1e-3
    top = torch.topk(b.abs(), 40_000).values[-1]
    b[1_000_000:1_030_000] = torch.where(torch.rand(30_000, generator=gen, device=dev) < 0.5, -top, top)   # 30,000 ties in one stretch
    c = torch.randn(n, generator=gen, device=dev) * 1e-3
    for s0 in range(0, n - 8192, 5 * 8192):
        c[s0:s0 + 6000] = torch.randn(6000, generator=gen, device=dev)
    d = torch.randn(1_500_000, generator=gen, device=dev)
    for rate in (0.002, 0.012, 0.05):
        check(ac, [a, b, c, d], rate, what="finish kernel, special cases")
    check(ac, [b, d], 0.5, k_override=[40_000 + 7, 3], what="finish kernel, tie quota")


def test_finish_kernel_sizes_around_its_limits(ac, dev):
    """Tensors of 4095, 4096 and 4097 segments (the last is not finished by one workgroup and takes
    the gather of its group), a single segment, a ragged last segment of one element."""
    gen = torch.Generator(device=dev).manual_seed(31415)
    sizes = [8192 * 4095 + 1, 8192 * 4096, 8192 * 4096 + 1, 300_000, 8192 * 40 + 1]
    g = [torch.randn(n, generator=gen, device=dev) * (10.0 ** -(i % 3)) for i, n in enumerate(sizes)]
    u = gpu_select(ac, g, 0.003)
    want = oracle_select_parallel([[t.cpu().numpy()] for t in g], 0.003, threads=5)
    for l, (o, i, v) in enumerate(want):
        a, k = u.offsets[l], int(o[1])
        assert u.offsets[l + 1] - a == k
        assert np.array_equal(u.idx[a:a + k].cpu().numpy().view(np.uint32), i), f"tensor {l}"
        assert np.array_equal(u.val[a:a + k].cpu().numpy().view(np.uint32), v.view(np.uint32)), f"tensor {l}"
