"""Seeded synthetic inputs for the AdaComp hot path: gradients, initial parameters
and staleness draws shaped like the benchmark configurations.

This module holds NO arithmetic of the method (no selection, no staleness or
learning-rate formula).  It is the only code that the CPU oracle's tests and the
HIP path's tests/bench have in common.  Tensors are produced with torch on the
device asked for (CPU, or the GPU and then copied to the host for the oracle), one
torch.Generator per (configuration, update, tensor), so any subset of tensors can
be regenerated on its own.  "N(0, x)" is read as standard deviation x.
"""
import torch

# tensor sizes ---------------------------------------------------------------
SIZES = {
    # small MNIST-style CNN: conv 5x5x1x32 + b, conv 5x5x32x64 + b, FC 3136x1024 + b, FC 1024x10 + b
    "cnn": [800, 32, 51200, 64, 3211264, 1024, 10240, 10],
    # AlexNet-like: 35K, 307K, 885K, 663K, 442K, 37.7M, 16.8M, 41K
    "mid": [34848, 307200, 884736, 663552, 442368, 37748736, 16777216, 40960],
    # 1B-element stream, 100 tensors of 10M
    "flat": [10_000_000] * 100,
    # a two-conv, two-FC MNIST network with the parameter count of Sec. 5.1 (211,690): conv 3x3x1x32 + b,
    # conv 3x3x32x32 + b, FC 1568x128 + b, FC 128x10 + b (the text gives the total only; these shapes sum to it)
    "paper_cnn": [288, 32, 9216, 32, 200704, 128, 1280, 10],
}

CONFIGS = {
    "cnn_select": dict(sizes="cnn", dist="heavy_tail", rates=[0.01], Q=1, seed=1000),
    "cnn_apply": dict(sizes="cnn", dist="heavy_tail", rates=[0.01], Q=200, max_staleness=200,
                      lr=0.01, seed=2000),
    "mid": dict(sizes="mid", dist="laplace", rates=[0.001, 0.01, 0.1], Q=64, max_staleness=64,
                lr=0.01, seed=3000),
    "flat": dict(sizes="flat", dist="mixture", rates=[0.005], Q=16, max_staleness=16,
                 lr=0.01, seed=4000),
    # the network size and worker count of Sec. 5.1 with the compression ratios of Sec. 5.3 and 5.4
    "paper_cnn": dict(sizes="paper_cnn", dist="heavy_tail", rates=[0.1, 0.01, 0.001, 0.0001], Q=200,
                      max_staleness=200, lr=0.01, seed=6000),
    "adversarial": dict(sizes="adversarial", dist="adversarial", rates=[0.0, None, 1.0],
                        lr=0.01, seed=5000),
}


def _gen(device, *seed_parts):
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for p in seed_parts:
        s = (s * 6364136223846793005 + int(p) + 1442695040888963407) % (1 << 63)
    g.manual_seed(s)
    return g


def adversarial_sizes(seed=5000, count=40, max_n=5_000_000):
    """`count` tensor sizes in [1, max_n], none a multiple of 64, two equal to 1."""
    g = _gen("cpu", seed, 17)
    out = []
    while len(out) < count:
        n = int(torch.randint(1, max_n + 1, (1,), generator=g).item())
        if n % 64 != 0:
            out.append(n)
    out[3] = 1
    out[count - 2] = 1
    return out


def sizes_of(cfg):
    c = CONFIGS[cfg]
    if c["sizes"] == "adversarial":
        return adversarial_sizes(c["seed"])
    return list(SIZES[c["sizes"]])


def _normal(n, std, gen, device):
    return torch.randn(n, generator=gen, device=device, dtype=torch.float32) * std


def heavy_tail(n, gen, device):
    """N(0, 1e-3) with an independent 1% of the entries scaled by 100."""
    x = _normal(n, 1e-3, gen, device)
    boost = torch.rand(n, generator=gen, device=device) < 0.01
    return torch.where(boost, x * 100.0, x)


def laplace(n, gen, device, b=1e-4):
    u = torch.rand(n, generator=gen, device=device, dtype=torch.float32) - 0.5
    return -b * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.49999997))


def mixture(n, gen, device):
    """95% N(0, 1e-5) + 5% N(0, 1e-2)."""
    x = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
    wide = torch.rand(n, generator=gen, device=device) < 0.05
    return x * torch.where(wide, 1e-2, 1e-5).to(torch.float32)


def adversarial(n, gen, device, tie_levels=(0.0, 0.01, 0.3), run=1000):
    """Edge-case tensor: 50% exact zeros of either sign, 1% fp32 denormals, +x/-x
    duplicates, and runs of `run` identical magnitudes with mixed signs planted at
    the magnitude quantiles in `tie_levels` (0.0 = at the maximum), so that a
    top-k threshold at those rates falls inside a run."""
    x = laplace(n, gen, device, b=1e-3)
    bits = x.view(torch.int32)
    r = torch.rand(n, generator=gen, device=device)
    # 1% denormals: exponent field 0, random mantissa, sign kept
    mant = torch.randint(1, 1 << 23, (n,), generator=gen, device=device, dtype=torch.int32)
    bits = torch.where(r < 0.01, (bits & -0x80000000) | mant, bits)
    # +x / -x duplicates: every element in the next 4% copies its left neighbour, negated
    if n > 1:
        dup = (r >= 0.01) & (r < 0.05)
        dup[0] = False
        left = torch.roll(bits, 1)
        bits = torch.where(dup, left ^ -0x80000000, bits)
    # 50% exact zeros, sign bit kept (so half are -0)
    bits = torch.where(r >= 0.5, bits & -0x80000000, bits)
    x = bits.view(torch.float32).clone()
    if n >= 4:
        sub = x.abs()
        if n > 200_000:
            pick = torch.randint(0, n, (200_000,), generator=gen, device=device)
            sub = sub[pick]
        srt = torch.sort(sub, descending=True).values
        for lev in tie_levels:
            mag = srt[min(int(lev * srt.numel()), srt.numel() - 1)]
            if lev == 0.0:
                mag = srt[0] * 2.0
            length = min(run, max(2, n // 3))
            start = int(torch.randint(0, n - length + 1, (1,), generator=gen, device=device).item())
            sign = torch.where(torch.rand(length, generator=gen, device=device) < 0.5, -1.0, 1.0)
            x[start:start + length] = mag * sign
    return x


_DISTS = {"heavy_tail": heavy_tail, "laplace": laplace, "mixture": mixture,
          "adversarial": adversarial}


ROW = 1024  # elements per row of the row-scaled variant


def gradient_layer(cfg, update, layer, n=None, device="cpu", row_spread=0.0, rows_shared=False):
    """Tensor `layer` of the gradient pushed by the worker of queue slot `update`.  With
    row_spread s > 0 every row of ROW consecutive elements is scaled by exp(s * N(0,1)): large
    entries then cluster in some rows, as they do in the gradient of a weight matrix (an outer
    product of a layer's inputs and its output deltas), instead of being spread evenly.  With
    rows_shared the scales of a tensor are the same for every worker (the same rows are hot in
    all queued updates), else each worker draws its own."""
    c = CONFIGS[cfg]
    if n is None:
        n = sizes_of(cfg)[layer]
    gen = _gen(device, c["seed"], 1 + update, layer)
    x = _DISTS[c["dist"]](n, gen, device)
    if row_spread > 0.0 and n > 0:
        rows = (n + ROW - 1) // ROW
        gen_rows = _gen(device, c["seed"], 0, layer, 4242) if rows_shared else gen
        scale = torch.exp(row_spread * torch.randn(rows, generator=gen_rows, device=device, dtype=torch.float32))
        x = x * scale.repeat_interleave(ROW)[:n]
    return x


def gradient(cfg, update=0, device="cpu", layers=None, row_spread=0.0, rows_shared=False):
    sizes = sizes_of(cfg)
    sel = range(len(sizes)) if layers is None else layers
    return [gradient_layer(cfg, update, l, sizes[l], device, row_spread, rows_shared) for l in sel]


def theta0(cfg, device="cpu", layers=None):
    """Initial parameters ~ N(0, 0.05)."""
    c = CONFIGS[cfg]
    sizes = sizes_of(cfg)
    sel = range(len(sizes)) if layers is None else layers
    return [_normal(sizes[l], 0.05, _gen(device, c["seed"], 0, l), device) for l in sel]


def staleness(cfg, Q=None):
    """Global staleness of each queued update, uniform in [1, max_staleness]."""
    c = CONFIGS[cfg]
    Q = c["Q"] if Q is None else Q
    gen = _gen("cpu", c["seed"], 999)
    return torch.randint(1, c["max_staleness"] + 1, (Q,), generator=gen).tolist()


def pull_timestamps(stale, t0=0):
    """Queue slot q is applied at PS time t0+q; a worker of staleness s pulled s
    iterations earlier, but never before the start of the trace (time t0)."""
    return [max(t0, t0 + q - s) for q, s in enumerate(stale)]
