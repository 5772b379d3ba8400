"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its
host-side argument checks answer without touching a GPU."""
import ctypes as C
import os
import re

import pytest

import oracle
import paper_1702_04683_amd as ac
from paper_1702_04683_amd import binding, build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if hip_build.is_stale():
        hip_build.build()
    return ac.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "adacomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adacomp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"adacomp_count", "adacomp_select_workspace", "adacomp_select", "adacomp_apply_workspace",
            "adacomp_apply", "adacomp_strerror"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None


def test_count_matches_oracle_rule(lib):
    import json
    rows = json.load(open(os.path.join(ROOT, "tests", "golden", "count_table.json")))["rows"]
    for n, c, k in rows:
        assert ac.adacomp_count(n, c) == k
    import random
    rnd = random.Random(3)
    for _ in range(20000):
        n = rnd.randrange(0, 1 << 32)
        c = rnd.choice([rnd.random(), rnd.random() ** 4, 1.0 / max(n, 1), 0.0, 1.0, 0.01, 0.005])
        assert ac.adacomp_count(n, c) == oracle.count(n, c), (n, c)


def test_strerror_covers_all_codes(lib):
    text = open(os.path.join(ROOT, "include", "adacomp.h")).read()
    codes = [int(v) for v in re.findall(r"ADACOMP_ERR_[A-Z_]+\s*=\s*(-\d+)", text)]
    assert len(codes) >= 10
    for c in codes + [0]:
        assert "unknown" not in ac.adacomp_strerror(c)
    assert "unknown" in ac.adacomp_strerror(-999)


def test_select_workspace_errors(lib):
    assert ac.adacomp_select_workspace([], 0.5) >= 0
    assert ac.adacomp_select_workspace([10, 0, 5], 0.5) > 0
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(ac.AdaCompError) as e:
            ac.adacomp_select_workspace([10], bad)
        assert e.value.code == -2
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_select_workspace([1 << 32], 0.5)
    assert e.value.code == -3
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_select_workspace([10], 0.5, k_override=[11])
    assert e.value.code == -8


def test_select_argument_checks_run_before_any_launch(lib):
    """All of these must fail on the host: there is no GPU here, a launch would not return a code."""
    n = (C.c_uint64 * 1)(100)
    off = (C.c_uint64 * 2)()
    layer = (binding._Layer * 1)()
    layer[0].data, layer[0].n = 0x1000, 100
    upd = binding._Update(1, C.cast(off, C.POINTER(C.c_uint64)), 0x2000, 0x3000, 0x4000, 0, 0)
    call = lambda rate, u, ws, nb: lib.adacomp_select(layer, 1, rate, None, C.byref(u), ws, nb, None)
    assert call(0.5, upd, 0x10000, 1 << 30) == -4          # capacity 0 < 50
    upd.cap = 50
    assert call(2.0, upd, 0x10000, 1 << 30) == -2
    assert call(0.5, upd, None, 1 << 30) == -5
    assert call(0.5, upd, 0x10001, 1 << 30) == -5          # misaligned workspace
    assert call(0.5, upd, 0x10000, 16) == -5               # too small
    upd.num_layers = 2
    assert call(0.5, upd, 0x10000, 1 << 30) == -6
    upd.num_layers = 1
    layer[0].data = 0x1002
    assert call(0.5, upd, 0x10000, 1 << 30) == -11
    layer[0].data = None
    assert call(0.5, upd, 0x10000, 1 << 30) == -1
    assert lib.adacomp_select(layer, 1, 0.5, None, None, 0x10000, 1 << 30, None) == -1


def test_select_noalloc_refuses_what_its_scratch_cannot_hold(lib):
    """The size check is made on the host, before the built-in buffer is even looked up."""
    sizes = [40_000_000]
    assert ac.adacomp_select_workspace(sizes, 0.01) > ac.SELECT_NOALLOC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "adacomp.h")).read()
    assert re.search(r"ADACOMP_SELECT_NOALLOC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text).groups() == ("32", "20")
    off = (C.c_uint64 * 2)()
    layer = (binding._Layer * 1)()
    layer[0].data, layer[0].n = 0x1000, sizes[0]
    upd = binding._Update(1, C.cast(off, C.POINTER(C.c_uint64)), 0x2000, 0x3000, 0x4000, sizes[0], 0)
    assert lib.adacomp_select_noalloc(layer, 1, 0.01, None, C.byref(upd), None) == -13
    assert lib.adacomp_select_noalloc(layer, 1, 2.0, None, C.byref(upd), None) == -2
    assert lib.adacomp_select_noalloc(layer, 1, 0.01, None, None, None) == -1


def test_apply_argument_checks_run_before_any_launch(lib):
    off = (C.c_uint64 * 2)(0, 3)
    par = (binding._Layer * 1)()
    par[0].data, par[0].n = 0x1000, 100
    cnt = (C.c_void_p * 1)(0x5000)
    st = binding._State(5, 1, C.cast(cnt, C.POINTER(C.c_void_p)))
    upd = (binding._Update * 1)()
    upd[0] = binding._Update(1, C.cast(off, C.POINTER(C.c_uint64)), 0x2000, 0x3000, 0x4000, 3, 5)
    call = lambda lr=0.1, ws=0x10000, nb=1 << 20: lib.adacomp_apply(par, 1, C.byref(st), upd, 1, lr, ws, nb, None)
    upd[0].pull_ts = 6
    assert call() == -7                                     # pulled in the future
    upd[0].pull_ts = 4
    assert call() == -9                                     # pulled before this call's first update
    upd[0].pull_ts = 5
    assert call(lr=float("inf")) == -10
    assert call(ws=None) == -5
    assert call(nb=8) == -5
    off[1] = 101
    upd[0].cap = 101
    assert call() == -6                                     # more entries than the tensor has parameters
    off[1] = 3
    upd[0].cap = 2
    assert call() == -4
    upd[0].cap = 3
    upd[0].num_layers = 2
    assert call() == -6
    upd[0].num_layers = 1
    st.num_layers = 2
    assert call() == -6
    st.num_layers = 1
    assert st.t == 5                                        # no failing call advanced the timestamp
    need = C.c_size_t()
    n = (C.c_uint64 * 1)(100)
    assert lib.adacomp_apply_workspace(n, 1, C.byref(st), upd, 1, C.byref(need)) == 0 and need.value >= 12
    upd[0].pull_ts = 3                                      # two timestamps back, nothing remembered
    assert lib.adacomp_apply_workspace(n, 1, C.byref(st), upd, 1, C.byref(need)) == -9
    off[1], upd[0].cap = 0, 0                               # ... which an update without entries never needs
    assert lib.adacomp_apply_workspace(n, 1, C.byref(st), upd, 1, C.byref(need)) == 0
    off[1], upd[0].cap = 3, 3
    ring = (binding._Update * 4)()
    ring_off = (C.c_uint64 * 8)()
    st.history_cap, st.history_len = 4, 1
    st.history, st.history_off = C.cast(ring, C.POINTER(binding._Update)), C.cast(ring_off, C.POINTER(C.c_uint64))
    assert call() == -9                                     # only one update remembered
    st.history_len = 2
    upd[0].pull_ts = 6
    assert call() == -7
    assert lib.adacomp_apply_workspace(n, 1, None, upd, 1, C.byref(need)) == -7


def test_hook_flipped_between_sizing_and_call_is_caught(lib, monkeypatch):
    """The environment switches are test hooks that choose between execution plans.  Both the sizing
    call and the real call derive the plan and its workspace layout from what they see; if a hook
    changes in between and the real call's plan needs more bytes than were sized, the call is
    refused with ADACOMP_ERR_WORKSPACE before anything is enqueued."""
    # select: small tensors are selected by one workgroup each and need next to no scratch; with the
    # hook they go through the streaming pipeline (histograms, segment tables, candidate regions)
    sizes = [200_000, 150_000, 70_000]
    need_default = ac.adacomp_select_workspace(sizes, 0.01)
    monkeypatch.setenv("ADACOMP_SELECT_SMALL", "0")
    need_pipeline = ac.adacomp_select_workspace(sizes, 0.01)
    assert need_pipeline > need_default
    off = (C.c_uint64 * 4)()
    layers = (binding._Layer * 3)()
    for l, n in enumerate(sizes):
        layers[l].data, layers[l].n = 0x100000 * (l + 1), n
    upd = binding._Update(3, C.cast(off, C.POINTER(C.c_uint64)), 0x2000, 0x3000, 0x4000, sum(sizes), 0)
    assert lib.adacomp_select(layers, 3, 0.01, None, C.byref(upd), 0x10000, need_default, None) == -5
    monkeypatch.delenv("ADACOMP_SELECT_SMALL")
    # the grouping hook only ever shrinks the candidate regions (groups reuse them): sized with one group, a call
    # that sees several groups fits; sized with several groups, a call that sees one group is refused
    big = [5_000_000] * 6
    monkeypatch.setenv("ADACOMP_SELECT_GROUP_MB", "8")
    need_groups = ac.adacomp_select_workspace(big, 0.01)
    monkeypatch.setenv("ADACOMP_SELECT_GROUP_MB", "0")
    need_one = ac.adacomp_select_workspace(big, 0.01)
    assert need_one > need_groups
    boff = (C.c_uint64 * 7)()
    blayers = (binding._Layer * 6)()
    for l, n in enumerate(big):
        blayers[l].data, blayers[l].n = 0x10000000 * (l + 1), n
    bupd = binding._Update(6, C.cast(boff, C.POINTER(C.c_uint64)), 0x2000, 0x3000, 0x4000, sum(big), 0)
    assert lib.adacomp_select(blayers, 6, 0.01, None, C.byref(bupd), 0x10000, need_groups, None) == -5
    monkeypatch.delenv("ADACOMP_SELECT_GROUP_MB")
    # apply: the update-by-update plan needs the table and one snapshot word per entry, the sweep also
    # the slice bounds of every update in every tile
    n = (C.c_uint64 * 1)(3_000_000)
    aoff = (C.c_uint64 * 2)(0, 30_000)
    par = (binding._Layer * 1)()
    par[0].data, par[0].n = 0x100000, 3_000_000
    cnt = (C.c_void_p * 1)(0x5000000)
    st = binding._State(0, 1, C.cast(cnt, C.POINTER(C.c_void_p)))
    ups = (binding._Update * 8)()
    for q in range(8):
        ups[q] = binding._Update(1, C.cast(aoff, C.POINTER(C.c_uint64)), 0x2000, 0x300000, 0x400000, 30_000, 0)
    need = C.c_size_t()
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "scatter")
    assert lib.adacomp_apply_workspace(n, 1, C.byref(st), ups, 8, C.byref(need)) == 0
    need_scatter = need.value
    monkeypatch.setenv("ADACOMP_APPLY_PLAN", "sweep")
    assert lib.adacomp_apply_workspace(n, 1, C.byref(st), ups, 8, C.byref(need)) == 0
    assert need.value > need_scatter
    assert lib.adacomp_apply(par, 1, C.byref(st), ups, 8, 0.1, 0x10000, need_scatter, None) == -5
    assert st.t == 0


def test_wire_host_side_checks(lib):
    off = [0, 130, 130, 131]
    B = 3 + 0 + 1
    assert ac.adacomp_wire_bound(off) == 4 + 3 + B + 1 + 131 + 131
    assert ac.adacomp_wire_bound(off) >= oracle.wire_bound(off)
    assert ac.adacomp_wire_workspace(off) % 256 == 0
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_wire_bound([0, 5, 3])
    assert e.value.code == -6
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_wire_bound([1, 5])
    assert e.value.code == -6
    with pytest.raises(ac.AdaCompError) as e:
        ac.adacomp_wire_bound([0, 1 << 33])
    assert e.value.code == -3


def test_global_staleness_validate_and_wire_argument_checks_run_before_any_launch(lib):
    """Every failing call below must fail on the host (no GPU here) and leave the state untouched."""
    off = (C.c_uint64 * 2)(0, 3)
    par = (binding._Layer * 1)()
    par[0].data, par[0].n = 0x1000, 100
    st = binding._State(5, 1, None)                         # the competitors' rule needs no counters
    upd = (binding._Update * 1)()
    upd[0] = binding._Update(1, C.cast(off, C.POINTER(C.c_uint64)), 0x2000, 0x3000, 0x4000, 3, 5)
    call = lambda lr=0.1, ws=0x10000, nb=1 << 12: lib.adacomp_apply_global_staleness(par, 1, C.byref(st), upd, 1, lr, ws, nb,
                                                                                       None)
    upd[0].pull_ts = 6
    assert call() == -7
    upd[0].pull_ts = 0                                      # any earlier pull is fine for this rule ...
    assert call(ws=None) == -5                              # ... so the next check is the workspace
    assert call(nb=8) == -5
    assert call(ws=0x10010) == -5
    assert call(lr=float("nan")) == -10
    upd[0].cap = 2
    assert call() == -4
    upd[0].cap = 3
    upd[0].val = 0x4002
    assert call() == -11
    upd[0].val = 0x4000
    st.num_layers = 3
    assert call() == -6
    st.num_layers = 1
    assert st.t == 5

    v = lambda u, n=0x6000, L=1, flags=0x7000: lib.adacomp_update_validate(C.byref(u), n, L, flags, None)
    assert v(upd[0], flags=None) == -1
    assert v(upd[0], n=None) == -1
    assert v(upd[0], L=2) == -6
    assert v(upd[0], flags=0x7002) == -11
    upd[0].cap = 1
    assert v(upd[0]) == -4
    upd[0].cap = 3

    words = C.c_uint64()
    pack = lambda u, wire=0x8000, cap=1 << 20, out=0x9000, ws=0x10000, nb=1 << 12: lib.adacomp_wire_pack(
        C.byref(u), wire, cap, out, ws, nb, None)
    assert pack(upd[0], out=None) == -1
    assert pack(upd[0], wire=None) == -1
    assert pack(upd[0], wire=0x8002) == -11
    assert pack(upd[0], out=0x9004) == -11
    assert pack(upd[0], ws=None) == -5
    assert pack(upd[0], nb=16) == -5
    upd[0].cap = 2
    assert pack(upd[0]) == -4
    upd[0].cap = 3
    unpack = lambda u, wire=0x8000, n=100, flags=0x7000, ws=0x10000, nb=1 << 12: lib.adacomp_wire_unpack(
        wire, n, C.byref(u), flags, ws, nb, None)
    assert unpack(upd[0], flags=None) == -1
    assert unpack(upd[0], wire=None) == -1
    assert unpack(upd[0], wire=0x8001) == -11
    assert unpack(upd[0], ws=0x10000, nb=0) == -5
    off[1] = 4                                              # the receiver expects more entries than the buffers hold
    assert unpack(upd[0]) == -4
    off[1] = 3
    assert lib.adacomp_wire_bound(off, 1, C.byref(words)) == 0 and words.value == 4 + 1 + 1 + 1 + 3 + 3
    assert lib.adacomp_wire_bound(off, 1, None) == -1
