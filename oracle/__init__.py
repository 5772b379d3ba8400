"""ctypes front end of the AdaComp CPU oracle (oracle/adacomp_oracle.c).

TEST INFRASTRUCTURE ONLY: tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this; the product package never does.  It takes and
returns numpy arrays in host memory and shares nothing with the HIP library.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adacomp_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

HISTORY_LISTS = 0    # sorted non-zero index lists + bisection (Sec. 4 "Complexity")
HISTORY_BITMAP = 1   # one bit per parameter per update (brute-force cross-check)
PER_PARAMETER = 0    # AdaComp, eq. 3
GLOBAL = 1           # competitors' rule, Sec. 5.2: sigma = i - j for every entry


def build(force=False):
    """Compile the oracle with gcc (plain C, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", _SRC, "-lm", "-o", _LIB + ".tmp"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # ADACOMP_ORACLE_LIB: load that build instead (tests/test_oracle_mutants.py points it at
        # deliberately broken copies to show that the pins notice)
        lib = C.CDLL(os.environ.get("ADACOMP_ORACLE_LIB") or build())
        u64, u32, f64, vp = C.c_uint64, C.c_uint32, C.c_double, C.c_void_p
        lib.adacomp_oracle_count.restype = u64
        lib.adacomp_oracle_count.argtypes = [u64, f64]
        lib.adacomp_oracle_select_layer.restype = C.c_int
        lib.adacomp_oracle_select_layer.argtypes = [vp, u64, u64, vp, vp]
        lib.adacomp_oracle_select.restype = C.c_int
        lib.adacomp_oracle_select.argtypes = [vp, vp, u32, f64, vp, vp, vp, vp, u64]
        lib.adacomp_oracle_ps_create.restype = vp
        lib.adacomp_oracle_ps_create.argtypes = [u32, vp, C.c_int]
        lib.adacomp_oracle_ps_destroy.restype = None
        lib.adacomp_oracle_ps_destroy.argtypes = [vp]
        lib.adacomp_oracle_ps_timestamp.restype = u64
        lib.adacomp_oracle_ps_timestamp.argtypes = [vp]
        lib.adacomp_oracle_ps_apply.restype = C.c_int
        lib.adacomp_oracle_ps_apply.argtypes = [vp, vp, vp, vp, vp, vp, u64, f64, C.c_int, vp]
        lib.adacomp_oracle_wire_bound.restype = u64
        lib.adacomp_oracle_wire_bound.argtypes = [vp, u32]
        lib.adacomp_oracle_wire_pack.restype = u64
        lib.adacomp_oracle_wire_pack.argtypes = [vp, vp, vp, u32, vp, u64]
        lib.adacomp_oracle_wire_unpack.restype = C.c_int
        lib.adacomp_oracle_wire_unpack.argtypes = [vp, u64, u32, u64, vp, vp, vp]
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def count(n, rate):
    """k for an n-entry tensor at compression ratio `rate` (Alg. 1, SELECT_GRAD)."""
    return int(_load().adacomp_oracle_count(int(n), float(rate)))


def select_layer(g, k):
    """Top-k by magnitude of one tensor -> (idx uint32 ascending, val float32)."""
    g = np.ascontiguousarray(g, dtype=np.float32).ravel()
    k = int(k)
    idx = np.empty(k, dtype=np.uint32)
    val = np.empty(k, dtype=np.float32)
    rc = _load().adacomp_oracle_select_layer(_ptr(g), g.size, k, _ptr(idx), _ptr(val))
    if rc:
        raise RuntimeError(f"oracle select_layer failed ({rc})")
    return idx, val


def select(layers, rate, k_override=None):
    """SELECT_GRAD over a list of tensors -> (layer_off uint64[L+1], idx, val)."""
    layers = [np.ascontiguousarray(g, dtype=np.float32).ravel() for g in layers]
    L = len(layers)
    n = np.array([g.size for g in layers], dtype=np.uint64)
    if k_override is None:
        ks = [count(g.size, rate) for g in layers]
        kov = None
    else:
        ks = [int(k) for k in k_override]
        kov = np.array(ks, dtype=np.uint64)
    cap = int(sum(ks))
    ptrs = (C.c_void_p * max(L, 1))(*[g.ctypes.data for g in layers])
    off = np.zeros(L + 1, dtype=np.uint64)
    idx = np.empty(cap, dtype=np.uint32)
    val = np.empty(cap, dtype=np.float32)
    rc = _load().adacomp_oracle_select(ptrs, _ptr(n), L, float(rate),
                                       _ptr(kov) if kov is not None else None,
                                       _ptr(off), _ptr(idx), _ptr(val), cap)
    if rc:
        raise RuntimeError(f"oracle select failed ({rc})")
    return off, idx, val


class ParameterServer:
    """Alg. 2 with the complete update trace.  `theta` is a list of float32 (or,
    with f64=True, float64) numpy arrays that apply() updates in place."""

    def __init__(self, theta, method=HISTORY_LISTS, f64=False):
        dt = np.float64 if f64 else np.float32
        for a in theta:
            if a.dtype != dt or not a.flags.c_contiguous:
                raise TypeError(f"theta arrays must be contiguous {dt}")
        self.theta = theta
        self.f64 = f64
        self.L = len(theta)
        n = np.array([a.size for a in theta], dtype=np.uint64)
        self._h = _load().adacomp_oracle_ps_create(self.L, _ptr(n), int(method))
        if not self._h:
            raise MemoryError("oracle ps_create")
        self._ptrs = (C.c_void_p * max(self.L, 1))(*[a.ctypes.data for a in theta])

    @property
    def t(self):
        return int(_load().adacomp_oracle_ps_timestamp(self._h))

    def apply(self, layer_off, idx, val, pull_ts, lr, mode=PER_PARAMETER, want_sigma=False):
        """One PS iteration: apply one sparse update pulled at timestamp pull_ts."""
        off = np.ascontiguousarray(layer_off, dtype=np.uint64)
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        val = np.ascontiguousarray(val, dtype=np.float32)
        if off.size != self.L + 1 or int(off[-1]) > idx.size or idx.size != val.size:
            raise ValueError("malformed update")
        sig = np.zeros(idx.size, dtype=np.uint64) if want_sigma else None
        rc = _load().adacomp_oracle_ps_apply(
            self._h, None if self.f64 else self._ptrs, self._ptrs if self.f64 else None,
            _ptr(off), _ptr(idx), _ptr(val), int(pull_ts), float(lr), int(mode),
            _ptr(sig) if sig is not None else None)
        if rc:
            raise RuntimeError(f"oracle ps_apply failed ({rc})")
        return sig

    def close(self):
        if self._h:
            _load().adacomp_oracle_ps_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def wire_bound(layer_off):
    off = np.ascontiguousarray(layer_off, dtype=np.uint64)
    return int(_load().adacomp_oracle_wire_bound(_ptr(off), off.size - 1))


def wire_pack(layer_off, idx, val):
    """The update as the words of the wire format (numpy uint32)."""
    off = np.ascontiguousarray(layer_off, dtype=np.uint64)
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    out = np.empty(wire_bound(off), dtype=np.uint32)
    n = int(_load().adacomp_oracle_wire_pack(_ptr(off), _ptr(idx), _ptr(val), off.size - 1, _ptr(out), out.size))
    if n == 0:
        raise ValueError("indices of a tensor do not ascend strictly")
    return out[:n].copy()


def wire_unpack(words, L, cap=None):
    """(layer_off, idx, val) of a packed update; raises ValueError on a malformed stream."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    if cap is None:
        cap = int(words.size)
    off = np.zeros(L + 1, dtype=np.uint64)
    idx = np.zeros(max(cap, 1), dtype=np.uint32)
    val = np.zeros(max(cap, 1), dtype=np.float32)
    rc = int(_load().adacomp_oracle_wire_unpack(_ptr(words), words.size, L, cap, _ptr(off), _ptr(idx), _ptr(val)))
    if rc:
        raise ValueError(f"malformed wire stream (code {rc})")
    total = int(off[L])
    return off, idx[:total].copy(), val[:total].copy()
