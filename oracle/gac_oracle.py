"""ctypes access to the CPU oracle (``gac_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  This module marshals numpy arrays into the plain C
entry points of the oracle; it holds no arithmetic of the method itself.  Only
tests, the smoke check and the CPU-baseline leg of the benchmark may import it.

Arrays: fp32 gradients are ``np.float32`` arrays, bf16 gradients are
``np.uint16`` arrays holding the raw bfloat16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# GAC_ORACLE_SRC / GAC_ORACLE_LIB let the mutation test point this wrapper at a
# deliberately broken copy of the source (built into a temporary library).
_SRC = os.environ.get("GAC_ORACLE_SRC", os.path.join(_HERE, "gac_oracle.cpp"))
_LIB = os.environ.get("GAC_ORACLE_LIB", os.path.join(_HERE, "libgac_oracle.so"))
# GAC_ORACLE_CXXFLAGS adds compiler flags (the sanitizer test builds an instrumented copy).
_EXTRA_FLAGS = os.environ.get("GAC_ORACLE_CXXFLAGS", "").split()

F32 = 0
BF16 = 1
SAFE, PROJECT, SKIP = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math"] + _EXTRA_FLAGS + ["-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _Decision(ctypes.Structure):
    _fields_ = [("c", ctypes.c_double), ("alpha", ctypes.c_double),
                ("regime", ctypes.c_int32), ("nonfinite", ctypes.c_int32)]


@dataclass
class Decision:
    c: float
    alpha: float
    regime: int
    nonfinite: int


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, vpp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
        i64p, dp = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)
        L.gac_oracle_sums.argtypes = [ctypes.c_int32, vpp, vpp, i64p, ctypes.c_int32, dp]
        L.gac_oracle_sums.restype = None
        L.gac_oracle_decide.argtypes = [dp, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                        ctypes.POINTER(_Decision)]
        L.gac_oracle_decide.restype = None
        for name in ("gac_oracle_project_decomposed", "gac_oracle_project_rank_one"):
            f = getattr(L, name)
            f.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, dp, ctypes.c_double,
                          ctypes.c_double, dp]
            f.restype = None
        L.gac_oracle_passthrough.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, dp]
        L.gac_oracle_passthrough.restype = None
        L.gac_oracle_snapshot.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32]
        L.gac_oracle_snapshot.restype = None
        L.gac_oracle_step.argtypes = [ctypes.c_int32, vpp, vpp, i64p, ctypes.c_int32,
                                      ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                      ctypes.POINTER(dp), dp, ctypes.POINTER(_Decision)]
        L.gac_oracle_step.restype = ctypes.c_int32
        fp = ctypes.POINTER(ctypes.c_float)
        L.gac_oracle_adamw.argtypes = [dp, fp, fp, fp, ctypes.c_int64] + [ctypes.c_double] * 5 + \
                                      [ctypes.c_int64, dp, dp, dp]
        L.gac_oracle_adamw.restype = None
        L.gac_oracle_clip.argtypes = [ctypes.c_int32, ctypes.POINTER(dp), i64p, ctypes.c_double, dp]
        L.gac_oracle_clip.restype = ctypes.c_double
        L.gac_oracle_alignment_stats.argtypes = [dp, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
                                                 ctypes.c_double, dp]
        L.gac_oracle_alignment_stats.restype = None
        L.gac_oracle_regime_counts.argtypes = [dp, ctypes.c_int64, ctypes.c_int64, ctypes.c_double,
                                               ctypes.c_double, i64p]
        L.gac_oracle_regime_counts.restype = None
        _lib = L
    return _lib


def _np_dtype(dtype: int):
    return np.uint16 if dtype == BF16 else np.float32


def _check(arrs: Sequence[np.ndarray], dtype: int) -> None:
    want = _np_dtype(dtype)
    for a in arrs:
        if a.dtype != want or not a.flags["C_CONTIGUOUS"]:
            raise TypeError(f"oracle arrays must be contiguous {want}, got {a.dtype}")


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _numel(arrs: Sequence[np.ndarray]):
    return (ctypes.c_int64 * len(arrs))(*[a.size for a in arrs])


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def sums(g: Sequence[np.ndarray], d: Sequence[np.ndarray], dtype: int) -> np.ndarray:
    """[<g,d>, <g,g>, <d,d>] over the whole tensor list."""
    _check(g, dtype), _check(d, dtype)
    assert len(g) == len(d) and all(a.size == b.size for a, b in zip(g, d))
    out = np.zeros(3, dtype=np.float64)
    lib().gac_oracle_sums(len(g), _ptr_array(g), _ptr_array(d), _numel(g), dtype, _dp(out))
    return out


def decide(s: np.ndarray, c_low: float, c_high: float, eps: float) -> Decision:
    s = np.ascontiguousarray(s, dtype=np.float64)
    dec = _Decision()
    lib().gac_oracle_decide(_dp(s), c_low, c_high, eps, ctypes.byref(dec))
    return Decision(dec.c, dec.alpha, dec.regime, dec.nonfinite)


def _project(fn, g, d, dtype, s, alpha, beta):
    _check([g, d], dtype)
    assert g.size == d.size
    s = np.ascontiguousarray(s, dtype=np.float64)
    out = np.empty(g.size, dtype=np.float64)
    fn(g.ctypes.data, d.ctypes.data, g.size, dtype, _dp(s), alpha, beta, _dp(out))
    return out


def project_decomposed(g, d, dtype, s, alpha, beta=1.0) -> np.ndarray:
    return _project(lib().gac_oracle_project_decomposed, g, d, dtype, s, alpha, beta)


def project_rank_one(g, d, dtype, s, alpha, beta=1.0) -> np.ndarray:
    return _project(lib().gac_oracle_project_rank_one, g, d, dtype, s, alpha, beta)


def passthrough(g: np.ndarray, dtype: int) -> np.ndarray:
    _check([g], dtype)
    out = np.empty(g.size, dtype=np.float64)
    lib().gac_oracle_passthrough(g.ctypes.data, g.size, dtype, _dp(out))
    return out


def snapshot(g: np.ndarray, d: np.ndarray, dtype: int) -> None:
    _check([g, d], dtype)
    assert g.size == d.size
    lib().gac_oracle_snapshot(g.ctypes.data, d.ctypes.data, g.size, dtype)


def step(g: Sequence[np.ndarray], d: Sequence[np.ndarray], dtype: int, c_low: float,
         c_high: float, eps: float, want_output: bool = True):
    """One whole update.  Returns (g_out list of fp64 arrays or None, sums, Decision);
    the state arrays ``d`` are overwritten in place with the raw gradient."""
    _check(g, dtype), _check(d, dtype)
    assert len(g) == len(d) and all(a.size == b.size for a, b in zip(g, d))
    n = len(g)
    outs: Optional[List[np.ndarray]] = None
    out_ptrs = None
    if want_output:
        outs = [np.empty(a.size, dtype=np.float64) for a in g]
        out_ptrs = (ctypes.POINTER(ctypes.c_double) * n)(*[_dp(o) for o in outs])
    s = np.zeros(3, dtype=np.float64)
    dec = _Decision()
    lib().gac_oracle_step(n, _ptr_array(g), _ptr_array(d), _numel(g), dtype, c_low, c_high, eps,
                          out_ptrs, _dp(s), ctypes.byref(dec))
    return outs, s, Decision(dec.c, dec.alpha, dec.regime, dec.nonfinite)


def adamw(g: np.ndarray, p: np.ndarray, m: np.ndarray, v: np.ndarray, lr: float, beta1: float,
          beta2: float, eps_adam: float, weight_decay: float, t: int):
    """One AdamW step; g is fp64, p/m/v are fp32; returns fp64 (p, m, v)."""
    g = np.ascontiguousarray(g, dtype=np.float64)
    for a in (p, m, v):
        if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"] or a.size != g.size:
            raise TypeError("p, m, v must be contiguous float32 of g's size")
    n = g.size
    po, mo, vo = (np.empty(n, dtype=np.float64) for _ in range(3))
    fp = ctypes.POINTER(ctypes.c_float)
    lib().gac_oracle_adamw(_dp(g), p.ctypes.data_as(fp), m.ctypes.data_as(fp),
                           v.ctypes.data_as(fp), n, lr, beta1, beta2, eps_adam, weight_decay,
                           int(t), _dp(po), _dp(mo), _dp(vo))
    return po, mo, vo


def clip(g: Sequence[np.ndarray], max_norm: float):
    """Global-norm clipping of a list of fp64 arrays in place; returns (scale applied, norm)."""
    for a in g:
        if a.dtype != np.float64 or not a.flags["C_CONTIGUOUS"]:
            raise TypeError("clip works on contiguous float64 arrays")
    n = len(g)
    ptrs = (ctypes.POINTER(ctypes.c_double) * n)(*[_dp(a) for a in g])
    norm = ctypes.c_double(0.0)
    scale = lib().gac_oracle_clip(n, ptrs, _numel(g), max_norm, ctypes.byref(norm))
    return scale, norm.value


def alignment_stats(c: np.ndarray, burn_in: int, c_low: float, q: float = 0.9):
    """(q-quantile of |c|, max |c|, fraction with |c| <= c_low, count) after the burn-in."""
    c = np.ascontiguousarray(c, dtype=np.float64)
    out = np.zeros(4, dtype=np.float64)
    lib().gac_oracle_alignment_stats(_dp(c), c.size, burn_in, c_low, q, _dp(out))
    return float(out[0]), float(out[1]), float(out[2]), int(out[3])


def regime_counts(c: np.ndarray, burn_in: int, c_low: float, c_high: float):
    """[safe, projected, skipped] counts of the cosines after the burn-in under one threshold pair."""
    c = np.ascontiguousarray(c, dtype=np.float64)
    out = np.zeros(3, dtype=np.int64)
    lib().gac_oracle_regime_counts(_dp(c), c.size, burn_in, c_low, c_high,
                                   out.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)))
    return [int(x) for x in out]
