"""Thin ctypes binding of libgac.so: the same entry points as include/gac.h.

Only argument marshalling happens here (torch tensors -> device pointers, Python
numbers -> C structs).  Every step of the method runs in the HIP kernels of the
library; there is no Python or CPU fallback, and a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

from . import build as _build

F32 = 0
BF16 = 1
SAFE, PROJECT, SKIP = 0, 1, 2
REGIME_NAMES = {SAFE: "safe", PROJECT: "project", SKIP: "skip"}

OK = 0
ERR_INVALID_ARG = -1
ERR_BAD_THRESHOLDS = -2
ERR_ALLOC = -3
ERR_HIP = -4
ERR_NONFINITE = -5
ERR_UNIMPLEMENTED = -6
ERR_TOO_LARGE = -7

FLAG_SNAPSHOT_IN_REDUCE = 1
STATIC_MAX_TENSORS = 1024


class GacConfig(ctypes.Structure):
    _fields_ = [("c_low", ctypes.c_double), ("c_high", ctypes.c_double), ("eps", ctypes.c_double),
                ("beta", ctypes.c_double), ("dtype", ctypes.c_int32), ("n_tensors", ctypes.c_int32),
                ("numel", ctypes.POINTER(ctypes.c_int64)), ("state_ptrs", ctypes.POINTER(ctypes.c_void_p)),
                ("device", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("chunk_elems", ctypes.c_int32), ("grid_blocks", ctypes.c_int32),
                ("apply_blocks", ctypes.c_int32), ("max_grad_norm", ctypes.c_double),
                ("history_capacity", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class GacResult(ctypes.Structure):
    _fields_ = [("dot", ctypes.c_double), ("gg", ctypes.c_double), ("dd", ctypes.c_double),
                ("c", ctypes.c_double), ("alpha", ctypes.c_double), ("coef", ctypes.c_double),
                ("grad_norm", ctypes.c_double), ("clip_coef", ctypes.c_double),
                ("scale_g", ctypes.c_double), ("coef_d", ctypes.c_double),
                ("regime", ctypes.c_int32), ("nonfinite", ctypes.c_int32),
                ("modified", ctypes.c_int32), ("reserved", ctypes.c_int32), ("step", ctypes.c_int64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class GacDiag(ctypes.Structure):
    _fields_ = [("first_step", ctypes.c_int64), ("last_step", ctypes.c_int64),
                ("n_values", ctypes.c_int64), ("n_nonfinite", ctypes.c_int64),
                ("regime_count", ctypes.c_int64 * 3), ("q90_abs_c", ctypes.c_double),
                ("max_abs_c", ctypes.c_double), ("frac_le_c_low", ctypes.c_double)]


MAX_PLACEMENT_CANDIDATES = 16


class GacPlacement(ctypes.Structure):
    _fields_ = [("n_candidates", ctypes.c_int32), ("chosen", ctypes.c_int32),
                ("apply_blocks", ctypes.c_int32), ("n_blocks_tried", ctypes.c_int32),
                ("probe_ms", ctypes.c_double * MAX_PLACEMENT_CANDIDATES),
                ("reduce_ms", ctypes.c_double * MAX_PLACEMENT_CANDIDATES),
                ("blocks_tried", ctypes.c_int32 * 4), ("blocks_ms", ctypes.c_double * 4),
                ("bytes_held_peak", ctypes.c_int64)]


class GacAdamWHyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps_adam", ctypes.c_double), ("weight_decay", ctypes.c_double),
                ("t_adam", ctypes.c_int64)]


class GacError(RuntimeError):
    def __init__(self, code: int, detail: str = ""):
        self.code = code
        msg = lib().gac_strerror(code).decode()
        super().__init__(f"gac error {code}: {msg}" + (f" ({detail})" if detail else ""))


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Opens libgac.so.  It is built only if it does not exist at all.  A library that was built
    from other sources than the ones beside it is refused (build again: python
    __graft_entry__.py); a stale or missing library is never replaced by another code path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    # PyTorch ships its own HIP runtime under the same soname as the system one.  Importing
    # torch first makes libgac.so bind to the runtime torch already loaded, so the tensors'
    # memory, the streams and the kernels all live in ONE runtime; the other order ends with
    # two runtimes in the process and failing HIP calls.
    import torch  # noqa: F401
    L = ctypes.CDLL(_build.LIB_PATH)
    vp, vpp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
    i64p, dp = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)
    resp = ctypes.POINTER(GacResult)
    sig = {
        "gac_default_config": (None, [ctypes.POINTER(GacConfig)]),
        "gac_init": (ctypes.c_int, [ctypes.POINTER(vp), ctypes.POINTER(GacConfig)]),
        "gac_destroy": (None, [vp]),
        "gac_step": (ctypes.c_int, [vp, vpp, vp, resp]),
        "gac_step_exchange": (ctypes.c_int, [vp, vpp, vp, resp]),
        "gac_reduce_local": (ctypes.c_int, [vp, vpp, vp, vp]),
        "gac_apply": (ctypes.c_int, [vp, vpp, vp, vp, resp]),
        "gac_step_adamw": (ctypes.c_int, [vp, vpp, vpp, vpp, vpp, vpp, ctypes.POINTER(GacAdamWHyper), vp, resp]),
        "gac_result_device": (ctypes.c_int, [vp, ctypes.POINTER(vp)]),
        "gac_state_export": (ctypes.c_int, [vp, vpp, i64p, vp]),
        "gac_state_import": (ctypes.c_int, [vp, vpp, ctypes.c_int64, vp]),
        "gac_reset": (ctypes.c_int, [vp, vp]),
        "gac_set_thresholds": (ctypes.c_int, [vp, ctypes.c_double, ctypes.c_double]),
        "gac_history_read": (ctypes.c_int, [vp, ctypes.c_int64, dp, ctypes.POINTER(ctypes.c_int32), i64p, i64p, vp]),
        "gac_diag_summary": (ctypes.c_int, [vp, ctypes.c_int64, ctypes.POINTER(GacDiag), vp]),
        "gac_threshold_sweep": (ctypes.c_int, [vp, ctypes.c_int64, ctypes.c_int32, dp, dp,
                                               ctypes.POINTER(ctypes.c_int32), vp]),
        "gac_place_state": (ctypes.c_int, [vp, vpp, ctypes.c_int32, ctypes.c_int64, vp,
                                           ctypes.POINTER(GacPlacement)]),
        "gac_plan_query": (ctypes.c_int, [i64p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, i64p, i64p]),
        "gac_profile_enable": (ctypes.c_int, [vp, ctypes.c_int32]),
        "gac_profile_read": (ctypes.c_int, [vp, dp, dp, dp, ctypes.POINTER(ctypes.c_int32)]),
        "gac_strerror": (ctypes.c_char_p, [ctypes.c_int]),
        "gac_last_hip_error": (ctypes.c_char_p, [vp]),
        "gac_version": (ctypes.c_char_p, []),
        "gac_source_hash": (ctypes.c_char_p, []),
        "gac_step_static": (ctypes.c_int, [ctypes.POINTER(GacConfig), vpp, ctypes.c_int64, vp, vp]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    built_from = L.gac_source_hash().decode()
    if built_from != _build.source_hash():
        raise RuntimeError(
            f"{_build.LIB_PATH} was built from other sources (hash {built_from[:12] or 'none'}, "
            f"sources {_build.source_hash()[:12]}): build again with python __graft_entry__.py")
    _lib = L
    return L


def torch_dtype_code(dtype) -> int:
    import torch
    if dtype == torch.float32:
        return F32
    if dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported gradient dtype {dtype}")


def ptr_list(tensors: Optional[Sequence]) -> Optional[ctypes.Array]:
    """Host array of the tensors' device pointers (tensors must be contiguous)."""
    if tensors is None or isinstance(tensors, ctypes.Array):
        return tensors  # an array built earlier by this function is passed through
    for t in tensors:
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    return (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def _stream_handle(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = getattr(stream, "cuda_stream", stream)
    return ctypes.c_void_p(int(h))


def gac_plan_query(numel: Sequence[int], dtype: int, chunk_elems: int = 0):
    arr = (ctypes.c_int64 * len(numel))(*numel)
    nc, tot = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = lib().gac_plan_query(arr, len(numel), dtype, chunk_elems, ctypes.byref(nc), ctypes.byref(tot))
    if rc != OK:
        raise GacError(rc)
    return nc.value, tot.value


def make_config(numel: Sequence[int], dtype: int, c_low: float = 0.05, c_high: float = 0.3,
                eps: float = 1e-8, beta: float = 1.0, state: Optional[Sequence] = None, device: int = -1,
                chunk_elems: int = 0, grid_blocks: int = 0, apply_blocks: int = 0,
                max_grad_norm: float = 0.0, history_capacity: int = 0, flags: int = 0):
    """A filled gac_config and the ctypes arrays it points to (keep them alive with it)."""
    cfg = GacConfig()
    lib().gac_default_config(ctypes.byref(cfg))
    cfg.c_low, cfg.c_high, cfg.eps, cfg.beta = c_low, c_high, eps, beta
    cfg.dtype, cfg.n_tensors = dtype, len(numel)
    numel_arr = (ctypes.c_int64 * len(numel))(*numel)
    cfg.numel = numel_arr
    state_ptrs = ptr_list(state)
    if state_ptrs is not None:
        cfg.state_ptrs = ctypes.cast(state_ptrs, ctypes.POINTER(ctypes.c_void_p))
    cfg.device, cfg.chunk_elems, cfg.grid_blocks = device, chunk_elems, grid_blocks
    cfg.apply_blocks = apply_blocks
    cfg.max_grad_norm, cfg.history_capacity, cfg.flags = max_grad_norm, history_capacity, flags
    return cfg, (numel_arr, state_ptrs)


def gac_step_static(cfg: GacConfig, grads: Sequence, step: int, result_out=None, stream=None) -> int:
    """The step that allocates nothing (no context).  ``cfg`` comes from make_config with
    ``state`` given; ``result_out`` is None or a device-accessible buffer of at least
    ctypes.sizeof(GacResult) bytes (a torch uint8 tensor, or an address).  Only enqueues work;
    returns the C return code after raising on errors."""
    if result_out is not None and hasattr(result_out, "data_ptr"):
        result_out = result_out.data_ptr()
    rc = lib().gac_step_static(ctypes.byref(cfg), ptr_list(grads), step, _stream_handle(stream),
                               ctypes.c_void_p(result_out) if result_out else None)
    if rc != OK:
        raise GacError(rc, lib().gac_last_hip_error(None).decode())
    return rc


class Gac:
    """One GAC context (gac_init ... gac_destroy) over a fixed list of tensor sizes."""

    def __init__(self, numel: Sequence[int], dtype: int, c_low: float = 0.05, c_high: float = 0.3,
                 eps: float = 1e-8, beta: float = 1.0, state: Optional[Sequence] = None,
                 device: int = -1, chunk_elems: int = 0, grid_blocks: int = 0, apply_blocks: int = 0,
                 max_grad_norm: float = 0.0, history_capacity: int = 0, flags: int = 0):
        L = lib()
        cfg, keep = make_config(numel, dtype, c_low, c_high, eps, beta, state, device, chunk_elems,
                                grid_blocks, apply_blocks, max_grad_norm, history_capacity, flags)
        self._numel, self._state_ptrs = keep
        self._state_keepalive = state
        self._ctx = ctypes.c_void_p()
        rc = L.gac_init(ctypes.byref(self._ctx), ctypes.byref(cfg))
        if rc != OK:
            self._ctx = ctypes.c_void_p()
            raise GacError(rc, L.gac_last_hip_error(None).decode())
        self.n_tensors = len(numel)
        self.dtype = dtype

    # -- lifetime
    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            lib().gac_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, allow_nonfinite: bool = True):
        if rc == OK or (allow_nonfinite and rc == ERR_NONFINITE):
            return rc
        raise GacError(rc, lib().gac_last_hip_error(self._ctx).decode())

    # -- the C entry points, same names
    def gac_step(self, grads: Sequence, stream=None, sync: bool = True) -> Optional[GacResult]:
        res = GacResult() if sync else None
        rc = lib().gac_step(self._ctx, ptr_list(grads), _stream_handle(stream),
                            ctypes.byref(res) if sync else None)
        self._check(rc)
        return res

    def gac_step_exchange(self, grads: Sequence, stream=None):
        """Returns (result, returned): ``returned`` are the tensors that held the reference
        state before the call (holding g' in the projection regime); ``grads`` now belong to
        the library as the new reference state.  Tensors are tracked by device pointer."""
        ptrs = ptr_list(list(grads))
        by_ptr = {t.data_ptr(): t for t in self._state_keepalive}
        res = GacResult()
        rc = lib().gac_step_exchange(self._ctx, ptrs, _stream_handle(stream), ctypes.byref(res))
        self._check(rc)
        if rc == ERR_NONFINITE:
            return res, list(grads)
        returned = [by_ptr[ptrs[j]] if ptrs[j] is not None else self._state_keepalive[j]
                    for j in range(len(grads))]
        self._state_keepalive = list(grads)
        return res, returned

    def gac_reduce_local(self, grads: Sequence, dev_sums3, stream=None) -> None:
        rc = lib().gac_reduce_local(self._ctx, ptr_list(grads), _stream_handle(stream),
                                    ctypes.c_void_p(dev_sums3.data_ptr()))
        self._check(rc)

    def gac_apply(self, grads: Sequence, dev_sums3, stream=None, sync: bool = True) -> Optional[GacResult]:
        res = GacResult() if sync else None
        rc = lib().gac_apply(self._ctx, ptr_list(grads), ctypes.c_void_p(dev_sums3.data_ptr()),
                             _stream_handle(stream), ctypes.byref(res) if sync else None)
        self._check(rc)
        return res

    def gac_step_adamw(self, grads: Sequence, master_p: Sequence, m: Sequence, v: Sequence,
                       p_lowp: Optional[Sequence], lr: float, beta1: float, beta2: float,
                       eps_adam: float, weight_decay: float, t_adam: int, stream=None,
                       sync: bool = True) -> Optional[GacResult]:
        hyper = GacAdamWHyper(lr, beta1, beta2, eps_adam, weight_decay, t_adam)
        res = GacResult() if sync else None
        rc = lib().gac_step_adamw(self._ctx, ptr_list(grads), ptr_list(master_p), ptr_list(m),
                                  ptr_list(v), ptr_list(p_lowp), ctypes.byref(hyper),
                                  _stream_handle(stream), ctypes.byref(res) if sync else None)
        self._check(rc)
        return res

    def gac_result_device(self) -> int:
        p = ctypes.c_void_p()
        self._check(lib().gac_result_device(self._ctx, ctypes.byref(p)))
        return p.value

    def gac_state_export(self, dst: Sequence, stream=None) -> int:
        step = ctypes.c_int64(0)
        self._check(lib().gac_state_export(self._ctx, ptr_list(dst), ctypes.byref(step), _stream_handle(stream)))
        return step.value

    def gac_state_import(self, src: Sequence, step: int, stream=None) -> None:
        self._check(lib().gac_state_import(self._ctx, ptr_list(src), step, _stream_handle(stream)))

    def gac_reset(self, stream=None) -> None:
        self._check(lib().gac_reset(self._ctx, _stream_handle(stream)))

    def gac_set_thresholds(self, c_low: float, c_high: float) -> None:
        self._check(lib().gac_set_thresholds(self._ctx, c_low, c_high))

    def gac_history_read(self, max_n: int = 4096, stream=None):
        """(list of c_t, list of regimes, step number of the first entry), oldest first."""
        c = (ctypes.c_double * max_n)()
        r = (ctypes.c_int32 * max_n)()
        n, first = ctypes.c_int64(0), ctypes.c_int64(0)
        self._check(lib().gac_history_read(self._ctx, max_n, c, r, ctypes.byref(n), ctypes.byref(first),
                                           _stream_handle(stream)))
        return list(c[:n.value]), list(r[:n.value]), first.value

    def gac_diag_summary(self, burn_in: int = 0, stream=None) -> GacDiag:
        d = GacDiag()
        self._check(lib().gac_diag_summary(self._ctx, burn_in, ctypes.byref(d), _stream_handle(stream)))
        return d

    def gac_place_state(self, grads, max_candidates: int = MAX_PLACEMENT_CANDIDATES,
                        max_extra_bytes: int = 0, stream=None) -> GacPlacement:
        rep = GacPlacement()
        self._check(lib().gac_place_state(self._ctx, ptr_list(grads), max_candidates, max_extra_bytes,
                                          _stream_handle(stream), ctypes.byref(rep)))
        return rep

    def gac_threshold_sweep(self, pairs, burn_in: int = 0, stream=None):
        """[[safe, projected, skipped], ...] per (c_low, c_high) pair over the recorded steps."""
        n = len(pairs)
        lo = (ctypes.c_double * max(n, 1))(*[float(p[0]) for p in pairs])
        hi = (ctypes.c_double * max(n, 1))(*[float(p[1]) for p in pairs])
        counts = (ctypes.c_int32 * (3 * max(n, 1)))()
        self._check(lib().gac_threshold_sweep(self._ctx, burn_in, n, lo, hi, counts, _stream_handle(stream)))
        return [list(counts[3 * i:3 * i + 3]) for i in range(n)]

    def gac_profile_enable(self, on: bool) -> None:
        self._check(lib().gac_profile_enable(self._ctx, 1 if on else 0))

    def gac_profile_read(self):
        """(ms_reduce, ms_finalize, ms_apply, n_steps), summed over the steps since the last read."""
        a, b, c, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_double(), ctypes.c_int32()
        self._check(lib().gac_profile_read(self._ctx, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                           ctypes.byref(n)))
        return a.value, b.value, c.value, n.value
