"""Helpers shared by the GPU parity tests: run the CPU oracle on host copies of the very
bits the GPU sees, and compare."""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np
import torch

from oracle import gac_oracle as O
from paper_2603_01501_amd import binding as B
from paper_2603_01501_amd import workloads as W

# Tolerances of the parity bar: cosine 1e-6 absolute; projected gradient relative L2
# 1e-5 for fp32 storage and 4e-3 for bf16 storage (the bf16 store rounds to 8 bits).
COS_TOL = 1e-6
SUM_RTOL = 1e-6
GRAD_TOL = {B.F32: 1e-5, B.BF16: 4e-3}


def code(dtype: torch.dtype) -> int:
    return B.torch_dtype_code(dtype)


def host_copies(ts: Sequence[torch.Tensor]) -> List[np.ndarray]:
    return [W.to_oracle_array(t) for t in ts]


def rel_l2(gpu: Sequence[torch.Tensor], want: Sequence[np.ndarray]) -> float:
    """||gpu - want|| / ||want|| over a whole list, accumulated in fp64."""
    num = den = 0.0
    for t, w in zip(gpu, want):
        a = t.detach().to("cpu").reshape(-1).to(torch.float64).numpy()
        num += float(np.dot(a - w, a - w))
        den += float(np.dot(w, w))
    return math.sqrt(num / den) if den > 0 else math.sqrt(num)


def check_projected_tensor(got: torch.Tensor, want: np.ndarray, x: torch.Tensor, y: torch.Tensor,
                           k: float, beta: float, dt: int, name: str = ""):
    """One tensor of the projected gradient against the oracle's fp64 values, element by element
    and as a whole.  got, x (raw gradient) and y (reference state) are device tensors in the
    storage dtype; want is the oracle's output.  The comparison itself runs in fp64 on the
    device that holds them (the oracle's values are uploaded as they are).

    Element bound, from the arithmetic of the pass (one fp32 FMA of exactly widened inputs, then
    for bf16 storage one round-to-nearest-even to 8 significant bits):
        |got - want| <= h |want| + 2^-22 (|beta x| + |k y|) + tiny,
    h = 2^-8 for bf16 (half an ulp at the bottom of a binade), 2^-24 for fp32.  The second term
    covers the fp32 roundings of beta x, of k itself and of the FMA measured against the
    UNCANCELLED size of the two terms (where beta x and k y nearly cancel, the error is that
    of the terms, not of their small sum), and the ~1e-9 relative difference between the
    GPU's k and the oracle's.  Whole tensor (>= 64 elements): relative L2 within the parity
    tolerance for the dtype.  Returns (sum of squared differences, sum of squared wants)."""
    if got.numel() == 0:
        return 0.0, 0.0
    dev = got.device
    w = torch.from_numpy(want).to(dev)
    a = got.detach().reshape(-1).to(torch.float64)
    mag = x.detach().reshape(-1).to(torch.float64).abs_().mul_(abs(beta))
    mag.add_(y.detach().reshape(-1).to(torch.float64).abs_(), alpha=abs(k))
    half_ulp, tiny = (2.0 ** -8, 2.0 ** -134) if dt == B.BF16 else (2.0 ** -24, 2.0 ** -150)
    tol = mag.mul_(2.0 ** -22).add_(w.abs(), alpha=half_ulp).add_(tiny)
    diff = a.sub_(w)
    excess = float((diff.abs() - tol).max())
    assert excess <= 0.0, f"{name}: an element is {excess:.3e} beyond its bound"
    num, den = float(torch.dot(diff, diff)), float(torch.dot(w, w))
    if got.numel() >= 64 and den > 0.0:
        err = math.sqrt(num / den)
        assert err <= GRAD_TOL[dt], f"{name}: rel-L2 {err:.3e}"
    return num, den


def check_projected_list(g_after, outs, g_before, d_before, s, alpha: float, beta: float, dt: int,
                         tensors=None) -> float:
    """Every tensor (or the given ones) through check_projected_tensor, then the list-wide
    relative L2.  s are the oracle's three sums; k = (alpha - beta) <g,d>/<d,d> (Appendix A.2)."""
    k = (alpha - beta) * s[0] / s[2]
    num = den = 0.0
    for j in (range(len(g_after)) if tensors is None else tensors):
        n, d = check_projected_tensor(g_after[j], outs[j], g_before[j], d_before[j], k, beta, dt, f"tensor {j}")
        num += n
        den += d
    err = math.sqrt(num / den) if den > 0 else math.sqrt(num)
    assert err <= GRAD_TOL[dt], f"projected gradient rel-L2 {err}"
    return err


def bits_equal(a: torch.Tensor, b: torch.Tensor) -> bool:
    if a.dtype == torch.bfloat16:
        return torch.equal(a.view(torch.int16), b.view(torch.int16))
    return torch.equal(a.view(torch.int32), b.view(torch.int32))


def check_step(res, g_before: Sequence[torch.Tensor], d_before: Sequence[torch.Tensor],
               g_after: Sequence[torch.Tensor], d_after: Sequence[torch.Tensor], dtype: torch.dtype,
               c_low: float, c_high: float, eps: float, expect_regime=None):
    """Runs the oracle on host copies of (g_before, d_before) and checks the GPU step result,
    the gradient it left behind and the new state against it.  Returns the oracle decision."""
    dt = code(dtype)
    g_h, d_h = host_copies(g_before), host_copies(d_before)
    outs, s, dec = O.step(g_h, d_h, dt, c_low, c_high, eps)
    got = np.array([res.dot, res.gg, res.dd])
    scale = math.sqrt(s[1] * s[2])
    # <g,d> can be tiny relative to |g||d| (orthogonal inputs): bound it by the norms
    assert abs(got[0] - s[0]) <= SUM_RTOL * max(scale, abs(s[0])), (got, s)
    assert abs(got[1] - s[1]) <= SUM_RTOL * s[1] and abs(got[2] - s[2]) <= SUM_RTOL * s[2], (got, s)
    assert abs(res.c - dec.c) <= COS_TOL, (res.c, dec.c)
    assert res.regime == dec.regime, (res.regime, dec.regime, res.c)
    assert res.nonfinite == dec.nonfinite == 0
    if expect_regime is not None:
        assert res.regime == expect_regime, (res.regime, res.c)
    if dec.regime == O.PROJECT:
        assert res.alpha == math.fabs(c_low / res.c)
        assert abs(res.alpha - dec.alpha) <= 1e-4 * dec.alpha
        check_projected_list(g_after, outs, g_before, d_before, s, dec.alpha, 1.0, dt)
    else:
        assert res.alpha == 1.0 and res.coef == 0.0
        for a, b in zip(g_after, g_before):
            assert bits_equal(a, b), "gradient must be untouched outside the projection regime"
    # the new reference state is the raw gradient, bit for bit, in every regime
    for a, b in zip(d_after, g_before):
        assert bits_equal(a, b), "state must equal the raw gradient bitwise"
    return dec, outs


def read_device_record(dev_addr: int) -> "B.GacResult":
    """A gac_result record copied from device (or host-mapped) memory at a raw address."""
    import ctypes
    rec = B.GacResult()
    hip = ctypes.CDLL("libamdhip64.so")  # after torch: binds to the runtime already in the process
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    rc = hip.hipMemcpy(ctypes.byref(rec), ctypes.c_void_p(dev_addr), ctypes.sizeof(rec), 2)  # device -> host
    assert rc == 0, f"hipMemcpy failed: {rc}"
    return rec


def clone_list(ts: Sequence[torch.Tensor]) -> List[torch.Tensor]:
    return [t.clone() for t in ts]


# Relative error allowed on the AdamW step (measured against its uncancelled size): about ten
# fp32 roundings (moments, square root, scaling, sum, division, step size) of 2^-24 each, plus
# half the relative error of the second moment.
ADAMW_STEP_RTOL = 2e-6


def adamw_param_tolerance(p_old: np.ndarray, m_old: np.ndarray, v_new: np.ndarray, g: np.ndarray,
                          lr: float, beta1: float, beta2: float, eps_adam: float, t: int) -> np.ndarray:
    """Element-wise bound for an fp32 AdamW parameter against the fp64 oracle: two roundings of
    the parameter (2 ulp) plus ADAMW_STEP_RTOL of the step evaluated with |m| and |g| - the first moment
    b1 m + (1-b1) g can cancel, and then the fp32 rounding of its two terms, not the size of
    the step itself, sets the error."""
    bc1, bc2 = 1.0 - beta1 ** t, 1.0 - beta2 ** t
    step_abs = lr * (beta1 * np.abs(m_old.astype(np.float64)) + (1.0 - beta1) * np.abs(g)) / bc1 / \
        (np.sqrt(v_new / bc2) + eps_adam)
    return 2.0 * np.spacing(np.abs(p_old)).astype(np.float64) + ADAMW_STEP_RTOL * step_abs


def check_adamw_tensor(p_new, m_new, v_new, po, mo, vo, p_old, m_old, v_old, x, y, k: float, beta: float,
                       lr: float, beta1: float, beta2: float, eps_adam: float, t: int, name: str = ""):
    """One tensor (or a slice of one) of the fused pass's optimizer state against the oracle's
    unfused composition, element by element, compared in fp64 on the device that holds the
    tensors.  p_new, m_new, v_new: fp32 device tensors after the step; po, mo, vo: the oracle's
    fp64 outputs (numpy); p_old, m_old, v_old: fp32 device tensors before the step; x, y: raw
    gradient and reference state (storage dtype, device).

    Bounds, from the kernel's arithmetic (every operation once in fp32, inputs exact).  With
    G = |beta x| + |k y| the uncancelled size of g' (its fp32 error is <= 2^-23 G):
      first moment   |dm| <= 2^-22 (b1 |m| + (1-b1) G)        (an FMA of two rounded terms; the two
                                                               terms can cancel, their errors cannot)
      second moment  |dv| <= 2^-21 (b2 v + (1-b2) G^2)        (all terms are non-negative)
      parameter      |dp| <= 2 ulp(p) + ADAMW_STEP_RTOL x step + (change of the step when the second
                     moment moves by its bound), the step evaluated with b1 |m| + (1-b1) G in
                     place of the new first moment
    Also returns the squared differences and norms of m and v for list-wide figures."""
    dev = p_new.device
    f64 = lambda a: a.detach().reshape(-1).to(torch.float64)
    up = lambda a: torch.from_numpy(a).to(dev)
    G = f64(x).abs_().mul_(abs(beta)).add_(f64(y).abs_(), alpha=abs(k))
    m_unc = f64(m_old).abs_().mul_(beta1).add_(G, alpha=1.0 - beta1)
    mo_d, vo_d, po_d = up(mo), up(vo), up(po)
    dm = f64(m_new).sub_(mo_d)
    excess = float((dm.abs() - m_unc * 2.0 ** -22 - 1e-300).max())
    assert excess <= 0.0, f"{name}: a first moment is {excess:.3e} beyond its bound"
    dv = f64(v_new).sub_(vo_d)
    tol_v = f64(v_old).mul_(beta2).add_(G * G, alpha=1.0 - beta2).mul_(2.0 ** -21)
    excess = float((dv.abs() - tol_v - 1e-300).max())
    assert excess <= 0.0, f"{name}: a second moment is {excess:.3e} beyond its bound"
    # The step lr m^ / (sqrt(v^) + eps): its own roundings (ADAMW_STEP_RTOL), and what the
    # allowed error of the second moment does to it (where g' nearly cancels and v was ~0, the
    # new second moment is small and carries the cancellation error of g'^2; evaluated, not
    # linearised: the step at the smallest second moment the bound allows minus the step at
    # the oracle's).  Both with the uncancelled first moment.
    bc1, bc2 = 1.0 - beta1 ** t, 1.0 - beta2 ** t
    m_unc.mul_(lr / bc1)
    step_mid = m_unc / vo_d.div(bc2).sqrt_().add_(eps_adam)
    step_hi = m_unc / vo_d.sub(tol_v).clamp_(min=0.0).div_(bc2).sqrt_().add_(eps_adam)
    _, e = torch.frexp(p_old.detach().reshape(-1))
    ulp = torch.ldexp(torch.ones_like(e, dtype=torch.float64), e - 24)
    tol_p = ulp.mul_(2.0).add_(step_hi, alpha=ADAMW_STEP_RTOL).add_(step_hi - step_mid)
    over = f64(p_new).sub_(po_d).abs_() - tol_p
    excess = float(over.max())
    if excess > 0.0:
        i = int(over.argmax())
        at = lambda a: float(a.detach().reshape(-1)[i])
        raise AssertionError(
            f"{name}: a parameter is {excess:.3e} beyond its bound at element {i}: p_old={at(p_old)!r} "
            f"p_new={at(p_new)!r} oracle={po[i]!r} m_old={at(m_old)!r} m_new={at(m_new)!r} oracle_m={mo[i]!r} "
            f"v_old={at(v_old)!r} v_new={at(v_new)!r} oracle_v={vo[i]!r} g={at(x)!r} d={at(y)!r} tol={float(tol_p[i])!r}")
    return (float(torch.dot(dm, dm)), float(torch.dot(mo_d, mo_d)),
            float(torch.dot(dv, dv)), float(torch.dot(vo_d, vo_d)))
