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
        err = rel_l2(g_after, outs)
        assert err <= GRAD_TOL[dt], f"projected gradient rel-L2 {err}"
    else:
        assert res.alpha == 1.0 and res.coef == 0.0
        for a, b in zip(g_after, g_before):
            assert bits_equal(a, b), "gradient must be untouched outside the projection regime"
    # the new reference state is the raw gradient, bit for bit, in every regime
    for a, b in zip(d_after, g_before):
        assert bits_equal(a, b), "state must equal the raw gradient bitwise"
    return dec, outs


def clone_list(ts: Sequence[torch.Tensor]) -> List[torch.Tensor]:
    return [t.clone() for t in ts]


def adamw_param_tolerance(p_old: np.ndarray, m_old: np.ndarray, v_new: np.ndarray, g: np.ndarray,
                          lr: float, beta1: float, beta2: float, eps_adam: float, t: int) -> np.ndarray:
    """Element-wise bound for an fp32 AdamW parameter against the fp64 oracle: two roundings of
    the parameter (2 ulp) plus 1e-5 of the step evaluated with |m| and |g| - the first moment
    b1 m + (1-b1) g can cancel, and then the fp32 rounding of its two terms, not the size of
    the step itself, sets the error."""
    bc1, bc2 = 1.0 - beta1 ** t, 1.0 - beta2 ** t
    step_abs = lr * (beta1 * np.abs(m_old.astype(np.float64)) + (1.0 - beta1) * np.abs(g)) / bc1 / \
        (np.sqrt(v_new / bc2) + eps_adam)
    return 2.0 * np.spacing(np.abs(p_old)).astype(np.float64) + 1e-5 * step_abs
