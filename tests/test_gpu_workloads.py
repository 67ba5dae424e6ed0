"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration
bench.py times (default chunk size and grids).

The statistics, the cosine and the regime are checked against the oracle over ALL elements
(the oracle's three sums take a few ns per element).  The projected gradient is checked
against the oracle element by element on every tensor for the 0.5B and 1.5B lists, and on a
sample of tensors (one of each kind, including the largest) for the 7.6B list, where
properties that hold at any size cover the rest.  State and untouched gradients are compared
bitwise on the GPU against clones.
"""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import gac_oracle as O
from paper_2603_01501_amd import binding as B
from paper_2603_01501_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
C_LOW, C_HIGH, EPS = 0.05, 0.3, 1e-8


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def oracle_decision(g, d, dtype, c_low, c_high):
    dt = U.code(dtype)
    g_h, d_h = U.host_copies(g), U.host_copies(d)
    s = O.sums(g_h, d_h, dt)
    return g_h, d_h, s, O.decide(s, c_low, c_high, EPS)


def check_result(res, s, dec):
    scale = math.sqrt(s[1] * s[2])
    assert abs(res.dot - s[0]) <= U.SUM_RTOL * max(scale, abs(s[0])), (res.dot, s[0])
    assert abs(res.gg - s[1]) <= U.SUM_RTOL * s[1] and abs(res.dd - s[2]) <= U.SUM_RTOL * s[2]
    assert abs(res.c - dec.c) <= U.COS_TOL, (res.c, dec.c)
    assert res.regime == dec.regime and res.nonfinite == 0


def check_projection(g_after, g_h, d_h, s, dec, dtype, tensors):
    """rel-L2 of the GPU's projected gradient against the oracle over the given tensors."""
    dt = U.code(dtype)
    num = den = 0.0
    for j in tensors:
        want = O.project_decomposed(g_h[j], d_h[j], dt, s, dec.alpha)
        got = g_after[j].detach().to("cpu").reshape(-1).to(torch.float64).numpy()
        diff = got - want
        num += float(np.dot(diff, diff))
        den += float(np.dot(want, want))
        del want, got, diff
    err = math.sqrt(num / den)
    assert err <= U.GRAD_TOL[dt], err
    return err


def run_case(shapes, dtype, rho, config_id, c_high, expect):
    g, d0 = W.correlated_pair(shapes, dtype, rho, 1e-3, config_id, device=DEV)
    d = U.clone_list(d0)
    ctx = B.Gac([W.numel(s) for s in shapes], U.code(dtype), c_high=c_high, state=d)
    ctx.gac_state_import(d0, 0)
    g_raw = U.clone_list(g)
    res = ctx.gac_step(g)
    torch.cuda.synchronize()
    g_h, d_h, s, dec = oracle_decision(g_raw, d0, dtype, C_LOW, c_high)
    check_result(res, s, dec)
    assert res.regime == expect, (res.regime, res.c)
    n = W.total_numel(shapes)
    assert abs(res.c - rho) <= 5 * (1 - rho * rho) / math.sqrt(n) + 2e-3
    assert all(U.bits_equal(a, b) for a, b in zip(d, g_raw)), "state must be the raw gradient"
    if expect == B.PROJECT:
        err = check_projection(g, g_h, d_h, s, dec, dtype, range(len(shapes)))
        say(f"  rho={rho} c={res.c:.6f} project rel-L2={err:.2e}")
    else:
        assert all(U.bits_equal(a, b) for a, b in zip(g, g_raw)), "gradient must be untouched"
        say(f"  rho={rho} c={res.c:.6f} regime={B.REGIME_NAMES[res.regime]}")
    ctx.close()


@pytest.mark.parametrize("c_high,expect", [(0.3, B.SKIP), (2.0, B.PROJECT)])
def test_half_billion_fp32_list(c_high, expect):
    """0.5B-style transformer gradient list, fp32, 218 tensors, rho = 0.9."""
    run_case(W.MODEL_05B.tensor_shapes(), torch.float32, 0.9, 2, c_high, expect)


@pytest.mark.parametrize("rho,c_high,expect", [(0.0, 0.3, B.SAFE), (0.5, 0.3, B.SKIP), (0.9, 0.3, B.SKIP),
                                               (0.99, 0.3, B.SKIP), (0.15, 0.3, B.PROJECT),
                                               (0.9, 2.0, B.PROJECT)])
def test_one_and_a_half_billion_bf16_list(rho, c_high, expect):
    """1.5B-style list, bf16 storage with fp32/fp64 accumulation, 254 tensors, rho sweep under
    the default thresholds, plus the two cases that reach the projection branch."""
    run_case(W.MODEL_15B.tensor_shapes(), torch.bfloat16, rho, 3, c_high, expect)


def test_seven_billion_bf16_list_consecutive_steps():
    """7.6B-style list (255 tensors, 7,615,487,488 elements, bf16), consecutive AR(1)
    gradients with the state carried by the library: step 1 safe (zero reference), step 2
    projected (thresholds 0.05 / 2.0), step 3 skipped (thresholds 0.05 / 0.3)."""
    dtype = torch.bfloat16
    shapes = W.MODEL_76B.tensor_shapes()
    numel = [W.numel(s) for s in shapes]
    N = sum(numel)
    stream = W.AR1Stream(shapes, dtype, 0.95, 1e-3, config_id=4, device=DEV)
    ctx = B.Gac(numel, B.BF16, c_high=2.0)
    g = [torch.empty(s, dtype=dtype, device=DEV) for s in shapes]

    say("step 1")
    stream.next_into(g)
    g1 = U.clone_list(g)
    res = ctx.gac_step(g)
    torch.cuda.synchronize()
    assert (res.c, res.regime, res.dd, res.step) == (0.0, B.SAFE, 0.0, 1)
    assert all(U.bits_equal(a, b) for a, b in zip(g, g1))

    say("step 2: GPU")
    stream.next_into(g)
    g2 = U.clone_list(g)
    res = ctx.gac_step(g)
    torch.cuda.synchronize()
    assert res.regime == B.PROJECT and res.step == 2
    assert abs(res.c - 0.95) <= 5 * (1 - 0.95 ** 2) / math.sqrt(N) + 2e-3
    say("step 2: oracle sums over all elements")
    g_h, d_h, s, dec = oracle_decision(g2, g1, dtype, C_LOW, 2.0)
    check_result(res, s, dec)
    # sampled tensors: embedding (largest), first layer q k v o gate up down norm norm, final norm
    sample = [0] + list(range(2, 11)) + [len(shapes) - 1]
    say("step 2: oracle projection on sampled tensors")
    err = check_projection(g, g_h, d_h, s, dec, dtype, sample)
    say(f"  c={res.c:.6f} alpha={res.alpha:.6f} rel-L2(sample)={err:.2e}")
    del g_h, d_h
    # properties over ALL elements (fp64 on the GPU): only the component along d changed,
    # and it was brought to sign(c) c_low |g|
    dot_gp_d = sum(float(torch.dot(a.reshape(-1).double(), b.reshape(-1).double())) for a, b in zip(g, g1))
    norm_d, norm_g = math.sqrt(res.dd), math.sqrt(res.gg)
    assert dot_gp_d / norm_d == pytest.approx(math.copysign(C_LOW, res.c) * norm_g, rel=2e-3)
    sq = sum(float(torch.dot(a.reshape(-1).double(), a.reshape(-1).double())) for a in g)
    assert sq == pytest.approx(res.gg * (1 - res.c ** 2 + C_LOW ** 2), rel=2e-3)
    state = [torch.empty_like(t) for t in g]
    ctx.gac_state_export(state)
    torch.cuda.synchronize()
    assert all(U.bits_equal(a, b) for a, b in zip(state, g2)), "state must be the raw g of step 2"
    del state, g1

    say("step 3")
    ctx.gac_set_thresholds(C_LOW, C_HIGH)
    stream.next_into(g)
    g3 = U.clone_list(g)
    res3 = ctx.gac_step(g)
    torch.cuda.synchronize()
    assert res3.regime == B.SKIP and res3.step == 3
    assert res3.dd == res.gg  # the same vector, reduced twice in the same order: same bits
    assert abs(res3.c - 0.95) <= 5 * (1 - 0.95 ** 2) / math.sqrt(N) + 2e-3
    assert all(U.bits_equal(a, b) for a, b in zip(g, g3))
    state = [torch.empty_like(t) for t in g]
    ctx.gac_state_export(state)
    torch.cuda.synchronize()
    assert all(U.bits_equal(a, b) for a, b in zip(state, g3))
    ctx.close()
