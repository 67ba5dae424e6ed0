"""GPU parity of the two optional parts of the step: global-norm clipping folded into pass 2
(Table 2 lists gradient clipping as on) and the recorded cosines with the statistics of
Table 3.  Oracle: the unfused composition (GAC step, then clipping of what the optimizer
sees) and the plain sort-and-interpolate statistics."""
import ctypes
import math

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
SHAPES = [(1,), (2049,), (0,), (32769,), (333, 301), (5,), (70001,)]


def oracle_clipped(g, d, dtype, c_high, max_norm):
    dt = U.code(dtype)
    g_h, d_h = U.host_copies(g), U.host_copies(d)
    outs, s, dec = O.step(g_h, d_h, dt, C_LOW, c_high, EPS)
    scale, norm = (1.0, math.sqrt(sum(float(np.dot(a, a)) for a in outs)))
    if dec.regime != O.SKIP and max_norm > 0:
        scale, norm = O.clip(outs, max_norm)
    return outs, s, dec, scale, norm, g_h


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("rho,c_high,regime", [(0.15, 0.3, B.PROJECT), (0.0, 0.3, B.SAFE), (0.9, 0.3, B.SKIP)])
@pytest.mark.parametrize("clip_at", [0.5, 3.0])   # max norm as a multiple of the gradient's norm
def test_clipping_folded_into_the_step(dtype, rho, c_high, regime, clip_at):
    g, d0 = W.correlated_pair(SHAPES, dtype, rho, 1e-3, config_id=31, device=DEV)
    probe = oracle_clipped(g, d0, dtype, c_high, 0.0)
    max_norm = clip_at * probe[4]
    outs, s, dec, scale, norm, g_h = oracle_clipped(g, d0, dtype, c_high, max_norm)
    d = U.clone_list(d0)
    ctx = B.Gac([W.numel(x) for x in SHAPES], U.code(dtype), c_high=c_high, state=d, max_grad_norm=max_norm)
    ctx.gac_state_import(d0, 0)
    g_raw = U.clone_list(g)
    res = ctx.gac_step(g)
    torch.cuda.synchronize()
    assert res.regime == dec.regime == regime
    assert res.grad_norm == pytest.approx(norm, rel=1e-6)
    assert res.clip_coef == pytest.approx(scale, rel=1e-6)
    clipped = scale < 1.0
    assert clipped == (clip_at < 1.0 and regime != B.SKIP)
    assert res.modified == int(regime == B.PROJECT or clipped)
    if res.modified:
        # what pass 2 computes is scale (g + k d): every element and every tensor against the oracle
        k0 = (dec.alpha - 1.0) * s[0] / s[2] if dec.regime == O.PROJECT else 0.0
        assert U.rel_l2(g, outs) <= U.GRAD_TOL[U.code(dtype)]
        for j in range(len(SHAPES)):
            U.check_projected_tensor(g[j], outs[j], g_raw[j], d0[j], scale * k0, scale, U.code(dtype), f"tensor {j}")
    else:
        assert all(U.bits_equal(a, b) for a, b in zip(g, g_raw))
    # the reference state keeps the raw, unclipped gradient
    assert all(U.bits_equal(a, b) for a, b in zip(d, g_raw))


def test_clipping_in_the_exchange_form_and_fused_adamw():
    dtype = torch.bfloat16
    numel = [W.numel(x) for x in SHAPES]
    for rho, regime in ((0.0, B.SAFE), (0.15, B.PROJECT)):
        g, d0 = W.correlated_pair(SHAPES, dtype, rho, 1e-3, config_id=32, device=DEV)
        probe = oracle_clipped(g, d0, dtype, C_HIGH, 0.0)
        max_norm = 0.25 * probe[4]
        outs, s, dec, scale, norm, g_h = oracle_clipped(g, d0, dtype, C_HIGH, max_norm)
        # exchange form: the clipped gradient arrives in the returned buffers, also when safe
        d = U.clone_list(d0)
        ctx = B.Gac(numel, B.BF16, state=d, max_grad_norm=max_norm)
        ctx.gac_state_import(d0, 0)
        mine = U.clone_list(g)
        res, returned = ctx.gac_step_exchange(mine)
        torch.cuda.synchronize()
        assert res.regime == regime and res.modified == 1 and res.clip_coef == pytest.approx(scale, rel=1e-6)
        assert U.rel_l2(returned, outs) <= U.GRAD_TOL[B.BF16]
        k0 = (dec.alpha - 1.0) * s[0] / s[2] if dec.regime == O.PROJECT else 0.0
        for j in range(len(SHAPES)):
            U.check_projected_tensor(returned[j], outs[j], g[j], d0[j], scale * k0, scale, B.BF16, f"tensor {j}")
        assert all(U.bits_equal(a, b) for a, b in zip(mine, g))
        # fused AdamW consumes the clipped gradient
        gen = torch.Generator(device=DEV)
        gen.manual_seed(5)
        p = [torch.randn(x, generator=gen, device=DEV) * 0.02 for x in SHAPES]
        m = [torch.randn(x, generator=gen, device=DEV) * 1e-4 for x in SHAPES]
        v = [torch.rand(x, generator=gen, device=DEV) * 1e-6 for x in SHAPES]
        p0, m0, v0 = U.clone_list(p), U.clone_list(m), U.clone_list(v)
        d2 = U.clone_list(d0)
        ctx2 = B.Gac(numel, B.BF16, state=d2, max_grad_norm=max_norm)
        ctx2.gac_state_import(d0, 0)
        hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps_adam=1e-8, weight_decay=1e-2)
        r2 = ctx2.gac_step_adamw(U.clone_list(g), p, m, v, None, t_adam=1, **hp)
        torch.cuda.synchronize()
        assert r2.clip_coef == res.clip_coef
        for j, shp in enumerate(SHAPES):
            if not W.numel(shp):
                continue
            pj, mj, vj = (W.to_oracle_array(t[j]) for t in (p0, m0, v0))
            po, mo, vo = O.adamw(outs[j], pj, mj, vj, 1e-3, 0.9, 0.999, 1e-8, 1e-2, 1)
            pg, mg, vg = (t[j].cpu().reshape(-1).double().numpy() for t in (p, m, v))
            assert np.linalg.norm(mg - mo) <= 1e-6 * np.linalg.norm(mo)
            assert np.linalg.norm(vg - vo) <= 1e-6 * np.linalg.norm(vo)
            tol = U.adamw_param_tolerance(pj, mj, vo, outs[j], 1e-3, 0.9, 0.999, 1e-8, 1)
            assert np.max(np.abs(pg - po) - tol) <= 0.0


def run_recorded_sequence(n_steps=150, capacity=64):
    """A run with a mix of regimes and one non-finite step.  Returns the context, what the
    library reported per step and what the oracle computes per step from the same gradients
    (its reference is the previous finite raw gradient, as in the library)."""
    shapes = [(20000,), (33,), (4097,)]
    numel = [W.numel(x) for x in shapes]
    ctx = B.Gac(numel, B.F32, history_capacity=capacity)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    rhos = [0.0, 0.02, 0.1, -0.2, 0.5, 0.04, -0.03, 0.25, 0.9, 0.0]
    seen_c, seen_r, want_c, want_r = [], [], [], []
    prev = None
    d_h = [np.zeros(n, dtype=np.float32) for n in numel]
    for t in range(n_steps):
        z = [torch.randn(x, generator=gen, device=DEV) for x in shapes]
        rho = rhos[t % len(rhos)]
        g = z if prev is None else [rho * a + math.sqrt(1 - rho * rho) * b for a, b in zip(prev, z)]
        if t == 100:
            g[0][3] = float("nan")
        prev = [x.clone() for x in g] if t != 100 else prev
        g_h = U.host_copies(g)
        dec = O.decide(O.sums(g_h, d_h, B.F32), C_LOW, C_HIGH, EPS)
        want_c.append(dec.c)
        want_r.append(dec.regime)
        if not dec.nonfinite:
            d_h = g_h
        res = B.GacResult()
        rc = B.lib().gac_step(ctx._ctx, B.ptr_list(g), None, ctypes.byref(res))
        assert rc == (B.ERR_NONFINITE if dec.nonfinite else B.OK)
        seen_c.append(res.c)
        seen_r.append(res.regime)
    return ctx, seen_c, seen_r, np.array(want_c), want_r, prev


def close_or_both_nan(a, b, tol=1e-6):
    return (math.isnan(a) and math.isnan(b)) or abs(a - b) <= tol


def test_recorded_cosines_and_table3_statistics():
    n_steps = 150
    ctx, seen_c, seen_r, want_c, want_r, prev = run_recorded_sequence(n_steps, 64)
    assert all(close_or_both_nan(a, b) for a, b in zip(seen_c, want_c)) and seen_r == want_r
    # no oracle cosine sits within rounding of a threshold, so counts can be compared exactly
    finite = np.abs(want_c[~np.isnan(want_c)])
    assert np.min(np.abs(finite - C_LOW)) > 1e-5 and np.min(np.abs(finite - C_HIGH)) > 1e-5
    c_hist, r_hist, first = ctx.gac_history_read()
    assert first == n_steps - 64 + 1 and len(c_hist) == 64
    assert all((math.isnan(a) and math.isnan(b)) or a == b for a, b in zip(c_hist, seen_c[-64:]))
    assert r_hist == seen_r[-64:]
    assert ctx.gac_history_read(max_n=10)[2] == n_steps - 9
    for burn_in in (0, 95, 120, 149, 150, 400):
        d = ctx.gac_diag_summary(burn_in)
        lo = max(first, burn_in + 1)
        window = want_c[lo - 1:]
        q, mx, frac, m = O.alignment_stats(window, 0, C_LOW)
        assert (d.n_values, d.n_nonfinite) == (m, int(np.isnan(window).sum()))
        assert abs(d.q90_abs_c - q) <= 1e-6 and abs(d.max_abs_c - mx) <= 1e-6
        assert d.frac_le_c_low == pytest.approx(frac, rel=1e-15, abs=0)
        assert list(d.regime_count) == O.regime_counts(window, 0, C_LOW, C_HIGH)
        if m:
            assert (d.first_step, d.last_step) == (lo, n_steps)
    # records start again after a reset
    ctx.gac_reset()
    assert ctx.gac_history_read()[0] == [] and ctx.gac_diag_summary(0).n_values == 0
    res = ctx.gac_step(prev)
    assert ctx.gac_history_read() == ([0.0], [B.SAFE], 1)


def test_threshold_sweep_over_the_record():
    n_steps = 110           # step 101 is the non-finite one: no pair counts it
    ctx, seen_c, seen_r, want_c, want_r, prev = run_recorded_sequence(n_steps, 128)
    # a grid of the Table 4 kind around the defaults, plus a never-skip pair
    pairs = [(lo, hi) for lo in (0.01, 0.03, 0.05, 0.1, 0.2) for hi in (0.25, 0.3, 0.4, 0.6)] + [(0.05, 2.0)]
    finite = np.abs(want_c[~np.isnan(want_c)])
    for lo, hi in pairs:
        assert np.min(np.abs(finite - lo)) > 1e-5 and np.min(np.abs(finite - hi)) > 1e-5
    for burn_in in (0, 50, 100, 101, 110):
        got = ctx.gac_threshold_sweep(pairs, burn_in)
        assert got == [O.regime_counts(want_c, burn_in, lo, hi) for lo, hi in pairs]
        assert all(sum(x) == max(0, n_steps - burn_in - (burn_in <= 100)) for x in got)
    # the pair in force reproduces the regimes the steps actually took
    assert ctx.gac_threshold_sweep([(C_LOW, C_HIGH)])[0] == list(ctx.gac_diag_summary(0).regime_count)
    # inclusive ends (Section 4.2): a threshold equal to a recorded |c| counts that step as
    # safe (lower end) or as skipped (upper end)
    c_hist = [abs(c) for c in ctx.gac_history_read()[0] if not math.isnan(c)]
    x = sorted(c_hist)[len(c_hist) // 2]
    safe, proj, skip = ctx.gac_threshold_sweep([(x, 10.0)])[0]
    assert safe == sum(c <= x for c in c_hist) and skip == 0
    safe, proj, skip = ctx.gac_threshold_sweep([(1e-12, x)])[0]
    assert skip == sum(c >= x for c in c_hist)
    # a ring shorter than the run only sees its last entries
    ctx2, *_ = run_recorded_sequence(n_steps, 16)
    assert ctx2.gac_threshold_sweep(pairs[:3], 0) == \
        [O.regime_counts(want_c, n_steps - 16, lo, hi) for lo, hi in pairs[:3]]
    # argument checks
    for bad in ([(0.3, 0.3)], [(0.05, 0.3), (0.0, 0.3)], [(0.05, float("nan"))]):
        with pytest.raises(B.GacError) as e:
            ctx.gac_threshold_sweep(bad)
        assert e.value.code == B.ERR_BAD_THRESHOLDS
    for bad in ([], [(0.05, 0.3)] * 65):
        with pytest.raises(B.GacError) as e:
            ctx.gac_threshold_sweep(bad)
        assert e.value.code == B.ERR_INVALID_ARG
