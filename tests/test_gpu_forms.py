"""GPU tests of the forms of the step that keep state differently from the default one:
checkpoint / resume (export the reference state and the step count, import them into a fresh
context: Algorithm 1's loop carries g_{t-1} and t, Appendix A.2 calls the former a snapshot)
and the snapshot form (two state buffers, the snapshot written by pass 1).  Both are compared
with an uninterrupted default context bit for bit, and that one with the oracle."""
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
DTYPES = [torch.float32, torch.bfloat16]

# a scaled-down policy plus ragged extras: a 5-element tensor, an empty one, one that ends one
# element past a vector boundary, one that spans several chunks with a ragged tail
SHAPES = W.scaled_down(W.MODEL_76B, 28, layers=1, vocab=2001).tensor_shapes() + [(5,), (0,), (2049,), (70001,)]
NUMEL = [W.numel(s) for s in SHAPES]


def new_ctx(dtype, state=None, **kw):
    return B.Gac(NUMEL, U.code(dtype), state=state, **kw)


def exported(ctx, dtype):
    out = [torch.empty(s, dtype=dtype, device=DEV) for s in SHAPES]
    step = ctx.gac_state_export(out)
    torch.cuda.synchronize()
    return out, step


def same_record(a, b):
    """Every field of two result records, bit for bit (NaN == NaN)."""
    for name, _ in B.GacResult._fields_:
        x, y = getattr(a, name), getattr(b, name)
        if isinstance(x, float) and math.isnan(x) and math.isnan(y):
            continue
        assert x == y, (name, x, y)


def close_record(a, b):
    """Two result records of the same step from forms that add the same products in different
    (each fixed) groupings: decisions equal, sums equal up to the rounding of the fp32 group
    sums and of the fp64 additions (each form is compared with the oracle separately)."""
    assert (a.regime, a.nonfinite, a.modified, a.step) == (b.regime, b.nonfinite, b.modified, b.step)
    if a.nonfinite:
        return
    scale = math.sqrt(a.gg * a.dd)
    assert abs(a.dot - b.dot) <= 1e-8 * max(scale, abs(a.dot))
    assert abs(a.gg - b.gg) <= 1e-8 * a.gg and abs(a.dd - b.dd) <= 1e-8 * a.dd
    assert abs(a.c - b.c) <= 1e-8
    for name in ("alpha", "coef", "grad_norm", "clip_coef", "scale_g", "coef_d"):
        x, y = getattr(a, name), getattr(b, name)
        assert abs(x - y) <= 1e-6 * max(abs(x), abs(y)), (name, x, y)


# ------------------------------------------------------------------ checkpoint / resume

@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
@pytest.mark.parametrize("caller_state", [False, True], ids=["library_state", "caller_state"])
def test_resumed_run_reproduces_the_uninterrupted_one(dtype, caller_state):
    """k steps, export (state, step count), destroy; a fresh context imports both and gets the
    same next gradients as a twin that never stopped: cosine, coefficient, step number,
    projected gradient and state agree bit for bit for four more steps, the record of c_t
    starts at step k+1, and the Table 3 statistics over the post-resume window match the
    oracle's."""
    k, more, cap = 7, 4, 32
    dt = U.code(dtype)
    stream = W.AR1Stream(SHAPES, dtype, 0.3, 1e-3, config_id=31, device=DEV)
    thresholds = dict(c_low=C_LOW, c_high=0.9)  # AR(1) with phi 0.3: the projection regime

    def fresh():
        state = [torch.zeros(s, dtype=dtype, device=DEV) for s in SHAPES] if caller_state else None
        return new_ctx(dtype, state=state, history_capacity=cap, **thresholds), state

    twin, twin_state = fresh()
    first, first_state = fresh()
    d_oracle = [np.zeros(n, dtype=np.uint16 if dtype == torch.bfloat16 else np.float32) for n in NUMEL]
    want_c = []
    for t in range(1, k + 1):
        g = stream.next()
        _, _, dec = O.step(U.host_copies(g), d_oracle, dt, C_LOW, 0.9, EPS)
        want_c.append(dec.c)
        r1 = twin.gac_step(U.clone_list(g))
        r2 = first.gac_step(g)
        same_record(r1, r2)
        assert abs(r1.c - dec.c) <= U.COS_TOL and r1.step == t
    saved, step = exported(first, dtype)
    assert step == k
    assert all(np.array_equal(W.to_oracle_array(a), b) for a, b in zip(saved, d_oracle))
    first.close()
    del first, first_state

    resumed, resumed_state = fresh()
    resumed.gac_state_import(saved, step)
    for t in range(k + 1, k + more + 1):
        g = stream.next()
        g_raw = U.clone_list(g)
        d_before = [W.from_bits(a, dtype).to(DEV) for a in d_oracle]
        outs, sums, dec = O.step(U.host_copies(g), d_oracle, dt, C_LOW, 0.9, EPS)
        want_c.append(dec.c)
        g_twin = U.clone_list(g)
        r1 = twin.gac_step(g_twin)
        r2 = resumed.gac_step(g)
        torch.cuda.synchronize()
        same_record(r1, r2)
        assert r2.step == t and r2.regime == dec.regime == B.PROJECT
        assert abs(r2.c - dec.c) <= U.COS_TOL
        assert all(U.bits_equal(a, b) for a, b in zip(g, g_twin)), "projected gradients differ"
        U.check_projected_list(g, outs, g_raw, d_before, sums, dec.alpha, 1.0, dt)
        s1, n1 = exported(twin, dtype)
        s2, n2 = exported(resumed, dtype)
        assert n1 == n2 == t
        assert all(U.bits_equal(a, b) for a, b in zip(s1, s2))
        assert all(U.bits_equal(a, b) for a, b in zip(s2, g_raw))
    # the record of the resumed context starts where it resumed
    c_hist, r_hist, first_step = resumed.gac_history_read()
    c_twin, r_twin, twin_first = twin.gac_history_read()
    assert first_step == k + 1 and twin_first == 1
    assert c_hist == c_twin[k:] and r_hist == r_twin[k:] and len(c_hist) == more
    # statistics over the post-resume window, with and without a burn-in that cuts into it
    for burn_in in (0, k, k + 2, k + more):
        d = resumed.gac_diag_summary(burn_in)
        lo = max(k + 1, burn_in + 1)
        window = np.array(want_c[lo - 1:])
        q, mx, frac, m = O.alignment_stats(window, 0, C_LOW)
        assert d.n_values == m == max(0, k + more - lo + 1) and d.n_nonfinite == 0
        assert abs(d.q90_abs_c - q) <= 1e-6 and abs(d.max_abs_c - mx) <= 1e-6
        assert d.frac_le_c_low == pytest.approx(frac, rel=1e-15, abs=0)
        assert list(d.regime_count) == O.regime_counts(window, 0, C_LOW, 0.9)
        if m:
            assert (d.first_step, d.last_step) == (lo, k + more)
        # the twin, asked for the same window, says the same
        if burn_in >= k:
            dtw = twin.gac_diag_summary(burn_in)
            assert (dtw.q90_abs_c, dtw.max_abs_c, dtw.n_values) == (d.q90_abs_c, d.max_abs_c, d.n_values)
    assert resumed.gac_threshold_sweep([(C_LOW, 0.9)], k)[0] == twin.gac_threshold_sweep([(C_LOW, 0.9)], k)[0]


def test_import_in_the_middle_of_a_ring_that_has_wrapped():
    """A resumed context whose ring is shorter than the steps since the resume reports only
    what the ring holds, with the right step numbers."""
    dtype = torch.float32
    cap = 4
    stream = W.AR1Stream(SHAPES, dtype, 0.3, 1e-3, config_id=32, device=DEV)
    ctx = new_ctx(dtype, history_capacity=cap, c_low=C_LOW, c_high=0.9)
    ctx.gac_state_import(stream.next(), 100)
    seen = []
    for _ in range(6):
        res = ctx.gac_step(stream.next())
        seen.append(res.c)
    assert res.step == 106
    c_hist, _, first = ctx.gac_history_read()
    assert (first, c_hist) == (103, seen[-4:])
    assert ctx.gac_history_read(max_n=2)[2] == 105
    d = ctx.gac_diag_summary(104)
    assert (d.first_step, d.last_step, d.n_values) == (105, 106, 2)
    with pytest.raises(B.GacError):
        ctx.gac_state_import(stream.next(), -1)


# ------------------------------------------------------------------ snapshot form

def step_both(ref, snap, g, dtype, lo, hi, d_before):
    """One step on the default context and on the snapshot-form context with the same
    gradient: each against the oracle (every element), and their records against each other
    (the two forms add the same products in different fixed orders)."""
    g_raw = U.clone_list(g)
    g_snap = U.clone_list(g)
    ref.gac_set_thresholds(lo, hi)
    snap.gac_set_thresholds(lo, hi)
    r1 = ref.gac_step(g)
    r2 = snap.gac_step(g_snap)
    torch.cuda.synchronize()
    state_ref, _ = exported(ref, dtype)
    U.check_step(r1, g_raw, d_before, g, state_ref, dtype, lo, hi, EPS)
    state_snap, n = exported(snap, dtype)
    assert n == r1.step
    U.check_step(r2, g_raw, d_before, g_snap, state_snap, dtype, lo, hi, EPS)
    close_record(r1, r2)
    return r1, state_ref


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
@pytest.mark.parametrize("chunk_elems,grid", [(0, 0), (2048, 3)])
def test_snapshot_form_matches_the_default_form(dtype, chunk_elems, grid):
    kw = dict(chunk_elems=chunk_elems, grid_blocks=grid, apply_blocks=grid)
    ref = new_ctx(dtype, **kw)
    snap = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, **kw)
    stream = W.AR1Stream(SHAPES, dtype, 0.3, 1e-3, config_id=33, device=DEV)
    thresholds = [(C_LOW, C_HIGH), (C_LOW, C_HIGH), (C_LOW, 0.9), (0.5, 0.9), (0.01, 0.2), (C_LOW, 0.9),
                  (C_LOW, 0.9)]
    d_before = [torch.zeros(s, dtype=dtype, device=DEV) for s in SHAPES]
    seen = set()
    for t, (lo, hi) in enumerate(thresholds, start=1):
        g = stream.next()
        r, d_before = step_both(ref, snap, g, dtype, lo, hi, d_before)
        assert r.step == t
        seen.add(r.regime)
    assert seen == {B.SAFE, B.PROJECT, B.SKIP}

    # a non-finite step changes neither the gradient nor the state, in either form
    g = stream.next()
    g[3].view(-1)[17] = float("inf")
    g_raw, g_snap = U.clone_list(g), U.clone_list(g)
    res = B.GacResult()
    for ctx, grads in ((ref, g), (snap, g_snap)):
        assert B.lib().gac_step(ctx._ctx, B.ptr_list(grads), None, ctypes.byref(res)) == B.ERR_NONFINITE
        assert res.nonfinite == 1 and res.regime == B.SKIP
    torch.cuda.synchronize()
    assert all(U.bits_equal(a, b) for a, b in zip(g_snap, g_raw))
    state_snap, _ = exported(snap, dtype)
    assert all(U.bits_equal(a, b) for a, b in zip(state_snap, d_before))
    # ... and the steps after it still agree (the spare buffer held the rejected gradient)
    for lo, hi in ((C_LOW, 0.9), (C_LOW, C_HIGH)):
        r, d_before = step_both(ref, snap, stream.next(), dtype, lo, hi, d_before)

    # import puts the state where the next step finds it, whichever buffer was current
    saved, step = exported(snap, dtype)
    for extra_steps in (0, 1):
        other = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, **kw)
        for _ in range(extra_steps):
            other.gac_step(stream.next())
        other.gac_state_import(saved, step)
        g = stream.next()
        g_a, g_b = U.clone_list(g), U.clone_list(g)
        ref.gac_state_import(saved, step)
        ref.gac_set_thresholds(C_LOW, 0.9)
        other.gac_set_thresholds(C_LOW, 0.9)
        r_a, r_b = ref.gac_step(g_a), other.gac_step(g_b)
        torch.cuda.synchronize()
        close_record(r_a, r_b)
        U.check_step(r_b, g, saved, g_b, exported(other, dtype)[0], dtype, C_LOW, 0.9, EPS)
    # reset: back to a zero reference
    snap.gac_reset()
    res = snap.gac_step(stream.next())
    assert (res.c, res.regime, res.dd, res.step) == (0.0, B.SAFE, 0.0, 1)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_snapshot_form_two_phase(dtype):
    """gac_reduce_local + gac_apply on a snapshot-form context is its gac_step."""
    one = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, c_high=0.9)
    two = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, c_high=0.9)
    stream = W.AR1Stream(SHAPES, dtype, 0.3, 1e-3, config_id=34, device=DEV)
    sums = torch.zeros(3, dtype=torch.float64, device=DEV)
    for t in range(1, 5):
        g = stream.next()
        g2 = U.clone_list(g)
        r1 = one.gac_step(g)
        two.gac_reduce_local(g2, sums)
        r2 = two.gac_apply(g2, sums)
        torch.cuda.synchronize()
        same_record(r1, r2)
        assert sums.tolist() == [r1.dot, r1.gg, r1.dd]
        assert all(U.bits_equal(a, b) for a, b in zip(g, g2))
        s1, _ = exported(one, dtype)
        s2, _ = exported(two, dtype)
        assert all(U.bits_equal(a, b) for a, b in zip(s1, s2))


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16"])
def test_snapshot_form_bits_do_not_depend_on_the_grid(dtype):
    """Every chunk has its own partial sums and they are combined in a fixed order, so the
    result is the same bit for bit on every run and for every number of workgroups."""
    stream = W.AR1Stream(SHAPES, dtype, 0.3, 1e-3, config_id=36, device=DEV)
    grads = [stream.next() for _ in range(3)]
    seen = []
    for grid, chunk in ((0, 0), (1, 0), (3, 0), (7, 0), (300, 0), (0, 0), (0, 2048), (5, 2048)):
        ctx = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, c_high=0.9, grid_blocks=grid, chunk_elems=chunk)
        out = []
        for g in grads:
            g_in = U.clone_list(g)
            r = ctx.gac_step(g_in)
            torch.cuda.synchronize()
            out.append((r.dot, r.gg, r.dd, r.c, r.coef, r.regime, [t.clone() for t in g_in]))
        seen.append((chunk, out))
        ctx.close()
    for chunk in (0, 2048):  # (the chunk size is part of the fixed order; the grid is not)
        runs = [o for c, o in seen if c == chunk]
        for other in runs[1:]:
            for a, b in zip(runs[0], other):
                assert a[:6] == b[:6]
                assert all(U.bits_equal(x, y) for x, y in zip(a[6], b[6]))
    assert B.PROJECT in [r[5] for r in seen[0][1]]


def test_snapshot_form_argument_checks():
    dtype = torch.float32
    state = [torch.zeros(s, dtype=dtype, device=DEV) for s in SHAPES]
    with pytest.raises(B.GacError) as e:  # needs two buffers of the library's own
        new_ctx(dtype, state=state, flags=B.FLAG_SNAPSHOT_IN_REDUCE)
    assert e.value.code == B.ERR_INVALID_ARG
    with pytest.raises(B.GacError) as e:
        new_ctx(dtype, flags=2)
    assert e.value.code == B.ERR_INVALID_ARG
    ctx = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE)
    g = [torch.zeros(s, dtype=dtype, device=DEV) for s in SHAPES]
    with pytest.raises(B.GacError) as e:
        ctx.gac_place_state(g)
    assert e.value.code == B.ERR_UNIMPLEMENTED
    p = [torch.zeros(s, dtype=torch.float32, device=DEV) for s in SHAPES]
    with pytest.raises(B.GacError) as e:
        ctx.gac_step_adamw(g, p, p, p, None, 1e-6, 0.9, 0.999, 1e-8, 1e-2, 1)
    assert e.value.code == B.ERR_UNIMPLEMENTED


def test_snapshot_form_replayed_from_a_hip_graph():
    """Which state buffer is current is device-side state, and so are the counters of its
    pass 1, so a captured asynchronous step can be replayed: every replay must equal an eager
    snapshot-form step on the same input, bit for bit."""
    dtype = torch.bfloat16
    stream = W.AR1Stream(SHAPES, dtype, 0.2, 1e-3, config_id=35, device=DEV)
    g = [torch.empty(s, dtype=dtype, device=DEV) for s in SHAPES]
    snap = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, c_high=0.9)
    ref = new_ctx(dtype, flags=B.FLAG_SNAPSHOT_IN_REDUCE, c_high=0.9, grid_blocks=5)
    stream.next_into(g)
    snap.gac_step(g, sync=False)  # the eager call uploads the pointer table (a capture cannot)
    ref.gac_step(U.clone_list(g))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        snap.gac_step(g, stream=torch.cuda.current_stream(), sync=False)
    res_dev = snap.gac_result_device()
    for t in range(2, 6):
        stream.next_into(g)
        g_ref = U.clone_list(g)
        g_raw = U.clone_list(g)
        r1 = ref.gac_step(g_ref)
        graph.replay()
        torch.cuda.synchronize()
        rec = U.read_device_record(res_dev)
        same_record(r1, rec)
        assert rec.step == t and rec.regime == B.PROJECT
        assert all(U.bits_equal(a, b) for a, b in zip(g, g_ref))
        state, n = exported(snap, dtype)
        assert n == t and all(U.bits_equal(a, b) for a, b in zip(state, g_raw))

