"""GPU test of gac_step_static, the step for callers that cannot allocate: called through the C
ABI and compared with gac_step (a context with the same configuration and caller-owned state)
bit for bit - result record, gradient, state - on calls in a row that share the library's one
static device array, the second on a smaller input than the first.  gac_step itself is checked
against the oracle here as everywhere else."""
import ctypes

import pytest
import torch

from paper_2603_01501_amd import binding as B
from paper_2603_01501_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
EPS = 1e-8

# first call: 300 tensors (four batches of the tensor table) with ragged tails, an empty tensor
# and several multi-chunk tensors; second call: a smaller list
BIG = [(5,), (0,), (2049,), (70001,), (300, 301)] + [(1000 + 37 * j,) for j in range(295)]
SMALL = [(4097,), (33,), (40000,)]


def same_record(a, b):
    for name, _ in B.GacResult._fields_:
        assert getattr(a, name) == getattr(b, name), (name, getattr(a, name), getattr(b, name))


def run_case(shapes, dtype, rho, c_low, c_high, step, **kw):
    """One update through both entry points on the same inputs."""
    numel = [W.numel(s) for s in shapes]
    code = U.code(dtype)
    g0, d0 = W.correlated_pair(shapes, dtype, rho, 1e-3, config_id=41, device=DEV)
    # the context-based entry point, checked against the oracle
    d_ref, g_ref = U.clone_list(d0), U.clone_list(g0)
    ctx = B.Gac(numel, code, c_low=c_low, c_high=c_high, eps=EPS, state=d_ref, **kw)
    ctx.gac_state_import(d0, step - 1)
    want = ctx.gac_step(g_ref)
    torch.cuda.synchronize()
    if not kw.get("max_grad_norm"):  # (clipping against the oracle: test_gpu_clip_diag.py)
        U.check_step(want, g0, d0, g_ref, d_ref, dtype, c_low, c_high, EPS)
    # the entry point that allocates nothing
    d_st, g_st = U.clone_list(d0), U.clone_list(g0)
    out = torch.zeros(ctypes.sizeof(B.GacResult), dtype=torch.uint8, device=DEV)
    cfg, keep = B.make_config(numel, code, c_low=c_low, c_high=c_high, eps=EPS, state=d_st, **kw)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]  # the driver's figure, not the caching allocator's
    assert B.gac_step_static(cfg, g_st, step, out) == B.OK
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before, "the call took device memory"
    got = U.read_device_record(out.data_ptr())
    same_record(want, got)
    assert all(U.bits_equal(a, b) for a, b in zip(g_st, g_ref)), "gradients differ"
    assert all(U.bits_equal(a, b) for a, b in zip(d_st, d_ref)), "states differ"
    ctx.close()
    return got


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_static_step_equals_context_step_on_calls_in_a_row(dtype):
    r = run_case(BIG, dtype, 0.15, 0.05, 0.3, step=1)
    assert r.regime == B.PROJECT and r.step == 1
    r = run_case(SMALL, dtype, 0.15, 0.05, 0.3, step=2)      # smaller input, same static array
    assert r.regime == B.PROJECT and r.step == 2
    r = run_case(SMALL, dtype, 0.0, 0.05, 0.3, step=3)
    assert r.regime == B.SAFE
    r = run_case(BIG, dtype, 0.9, 0.05, 0.3, step=4)
    assert r.regime == B.SKIP
    # tuning fields and clipping are honoured like in gac_init
    r = run_case(BIG, dtype, 0.15, 0.05, 0.3, step=5, chunk_elems=2048, grid_blocks=7, apply_blocks=5,
                 max_grad_norm=1e-3)
    assert r.regime == B.PROJECT and r.clip_coef < 1.0
    # empty list
    cfg, keep = B.make_config([], U.code(dtype), state=[])
    out = torch.zeros(ctypes.sizeof(B.GacResult), dtype=torch.uint8, device=DEV)
    assert B.gac_step_static(cfg, [], 9, out) == B.OK
    torch.cuda.synchronize()
    rec = U.read_device_record(out.data_ptr())
    assert (rec.c, rec.regime, rec.step) == (0.0, B.SAFE, 9)


def test_static_step_replayed_from_a_hip_graph():
    """gac_step_static only launches kernels, so a caller under stream capture can record it.
    Captured once (after one eager call, which also settles the library's per-device set-up) and
    replayed with eager work and synchronisations in between, every replay must equal gac_step
    on the same inputs; the step number is an argument and therefore the captured one."""
    dtype = torch.bfloat16
    shapes = [(70000,), (33,), (0,), (4096,), (9001,)] + [(257 + j,) for j in range(120)]  # two table batches
    numel = [W.numel(s) for s in shapes]
    code = U.code(dtype)
    src = W.AR1Stream(shapes, dtype, 0.2, 1e-3, config_id=43, device=DEV)
    g = [torch.empty(s, dtype=dtype, device=DEV) for s in shapes]
    d = [torch.zeros(s, dtype=dtype, device=DEV) for s in shapes]
    out = torch.zeros(ctypes.sizeof(B.GacResult), dtype=torch.uint8, device=DEV)
    cfg, keep = B.make_config(numel, code, c_low=0.05, c_high=0.3, eps=EPS, state=d)
    ref = B.Gac(numel, code, c_low=0.05, c_high=0.3, eps=EPS)
    src.next_into(g)
    ref.gac_step(U.clone_list(g))
    B.gac_step_static(cfg, g, 1, out)       # eager: the first reference is the first gradient
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    src.next_into(g)
    g_in = U.clone_list(g)
    with torch.cuda.graph(graph, stream=side):
        B.gac_step_static(cfg, g, 7, out, stream=torch.cuda.current_stream())
    regimes = []
    for i in range(4):
        if i:
            src.next_into(g)
            g_in = U.clone_list(g)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        g_ref = U.clone_list(g_in)
        want = ref.gac_step(g_ref)
        torch.cuda.synchronize()
        got = U.read_device_record(out.data_ptr())
        assert got.step == 7
        for name, _ in B.GacResult._fields_:
            if name != "step":
                assert getattr(want, name) == getattr(got, name), (i, name)
        assert all(U.bits_equal(a, b) for a, b in zip(g, g_ref)), f"replay {i}"
        assert all(U.bits_equal(a, b) for a, b in zip(d, g_in)), f"replay {i}: state"
        regimes.append(got.regime)
        _ = sum(float(t.float().sum()) for t in g)  # eager work between replays
    assert B.PROJECT in regimes
    ref.close()


def test_static_step_rejects_what_does_not_fit():
    n = B.STATIC_MAX_TENSORS + 1
    bufs = [torch.zeros(8, device=DEV) for _ in range(2)]
    state = [bufs[0]] * n
    grads = [bufs[1]] * n
    cfg, keep = B.make_config([8] * n, B.F32, state=state)
    with pytest.raises(B.GacError) as e:
        B.gac_step_static(cfg, grads, 1)
    assert e.value.code == B.ERR_TOO_LARGE
    assert b"capacity" in B.lib().gac_strerror(B.ERR_TOO_LARGE)
    cfg, keep = B.make_config([8], B.F32, state=bufs[:1], grid_blocks=1025)
    with pytest.raises(B.GacError) as e:
        B.gac_step_static(cfg, bufs[1:], 1)
    assert e.value.code == B.ERR_TOO_LARGE
    # the other checks of gac_init and gac_step apply as well
    for bad in (dict(c_low=0.3, c_high=0.3), dict(eps=-1.0)):
        cfg, keep = B.make_config([8], B.F32, state=bufs[:1], **bad)
        with pytest.raises(B.GacError) as e:
            B.gac_step_static(cfg, bufs[1:], 1)
        assert e.value.code == B.ERR_BAD_THRESHOLDS
    for bad, grads in ((dict(), bufs[:1]), (dict(flags=1), bufs[1:]), (dict(history_capacity=8), bufs[1:])):
        cfg, keep = B.make_config([8], B.F32, state=bufs[:1], **bad)
        with pytest.raises(B.GacError) as e:
            B.gac_step_static(cfg, grads, 1)
        assert e.value.code == B.ERR_INVALID_ARG
    cfg, keep = B.make_config([8], B.F32)  # no state given
    with pytest.raises(B.GacError) as e:
        B.gac_step_static(cfg, bufs[1:], 1)
    assert e.value.code == B.ERR_INVALID_ARG
    # nothing above launched anything: the buffers are untouched
    torch.cuda.synchronize()
    assert float(bufs[0].abs().sum()) == 0.0 and float(bufs[1].abs().sum()) == 0.0
