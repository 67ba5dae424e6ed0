#!/usr/bin/env python3
"""GAC step benchmark on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7.6B|1.5B|0.5B|flat]

A "step" is one whole GAC update through the C ABI (reduce + finalize + apply) on one
synthetic gradient list already resident in HBM.  Consecutive gradients come from an AR(1)
stream (phi = 0.95) so the reference state carries from step to step; the next gradient is
generated between steps, outside the timed region, and every step is bracketed by a device
synchronisation on both sides; the step time is taken between two events recorded on the stream
right before and after the call.  The headline line uses thresholds (c_low, c_high) = (0.05, 2.0)
so that the projection branch (the full 6 N s bytes: cosine + projection + state update)
runs; the same workload under the paper's default thresholds (0.05, 0.3), where such aligned
gradients are skipped (4 N s bytes), is reported in "paper_default_thresholds".

The headline is timed with the library's state where gac_init allocated it.  Afterwards the
library is asked to place its state buffer (gac_place_state: it times both passes with the state
at successive allocations and keeps the fastest) and the projection step is timed again;
"state_placement" in the output holds what was timed and chosen and the step time after it
(a secondary figure: since pass 2 draws its chunks in order the two differ by under 1 %);
--no-placement skips it.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="7.6B",
                    choices=["7.6B", "1.5B", "0.5B", "flat", "14B-adamw", "7.6B-adamw", "1.5B-adamw"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-placement", action="store_true",
                    help="skip the secondary measurement after gac_place_state")
    ap.add_argument("--chunk-elems", type=int, default=0)
    ap.add_argument("--grid-blocks", type=int, default=0)
    ap.add_argument("--apply-blocks", type=int, default=0)
    ap.add_argument("--free-gb", type=float, default=0.0,
                    help="hold a ballast (2 GiB pieces) so that only this much device memory is free "
                         "when the library is initialised: what gac_place_state can do next to a trainer")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the steps, run one plain copy of known size (gac_state_export of "
                         "the whole state: N*s bytes read, N*s written) so that a counter "
                         "profile of this command can scale its byte counters")
    return ap.parse_args()


def workload(name):
    import torch
    from paper_2603_01501_amd import workloads as W
    if name == "7.6B":
        return W.MODEL_76B.tensor_shapes(), torch.bfloat16, 4, "7.6B-style gradient list (255 tensors)"
    if name == "1.5B":
        return W.MODEL_15B.tensor_shapes(), torch.bfloat16, 3, "1.5B-style gradient list (254 tensors)"
    if name == "0.5B":
        return W.MODEL_05B.tensor_shapes(), torch.float32, 2, "0.5B-style gradient list (218 tensors)"
    return [(W.FLAT_N,)], torch.float32, 1, "flat vector"


def recorded_traffic(kernel_src_sha, workload_name):
    """HBM bytes per apply-kernel launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE,
    scaled by a copy kernel of known size) on this workload; null for a workload without a
    counter summary, and unless the recorded figures belong to the kernel source as it is now."""
    name = {"7.6B": "apply_kernel_7.6B_bf16_pmc.txt", "0.5B": "apply_kernel_0.5B_fp32_pmc.txt",
            "14B-adamw": "apply_adamw_kernel_14B_bf16_pmc.txt"}.get(workload_name)
    if name is None:
        return None
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            vals[k.strip()] = v.strip()
    if vals.get("kernel_code_sha256") != kernel_src_sha:
        return None
    try:
        return float(vals["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def timed_steps(ctx, stream, g, n_steps, torch):
    """Runs n_steps GAC steps.  Returns (GPU ms per step, wall ms per step, last result): the
    first from a pair of events recorded on the stream the library launches on, right before
    and right after the call (the step as the GPU sees it: the reduction's first wave to the
    in-place pass's last), the second from the host clock around the call and a device
    synchronisation on both sides (adds the launch latency and the wake-up of the waiting host
    thread)."""
    from paper_2603_01501_amd import binding as B
    gpu_ms, wall_ms, res = [], [], None
    g_ptrs = B.ptr_list(g)              # the gradient buffers do not move between steps
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(n_steps)]
    for e0, e1 in events:
        stream.next_into(g)             # untimed: the next gradient of the AR(1) stream
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        res = ctx.gac_step(g_ptrs)      # waits for the regime, like a training loop would
        e1.record()
        torch.cuda.synchronize()
        wall_ms.append((time.perf_counter() - t0) * 1e3)
    gpu_ms = [e0.elapsed_time(e1) for e0, e1 in events]
    return gpu_ms, wall_ms, res


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(shapes, dtype, torch):
    """The oracle, as it is, on one host core, on the leading tensors of the same list."""
    from oracle import gac_oracle as O
    from paper_2603_01501_amd import binding as B
    from paper_2603_01501_amd import workloads as W
    budget, take, n = 1_200_000_000, [], 0
    for s in shapes:
        if take and n + W.numel(s) > budget:
            break
        take.append(s)
        n += W.numel(s)
    g, d = W.correlated_pair(take, dtype, 0.15, 1e-3, config_id=40, device="cuda:0")
    g_h = [W.to_oracle_array(t) for t in g]
    d_h = [W.to_oracle_array(t) for t in d]
    del g, d
    torch.cuda.empty_cache()
    code = B.torch_dtype_code(dtype)
    # repeat the step on the same sample until about 10 s of CPU work have been timed
    reps, total = 0, 0.0
    while total < 10.0 and reps < 8:
        d_run = [a.copy() for a in d_h]  # the oracle overwrites the state in place
        t0 = time.perf_counter()
        _, _, dec = O.step(g_h, d_run, code, 0.05, 0.3, 1e-8)
        total += time.perf_counter() - t0
        reps += 1
        assert dec.regime == O.PROJECT
    dt = total / reps
    es = 2 if dtype == torch.bfloat16 else 4
    return {"value": 6.0 * n * es / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"one projection-regime step on the first {len(take)} tensors of the list "
                      f"({n} elements), mean of {reps} runs, {dt:.1f} s each, single-threaded",
            "ms_per_step_extrapolated": dt * 1e3 * (sum(W.numel(s) for s in shapes) / n),
            "host_cpus": os.cpu_count(), "cpu_model": cpu_model()}


def main_adamw(args):
    """GAC fused with AdamW (gac_step_adamw) on a bf16 gradient list with fp32 m, v and master
    parameters.  Consecutive gradients are g_t = 0.9 d + sqrt(1 - 0.81) std n_t, where d is the
    reference state (the previous raw gradient), generated between steps outside the timed
    region; thresholds (0.05, 2.0) so that the projection branch and the optimizer both run."""
    import math
    import torch
    from paper_2603_01501_amd import binding as B
    from paper_2603_01501_amd import build as gac_build
    from paper_2603_01501_amd import workloads as W
    model = {"14B-adamw": W.MODEL_14B, "7.6B-adamw": W.MODEL_76B, "1.5B-adamw": W.MODEL_15B}[args.workload]
    shapes = model.tensor_shapes()
    numel = [W.numel(s) for s in shapes]
    N = sum(numel)
    dev = "cuda:0"
    dtype = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.tensor_seed(5, 0))
    d = [torch.empty(s, dtype=dtype, device=dev) for s in shapes]
    g = [torch.empty(s, dtype=dtype, device=dev) for s in shapes]
    # one list after the other (parameters, then first moments, then second moments): the three
    # arrays of a tensor then sit in different parts of HBM, which the fused pass prefers (~2 %)
    p = [torch.randn(s, generator=gen, device=dev).mul_(0.02) for s in shapes]
    m = [torch.randn(s, generator=gen, device=dev).mul_(1e-4) for s in shapes]
    v = [torch.rand(s, generator=gen, device=dev).mul_(1e-6) for s in shapes]

    def next_gradient(first):
        w = math.sqrt(1.0 - 0.81) * 1e-3
        for gj, dj in zip(g, d):
            z = torch.randn(gj.shape, generator=gen, device=dev, dtype=torch.float32)
            if first:
                gj.copy_(z.mul_(1e-3))
            else:
                gj.copy_(z.mul_(w).add_(dj.float(), alpha=0.9))
            del z

    ctx = B.Gac(numel, B.BF16, c_low=0.05, c_high=2.0, state=d, chunk_elems=args.chunk_elems,
                grid_blocks=args.grid_blocks, apply_blocks=args.apply_blocks)
    ptrs = [B.ptr_list(x) for x in (g, p, m, v)]
    hyper = dict(lr=1e-6, beta1=0.9, beta2=0.999, eps_adam=1e-8, weight_decay=1e-2)  # Table 2
    ms, res, t_adam = [], None, 0
    for i in range(1 + args.warmup + args.steps):
        next_gradient(i == 0)
        if i == 1 + args.warmup:
            ctx.gac_profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = ctx.gac_step_adamw(ptrs[0], ptrs[1], ptrs[2], ptrs[3], None, t_adam=t_adam + 1, **hyper)
        torch.cuda.synchronize()
        if i > args.warmup:
            ms.append((time.perf_counter() - t0) * 1e3)
        if res.regime != B.SKIP:
            t_adam += 1
    assert res.regime == B.PROJECT, (res.regime, res.c)
    k_red, k_fin, k_app, n = ctx.gac_profile_read()
    if args.calibration_copy:
        # one plain copy of known size for a counter profile of this command: the state of a
        # second, small context (2^30 bf16 elements: 2 GiB read, 2 GiB written) is exported
        side = B.Gac([1 << 30], B.BF16)
        dst = [torch.empty(1 << 30, dtype=dtype, device=dev)]
        side.gac_state_export(dst)
        torch.cuda.synchronize()
        side.close()
        del dst
    ms_step = sum(ms) / len(ms)
    red_bytes, app_bytes = 4.0 * N, 30.0 * N  # bf16 g,d read; + fp32 p,m,v read and written, d written
    out = {"metric": "fused GAC + AdamW step ms and achieved HBM GB/s", "value": (red_bytes + app_bytes) / ms_step / 1e6,
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{model.name}-style list, {len(shapes)} tensors, N={N}, bf16 g and d, fp32 m, v, p; "
                                  "phi=0.9 consecutive gradients, thresholds (0.05, 2.0): projection regime, "
                                  "34 bytes per element per step", "cosine": res.c, "t_adam": t_adam},
           "roofline": {"bound": "hbm", "kernel": "apply_adamw_kernel", "achieved": app_bytes / (k_app / n) / 1e6,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": app_bytes / (k_app / n) / 1e6 / HBM_PEAK_GBS,
                        "traffic": recorded_traffic(gac_build.kernel_code_sha256(), args.workload),
                        "algorithmic_bytes_per_launch": app_bytes, "avg_launch_ms": k_app / n},
           "kernels": {"reduce_kernel": {"avg_ms": k_red / n, "GBps": red_bytes / (k_red / n) / 1e6},
                       "apply_adamw_kernel": {"avg_ms": k_app / n, "GBps": app_bytes / (k_app / n) / 1e6}}}
    print(json.dumps(out), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU GAC step; run it with --gpus 1 "
              "(the sharded form needs only a 3-scalar all-reduce and is not benchmarked here)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_01501_amd import binding as B
    from paper_2603_01501_amd import build as gac_build
    from paper_2603_01501_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload.endswith("-adamw"):
        return main_adamw(args)
    shapes, dtype, config_id, desc = workload(args.workload)
    numel = [W.numel(s) for s in shapes]
    N = sum(numel)
    es = 2 if dtype == torch.bfloat16 else 4
    code = B.torch_dtype_code(dtype)
    storage = str(dtype).split(".")[-1]
    GiB = float(2 ** 30)

    stream = W.AR1Stream(shapes, dtype, 0.95, 1e-3, config_id=config_id, device="cuda:0")
    g = [torch.empty(s, dtype=dtype, device="cuda:0") for s in shapes]

    # --free-gb: what a trainer's parameters, optimizer state and activations would leave.  The
    # ballast is taken in 2 GiB pieces before the library allocates anything.
    ballast = []
    if args.free_gb > 0:
        torch.cuda.synchronize()
        free_now = torch.cuda.mem_get_info()[0]
        take = free_now - int(args.free_gb * GiB)
        while take > 0:
            piece = min(take, 2 * 2 ** 30)
            ballast.append(torch.empty(piece, dtype=torch.uint8, device="cuda:0"))
            take -= piece
    free_at_init = torch.cuda.mem_get_info()[0]

    def settle(ctx, strm, freed_bytes, limit_s=20.0):
        """Untimed: steps until the step time is steady.  After large frees (the placement
        search) the driver clears the freed device memory in the background, which takes HBM
        bandwidth from whatever runs meanwhile: measured ~2.5 s per 100 GB, so wait at least
        4 s per 100 GB freed, then until two batches of steps agree."""
        t0 = time.perf_counter()
        min_s = 1.0 + 4.0 * freed_bytes / 100e9
        prev = None
        while time.perf_counter() - t0 < limit_s:
            ms, _, _ = timed_steps(ctx, strm, g, 4, torch)
            cur = min(ms)
            steady = prev is not None and abs(cur - prev) <= 0.003 * prev
            if steady and time.perf_counter() - t0 >= min_s:
                break
            prev = cur
            time.sleep(0.25)

    def summary(ms):
        return {"mean": sum(ms) / len(ms), "min": min(ms), "median": sorted(ms)[len(ms) // 2]}

    def measure(ctx, strm, steps, want_regime, bytes_per_step, kernel_split=True):
        """`steps` timed steps with nothing but the step in the stream, then (kernel_split) as
        many again with the library's per-kernel events switched on."""
        gpu_ms, wall_ms, res = timed_steps(ctx, strm, g, steps, torch)
        assert res.regime == want_regime, f"expected regime {want_regime}, got {res.regime} (c={res.c})"
        out = {"regime": B.REGIME_NAMES[res.regime], "cosine": res.c,
               "ms_per_step": summary(gpu_ms)["mean"], "ms_per_step_min": min(gpu_ms),
               "ms_per_step_median": summary(gpu_ms)["median"], "ms_per_step_wall": summary(wall_ms)["mean"],
               "bytes_per_step": bytes_per_step,
               "GBps": bytes_per_step / summary(gpu_ms)["mean"] / 1e6}
        if kernel_split:
            ctx.gac_profile_enable(True)
            timed_steps(ctx, strm, g, steps, torch)
            k_red, k_fin, k_app, n = ctx.gac_profile_read()
            ctx.gac_profile_enable(False)
            out["kernel_ms"] = {"reduce": k_red / n, "apply": k_app / n}
        return out

    # ---- one context for the in-place form, with the state where gac_init allocated it
    ctx = B.Gac(numel, code, c_low=0.05, c_high=2.0, chunk_elems=args.chunk_elems,
                grid_blocks=args.grid_blocks, apply_blocks=args.apply_blocks)
    # step 1 meets a zero reference and is always safe; it is part of the warm-up
    timed_steps(ctx, stream, g, 1 + args.warmup, torch)

    # headline: projection regime, 6 N s bytes
    head = measure(ctx, stream, args.steps, B.PROJECT, 6.0 * N * es)
    ms_step = head["ms_per_step"]
    value = head["GBps"]
    ms_red, ms_app = head["kernel_ms"]["reduce"], head["kernel_ms"]["apply"]

    # the same gradients under the paper's thresholds (Appendix C): aligned like this they are skipped
    n_side = max(3, min(8, args.steps))
    ctx.gac_set_thresholds(0.05, 0.3)
    skip = measure(ctx, stream, n_side, B.SKIP, 4.0 * N * es)
    if args.calibration_copy:
        ctx.gac_state_export(g)
        torch.cuda.synchronize()

    placement = None
    if not args.no_placement:
        # Secondary measurement: the library is asked to find the best place for its state
        # relative to these gradient buffers (gac_place_state) and the projection step is timed
        # again.  Not part of the headline: it needs spare device memory during the search.
        ctx.gac_set_thresholds(0.05, 2.0)
        rep = ctx.gac_place_state(g)
        settle(ctx, stream, float(rep.bytes_held_peak))
        placed = measure(ctx, stream, n_side, B.PROJECT, 6.0 * N * es)
        ctx.gac_set_thresholds(0.05, 0.3)
        placement = {
            "what": "gac_place_state (set-up call, after the headline was timed): times the two passes with the "
                    "state at successive allocations and keeps the fastest, then tunes the workgroup count of "
                    "the in-place pass; 'after' is the projection step timed again",
            "candidates_timed": rep.n_candidates, "chosen": rep.chosen,
            "apply_probe_ms": [round(rep.probe_ms[i], 3) for i in range(rep.n_candidates)],
            "reduce_ms": [round(rep.reduce_ms[i], 3) for i in range(rep.n_candidates)],
            "apply_blocks": rep.apply_blocks,
            "blocks_tried": {int(rep.blocks_tried[i]): round(rep.blocks_ms[i], 3) for i in range(rep.n_blocks_tried)},
            "bytes_held_peak": rep.bytes_held_peak,
            "free_bytes_before_gac_init": free_at_init,
            "after": placed}

    if args.free_gb > 0:
        # memory-pressure mode: only the in-place form is measured (the other forms need a
        # second state buffer or caller-allocated state, for which there is no room)
        ctx.close()
        out = {"metric": "GAC step ms and achieved HBM GB/s (% of peak) with limited free device memory",
               "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
               "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
               "dtype": "f32", "storage_dtype": storage, "data": "synthetic",
               "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
               "config": {"workload": f"{desc}, N={N}, {storage} storage, AR(1) phi=0.95, thresholds (0.05, 2.0), "
                                      f"{args.free_gb} GiB of device memory free when the library is initialised",
                          "ms_per_step_wall": head["ms_per_step_wall"]},
               "kernels": {"reduce_kernel": {"avg_ms": ms_red}, "apply_kernel": {"avg_ms": ms_app}},
               "state_placement": placement, "paper_default_thresholds": skip}
        print(json.dumps(out), flush=True)
        return

    # consecutive gradients with correlation 0.15: inside the paper's projection band, so the
    # projection kernel runs with the paper's own thresholds
    del stream
    torch.cuda.empty_cache()
    stream15 = W.AR1Stream(shapes, dtype, 0.15, 1e-3, config_id=config_id + 20, device="cuda:0")
    timed_steps(ctx, stream15, g, 2, torch)  # the first one meets the other stream's last gradient
    rho015 = measure(ctx, stream15, n_side, B.PROJECT, 6.0 * N * es)
    ctx.close()
    torch.cuda.empty_cache()

    # ---- snapshot form: two library-owned state buffers, the snapshot written by pass 1
    snap = B.Gac(numel, code, c_low=0.05, c_high=0.3, chunk_elems=args.chunk_elems,
                 grid_blocks=args.grid_blocks, apply_blocks=args.apply_blocks,
                 flags=B.FLAG_SNAPSHOT_IN_REDUCE)
    timed_steps(snap, stream15, g, 3, torch)
    snap_proj = measure(snap, stream15, n_side, B.PROJECT, 6.0 * N * es)
    snap.gac_set_thresholds(0.2, 0.3)      # |c| = 0.15 <= c_low: the safe regime
    snap_safe = measure(snap, stream15, n_side, B.SAFE, 3.0 * N * es)
    snap.close()
    del stream15
    torch.cuda.empty_cache()
    stream = W.AR1Stream(shapes, dtype, 0.95, 1e-3, config_id=config_id, device="cuda:0")

    def run_exchange(c_high, warmup, steps):
        """The same steps through gac_step_exchange: buffers change hands, no snapshot copy."""
        state = [torch.zeros(s, dtype=dtype, device="cuda:0") for s in shapes]
        xctx = B.Gac(numel, code, c_low=0.05, c_high=c_high, state=state, chunk_elems=args.chunk_elems,
                     grid_blocks=args.grid_blocks, apply_blocks=args.apply_blocks)
        mine, ms, res = g, [], None
        for i in range(1 + warmup + steps):
            stream.next_into(mine)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            res, mine = xctx.gac_step_exchange(mine)
            e1.record()
            torch.cuda.synchronize()
            if i > warmup:
                ms.append(e0.elapsed_time(e1))
        xctx.close()
        del state, mine
        torch.cuda.empty_cache()
        return ms, res

    ms_xp, res_xp = run_exchange(2.0, 1, n_side)
    g = [torch.empty(s, dtype=dtype, device="cuda:0") for s in shapes]  # the old ones changed hands
    ms_xs, res_xs = run_exchange(0.3, 1, n_side)
    assert res_xp.regime == B.PROJECT and res_xs.regime == B.SKIP

    sha = gac_build.kernel_code_sha256()
    apply_bytes = 4.0 * N * es
    achieved = apply_bytes / (ms_app * 1e-3) / 1e9
    out = {
        "metric": "GAC step ms and achieved HBM GB/s (% of peak) on 7.6B-param bf16 gradient"
                  if args.workload == "7.6B" else f"GAC step ms and achieved HBM GB/s (% of peak) on {desc}",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "storage_dtype": storage, "data": "synthetic",
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "timing": "value, ms_per_step and pct_of_hbm_peak are WHOLE-STEP figures (6*N*s bytes over the time "
                  "between two events on the library's stream around gac_step, mean of the timed steps); "
                  "ms_per_step_wall is the host clock around the same call with a device synchronisation "
                  "on both sides; roofline.* is for ONE kernel (the in-place pass), timed in a second loop "
                  "of the same length with the library's per-kernel events on",
        "config": {"workload": f"{desc}, N={N}, {storage} storage, AR(1) phi=0.95, "
                               "thresholds (0.05, 2.0): projection regime, 6*N*s bytes per step",
                   "n_tensors": len(shapes), "numel": N, "bytes_per_step": 6.0 * N * es,
                   "cosine": head["cosine"], "regime": head["regime"],
                   "ms_per_step_min": head["ms_per_step_min"], "ms_per_step_median": head["ms_per_step_median"],
                   "ms_per_step_wall": head["ms_per_step_wall"],
                   "free_gb_requested": args.free_gb if args.free_gb > 0 else None},
        "roofline": {"bound": "hbm", "kernel": "apply_kernel (projection + state update)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": recorded_traffic(sha, args.workload),
                     "algorithmic_bytes_per_launch": apply_bytes, "avg_launch_ms": ms_app},
        "kernels": {"reduce_kernel (with the finalize step in its last workgroup)":
                        {"avg_ms": ms_red, "bytes": 2.0 * N * es, "GBps": 2.0 * N * es / (ms_red * 1e-3) / 1e9},
                    "apply_kernel": {"avg_ms": ms_app, "bytes": apply_bytes, "GBps": achieved}},
        "state_placement": placement,
        "paper_default_thresholds": {"thresholds": [0.05, 0.3], **skip,
                                     "what": "the same phi=0.95 gradients: skipped, reduction + state copy"},
        "paper_default_thresholds_rho015": {"thresholds": [0.05, 0.3], **rho015,
                                            "what": "AR(1) phi=0.15 gradients: projected under the paper's own thresholds"},
        "snapshot_form": {"what": "GAC_FLAG_SNAPSHOT_IN_REDUCE: pass 1 writes the snapshot; a step that neither "
                                  "projects nor clips has no pass 2 (state not placed: gac_place_state does "
                                  "not cover this form)",
                          "safe_phi015_thresholds_0.2_0.3": snap_safe,
                          "projection_phi015_paper_thresholds": snap_proj},
        "exchange_form": {"what": "gac_step_exchange: the gradient buffers become the reference state and "
                                  "the old state buffers come back (holding g' when projected)",
                          "projection": {"ms_per_step": sum(ms_xp) / len(ms_xp), "bytes_per_step": 5.0 * N * es,
                                         "GBps": 5.0 * N * es / (sum(ms_xp) / len(ms_xp)) / 1e6},
                          "paper_default_thresholds_skip": {"ms_per_step": sum(ms_xs) / len(ms_xs),
                                                            "bytes_per_step": 2.0 * N * es,
                                                            "GBps": 2.0 * N * es / (sum(ms_xs) / len(ms_xs)) / 1e6}},
    }
    del ballast
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shapes, dtype, torch)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
