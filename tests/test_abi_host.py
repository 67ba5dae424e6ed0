"""CPU-only checks of the C-ABI library: it loads, it exports every function that
include/gac.h declares, and the host logic that runs before any GPU call behaves
(argument validation, threshold validation per Section 4.2, chunk planning)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2603_01501_amd import binding as B
from paper_2603_01501_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gac_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 23 and "gac_threshold_sweep" in names and "gac_place_state" in names and "gac_init" in names and "gac_step" in names
    for n in names:
        assert hasattr(L, n), f"libgac.so does not export {n}"
    assert B.lib().gac_version().decode().startswith("gac-mi355x")


def test_struct_layouts_match_header(tmp_path):
    """Sizes and field offsets of the ctypes mirrors against what a C compiler makes of gac.h."""
    structs = {"gac_config": B.GacConfig, "gac_result": B.GacResult, "gac_diag": B.GacDiag,
               "gac_adamw_hyper": B.GacAdamWHyper, "gac_placement": B.GacPlacement}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "gac.h"', 'int main(void) {']
    for cname, cls in structs.items():
        lines.append(f'  printf("{cname} size %zu\\n", sizeof({cname}));')
        for fname, _ in cls._fields_:
            lines.append(f'  printf("{cname} {fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    seen = 0
    for line in out.splitlines():
        cname, field, value = line.split()
        cls = structs[cname]
        want = ctypes.sizeof(cls) if field == "size" else getattr(cls, field).offset
        assert int(value) == want, line
        seen += 1
    assert seen == sum(len(c._fields_) + 1 for c in structs.values())
    assert ctypes.sizeof(B.GacResult) == 104  # the static scratch reserves 128 bytes for it


def test_default_config_is_the_papers():
    cfg = B.GacConfig()
    B.lib().gac_default_config(ctypes.byref(cfg))
    # Appendix C "GAC thresholds": c_low 0.05, c_high 0.3, eps 1e-8; Appendix A.2: beta 1
    assert (cfg.c_low, cfg.c_high, cfg.eps, cfg.beta) == (0.05, 0.3, 1e-8, 1.0)
    assert cfg.dtype == B.BF16 and cfg.n_tensors == 0 and cfg.device == -1


@pytest.mark.parametrize("c_low,c_high", [(0.0, 0.3), (-0.1, 0.3), (0.3, 0.3), (0.4, 0.3),
                                          (float("nan"), 0.3), (0.05, float("nan"))])
def test_bad_thresholds_are_rejected_before_any_gpu_call(c_low, c_high):
    with pytest.raises(B.GacError) as e:
        B.Gac([16], B.F32, c_low=c_low, c_high=c_high)
    assert e.value.code == B.ERR_BAD_THRESHOLDS


def test_bad_arguments():
    for kwargs in (dict(eps=-1.0), dict(beta=-0.5), dict(max_grad_norm=-1.0)):
        with pytest.raises(B.GacError) as e:
            B.Gac([16], B.F32, **kwargs)
        assert e.value.code == B.ERR_BAD_THRESHOLDS
    for args, kwargs in (([[16], 7], {}), ([[-1], B.F32], {}), ([[16], B.F32], dict(chunk_elems=1000))):
        with pytest.raises(B.GacError) as e:
            B.Gac(*args, **kwargs)
        assert e.value.code == B.ERR_INVALID_ARG
    assert B.lib().gac_init(None, None) == B.ERR_INVALID_ARG
    assert B.lib().gac_step(None, None, None, None) == B.ERR_INVALID_ARG
    B.lib().gac_destroy(None)
    assert b"c_low" in B.lib().gac_strerror(B.ERR_BAD_THRESHOLDS)


def test_plan_query_counts_chunks_without_straddling():
    # bf16 default chunk: 32768 elements; fp32: 16384
    assert B.gac_plan_query([32768, 1, 0, 32769], B.BF16) == (1 + 1 + 0 + 2, 65538)
    assert B.gac_plan_query([32768, 1, 0, 32769], B.F32) == (2 + 1 + 0 + 3, 65538)
    assert B.gac_plan_query([], B.F32) == (0, 0)
    assert B.gac_plan_query([5000], B.F32, 2048) == (3, 5000)
    with pytest.raises(B.GacError):
        B.gac_plan_query([5000], B.F32, 100)


def test_workload_shapes_match_the_stated_sizes():
    # tensor counts and element totals of the synthetic gradient lists
    cases = [(W.MODEL_05B, 218, 494_005_120), (W.MODEL_15B, 254, 1_543_656_960),
             (W.MODEL_76B, 255, 7_615_487_488), (W.MODEL_14B, 435, 14_769_689_600)]
    for model, n_tensors, total in cases:
        shapes = model.tensor_shapes()
        assert len(shapes) == n_tensors
        assert W.total_numel(shapes) == total
        nchunks, tot = B.gac_plan_query([W.numel(s) for s in shapes], B.BF16)
        assert tot == total and nchunks >= total // 32768
