"""The C ABI called from a plain C++ program (tests/c_abi_check.cpp: no Python binding, no
PyTorch in the process), on the hand-worked length-8 cases of tests/golden/: the expected
values there come from Eq. 1 / Appendix A.1, Section 4.2 and Eq. 4 by hand, not from any
implementation, so this checks the library against the paper directly."""
import os
import subprocess

import numpy as np
import pytest

from paper_2603_01501_amd import build as gac_build
from tests.golden_cases import load_cases

pytestmark = pytest.mark.gpu
REGIME = {"safe": 0, "project": 1, "skip": 2}


def bf16_round(x):
    """Nearest bf16 (ties to even) of float32 values, as float64."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def run_case(case, dtype, entry="step"):
    if not os.path.exists(gac_build.C_CHECK_BIN):
        gac_build.build_c_abi_check()
    args = [gac_build.C_CHECK_BIN, f"{dtype}:{entry}", repr(case["eps"]), "0.05", "0.3", "8"]
    args += [repr(x) for x in case["d"]] + [repr(x) for x in case["g"]]
    r = subprocess.run(args, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    out = {}
    for line in r.stdout.splitlines():
        key, val = line.split(":", 1)
        out[key] = [float(x) for x in val.split()]
    return out


@pytest.mark.parametrize("entry", ["step", "static", "snapshot"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", load_cases(), ids=lambda c: c["case"])
def test_plain_c_caller_matches_hand_worked_case(case, dtype, entry):
    """gac_step, gac_step_static (no context, nothing allocated) and gac_step on a snapshot-form
    context, each from plain C on the hand-worked cases."""
    out = run_case(case, dtype, entry)
    assert out["sums"] == case["sums"]                      # small integers: exact
    assert out["c"][0] == pytest.approx(case["c"], abs=1e-12)
    assert int(out["regime"][0]) == REGIME[case["regime"]]
    assert out["alpha"][0] == pytest.approx(case["alpha"], rel=1e-12)
    assert int(out["step"][0]) == 1
    want = np.array(case["gprime"])
    got = np.array(out["gprime"])
    if dtype == "f32":
        assert np.max(np.abs(got - want)) <= 2e-7 * np.max(np.abs(want))
    else:
        # one bf16 rounding of the fp32 result; allow the neighbouring code where the
        # exact value sits within fp32 error of a rounding boundary
        near = bf16_round(want)
        assert np.all(np.abs(got - want) <= np.abs(near - want) + 1e-6 * np.abs(want) + 1e-12)
    assert out["state"] == case["g"]                        # the raw gradient, bit for bit
