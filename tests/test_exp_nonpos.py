"""The verification kernels' own double-precision exponential (csrc/exp_nonpos.h) against the long-double library
routine.  The header is plain C on the host side: this test compiles tests/exp_nonpos_check.c with the host compiler,
runs it over its fixed grid (1.2e7 arguments in [-745, 0], the switching points of the argument reduction, special
values) and holds the routine to the error bound it states: at most 1.05 units in the last place for normal results
(every decision of the layer-wise verification sits on sums of these values; the CPU oracle uses numpy's exp, and
the two must agree far inside the 1e-6 band in which accept decisions are exempt from bit-exactness)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs a host C compiler")
def test_exp_nonpos_against_long_double_exp(tmp_path):
    exe = str(tmp_path / "exp_nonpos_check")
    src = os.path.join(ROOT, "tests", "exp_nonpos_check.c")
    inc = os.path.join(ROOT, "paper_2409_16560_amd", "csrc")
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-I" + inc, "-o", exe, src, "-lm"], check=True)
    out = subprocess.run([exe], check=True, stdout=subprocess.PIPE, text=True, timeout=600).stdout
    vals = {l.split()[0]: l.split()[1] for l in out.splitlines() if l.strip()}
    print(out)
    assert int(vals["points"]) > 12_000_000
    assert float(vals["worst_normal_ulp"]) <= 1.05
    assert float(vals["worst_denormal_ulp"]) <= 1.5
    assert float(vals["exp0"]) == 1.0 and float(vals["exp_minus_1e6"]) == 0.0
    assert int(vals["monotone_violations"]) == 0
