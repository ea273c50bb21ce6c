"""The compress kernels take the group scale, range / levels (Sec. 3.2), with one FMA correction step
instead of a division sequence.  scale_division_check.c shows on the host that the step returns the
correctly rounded binary32 quotient: here for every 64th binary32 numerator up to 2^17 and for every
difference and sum of binary16 values of neighbouring binades (about a second); run it with stride 1
for every numerator (a minute).  The kernels themselves are compared with the oracle's division in the
GPU parity tests (test_scale_for_every_binary16_range)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_fma_correction_step_is_the_correctly_rounded_quotient(tmp_path):
    exe = str(tmp_path / "scale_division_check")
    subprocess.run(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-o", exe,
                    os.path.join(HERE, "scale_division_check.c"), "-lm"], check=True)
    res = subprocess.run([exe, "64"], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.count("0 mismatches") == 3, res.stdout
