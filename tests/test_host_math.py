"""Host checks of arithmetic identities the kernels rely on (no GPU)."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _cpu_has_fma():
    try:
        with open("/proc/cpuinfo") as f:
            return any(" fma " in line + " " for line in f if line.startswith("flags"))
    except OSError:
        return False


@pytest.mark.skipif(not _cpu_has_fma(), reason="needs a hardware fused multiply-add")
def test_reciprocal_division_is_exact_for_all_fp16_pairs(tmp_path):
    exe = str(tmp_path / "check_exact_division")
    subprocess.run(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
                    os.path.join(HERE, "check_exact_division.c"), "-o", exe, "-lm"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == 0x7bff * 0x7c00      # every finite s > 0 times every finite v >= 0
    assert int(out[1]) == 0
