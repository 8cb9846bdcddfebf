"""Host check of the division shortcuts in the quantizer kernel (no GPU): compiles and runs
tests/host/quant_division_check.c, which compares them with IEEE fp32 division."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _cpu_has_fma():
    try:
        with open("/proc/cpuinfo") as f:
            return any(" fma" in line for line in f if line.startswith("flags"))
    except OSError:
        return False


@pytest.mark.skipif(shutil.which("gcc") is None or not _cpu_has_fma(), reason="needs gcc and a CPU with fused multiply-add")
def test_division_shortcuts_match_ieee_division(tmp_path):
    exe = str(tmp_path / "quant_division_check")
    subprocess.run(["gcc", "-O2", "-mfma", "-ffp-contract=off", os.path.join(HERE, "host", "quant_division_check.c"),
                    "-o", exe, "-lm"], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.count("0 mismatches") >= 3 and "code quotients" in r.stdout, r.stdout
