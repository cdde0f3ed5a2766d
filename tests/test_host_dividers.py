"""The host-prepared index dividers (fast_div_setup) are exact: a C++ host program built from
the library's own header brute-forces them.  No GPU: only the host half of the header is used."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None,
                    reason="needs hipcc for the HIP runtime headers the library header includes")
def test_index_dividers_are_exact(tmp_path):
    exe = str(tmp_path / "dividers")
    hipcc = HIPCC if os.path.exists(HIPCC) else shutil.which("hipcc")
    # host compilation only: no device code is generated, nothing here touches a GPU
    subprocess.run([hipcc, "-std=c++20", "-O2", "-x", "c++", "-D__HIP_PLATFORM_AMD__",
                    "-I", os.path.join(ROOT, "paper_2004_11077_amd", "csrc"),
                    "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
                    os.path.join(ROOT, "tests", "host", "dividers.cpp"), "-o", exe],
                   check=True, capture_output=True, text=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    word, divisors, checks = run.stdout.split()
    assert word == "ok" and int(divisors) > 90000 and int(checks) > 10 ** 7
