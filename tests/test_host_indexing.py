"""Host arithmetic the kernels' indexing rests on, checked by C++ host programs built from the
library's own header: the prepared index dividers (fast_div_setup) against plain division, and
the dealing of the transforms' work groups to XCDs (a one-to-one map that keeps a unit of
tiles on one XCD, the same XCD in every stage kernel where the library says so).  No GPU: only the host half of the header is used."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


needs_hipcc = pytest.mark.skipif(
    not os.path.exists(HIPCC) and shutil.which("hipcc") is None,
    reason="needs hipcc for the HIP runtime headers the library header includes")


def run_host_program(tmp_path, name):
    exe = str(tmp_path / name)
    hipcc = HIPCC if os.path.exists(HIPCC) else shutil.which("hipcc")
    # host compilation only: no device code is generated, nothing here touches a GPU
    subprocess.run([hipcc, "-std=c++20", "-O2", "-x", "c++", "-D__HIP_PLATFORM_AMD__",
                    "-I", os.path.join(ROOT, "paper_2004_11077_amd", "csrc"),
                    "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include",
                    os.path.join(ROOT, "tests", "host", name + ".cpp"), "-o", exe],
                   check=True, capture_output=True, text=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    return run.stdout.split()


@needs_hipcc
def test_index_dividers_are_exact(tmp_path):
    word, divisors, checks = run_host_program(tmp_path, "dividers")
    assert word == "ok" and int(divisors) > 90000 and int(checks) > 10 ** 7


@needs_hipcc
def test_work_groups_are_dealt_one_to_one_with_a_unit_on_one_xcd(tmp_path):
    word, shapes, dealt, aligned = run_host_program(tmp_path, "image_groups")
    assert word == "ok" and int(shapes) == 2 * 3 * 9 * 7 * 7 and int(dealt) > 300 and int(aligned) > 10
