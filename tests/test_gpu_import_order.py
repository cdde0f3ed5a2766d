"""The library must work whichever of PyTorch and the package is imported (and used) first."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

CODE = """
import paper_2004_11077_amd as wn
d = wn.ConvDesc(1, 8, 8, 16, 16, m=4)
assert wn.wino_workspace_bytes(d) > 0          # loads libwino.so before PyTorch is imported
import torch
sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
assert wn.wino_probe_peak(wn.PROBE_VALU_MAD24, 8, 16, sink) == 8 * 256 * 16 * 8
torch.cuda.synchronize()
assert int(sink.item()) == 0
print("ok")
"""


def test_package_used_before_torch_is_imported():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", CODE], cwd=root, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
