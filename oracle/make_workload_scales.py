"""Writes workload_scales.json: the per-tensor scales of every benchmark workload.

Oracle-side script (test infrastructure): it calls only the oracle and the
seeded input generator.  Each scale is calibrated stage after stage with the
oracle's rule (scale = float32(max|real| / qmax)) on the seeded tensors, and
stored as the exact float32 value (repr of its double).  The benchmark and the
tests read the file as caller-supplied inputs of the library.

    python -m oracle.make_workload_scales
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402
from oracle import quantised as q  # noqa: E402


def main():
    out = {}
    for name, wl in si.WORKLOADS.items():
        L = si.make_layer(wl)
        cfg = q.LayerConfig(m=wl.m, base=wl.base, bits_hadamard=wl.bits_hadamard, out_type="i8")
        _, sc = q.run_layer(L["xq"], L["wq"], L["s_x"], L["s_w"], cfg)
        out[name] = {k: float(v) for k, v in sc.items()}
        print(name, out[name], flush=True)
    with open(os.path.join(ROOT, "workload_scales.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)


if __name__ == "__main__":
    main()
