"""Seeded synthetic layer inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the convolution method.  It only draws the
tensors a layer is fed with and casts them to the int8 codes the library's
boundary takes (activations NHWC int8, weights KCRS int8, one symmetric scale
each: scale = max|v| / 127, round half to even, codes in [-127, 127]).

The tensors stand in for CIFAR10 activations and trained ResNet18 weights,
which are not available here: only shapes and value distributions are kept.
Activations are half-normal |N(0,1)| (post-ReLU-like), weights N(0, 2/(9C))
(He initialisation of a 3x3 layer); ``outliers`` > 0 sets that fraction of the
activations (Bernoulli mask) to 8.0.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    H: int
    W: int
    C: int
    K: int
    m: int
    base: str = "legendre"
    bits_hadamard: int = 8
    seed: int = 0
    outliers: float = 0.0

    @property
    def tiles(self):
        return self.N * (-(-self.H // self.m)) * (-(-self.W // self.m))


# The benchmark configurations (ResNet18-on-32x32-image layer shapes).
WORKLOADS = {
    "cfg1_f2_canonical": Workload("cfg1_f2_canonical", 1, 8, 8, 16, 16, 2, "canonical", 8, 0),
    "cfg1_f2_legendre": Workload("cfg1_f2_legendre", 1, 8, 8, 16, 16, 2, "legendre", 8, 0),
    "cfg2_f4_c64": Workload("cfg2_f4_c64", 128, 32, 32, 64, 64, 4, "legendre", 8, 1),
    "cfg3_f4_c128_h9": Workload("cfg3_f4_c128_h9", 128, 16, 16, 128, 128, 4, "legendre", 9, 2),
    "cfg4a_f4_c256": Workload("cfg4a_f4_c256", 256, 8, 8, 256, 256, 4, "legendre", 8, 3, 0.01),
    "cfg4b_f4_c512": Workload("cfg4b_f4_c512", 256, 4, 4, 512, 512, 4, "legendre", 8, 3, 0.01),
    "cfg4a_f6_c256": Workload("cfg4a_f6_c256", 256, 8, 8, 256, 256, 6, "legendre", 8, 3, 0.01),
    "cfg4b_f6_c512": Workload("cfg4b_f6_c512", 256, 4, 4, 512, 512, 6, "legendre", 8, 3, 0.01),
}

# The 3x3 stride-1 layers of a ResNet18 for 32x32x3 images, as (C, K, H=W).
RESNET18_STACK = ([(3, 64, 32)] + [(64, 64, 32)] * 4 + [(128, 128, 16)] * 3
                  + [(256, 256, 8)] * 3 + [(512, 512, 4)] * 3)


def cast_int8(v):
    """Symmetric per-tensor int8 codes of a real tensor and their scale."""
    v = np.asarray(v, dtype=np.float32)
    amax = float(np.max(np.abs(v))) if v.size else 0.0
    s = np.float32(amax / 127.0) if amax > 0 else np.float32(1.0)
    q = np.clip(np.rint(v / s), -127, 127).astype(np.int8)
    return q, s


def make_real(N, H, W, C, K, seed, outliers=0.0, r=3):
    """fp32 activations [N,H,W,C] and weights [K,C,r,r]."""
    rng = np.random.default_rng(seed)
    x = np.abs(rng.standard_normal((N, H, W, C), dtype=np.float32))
    w = rng.standard_normal((K, C, r, r), dtype=np.float32) * np.float32(np.sqrt(2.0 / (9.0 * C)))
    if outliers > 0:
        mask = rng.random((N, H, W, C), dtype=np.float32) < outliers
        x = np.where(mask, np.float32(8.0), x)
    return x, w


def make_layer(wl):
    """dict(x, w: fp32; xq, wq: int8; s_x, s_w: float32) for a Workload."""
    x, w = make_real(wl.N, wl.H, wl.W, wl.C, wl.K, wl.seed, wl.outliers)
    xq, s_x = cast_int8(x)
    wq, s_w = cast_int8(w)
    return {"x": x, "w": w, "xq": xq, "wq": wq, "s_x": s_x, "s_w": s_w}


def workload_scales(name):
    """Caller-supplied scales of a benchmark workload (float values of float32
    scales), read from workload_scales.json beside this file."""
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_scales.json")
    with open(path) as f:
        return json.load(f)[name]
