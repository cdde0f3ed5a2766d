#!/usr/bin/env python3
"""Benchmark of the quantised Legendre-base Winograd convolution layer on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
weight transform, input transform, per-point int8 MFMA contraction and output
transform of one 3x3 layer, inputs resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA, published
# Non-packed vector ALU issue rate: 256 CU x 64 lanes x 2.4 GHz lane-operations/s
# (the published 157.3 TFLOP/s fp32 figure counts packed 2-wide FMAs as 4 flops).
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12

MIN_TIMED_LAUNCHES = 200       # a reported step is the mean over at least this many steps
WARM_SECONDS = 0.3             # back-to-back steps before anything is timed, whatever --warmup says
STAGE_SAMPLES = 32             # event pairs per launch; the median is reported


def profile_counters(workload):
    """Per-launch counters from profiles/hbm_traffic_<workload>.txt (rocprofv3 --pmc runs of
    this program).  Lines ``TRAFFIC <launch> fetched_KiB=<f> written_KiB=<w>`` hold FETCH_SIZE /
    WRITE_SIZE per dispatch, already scaled by what the same counters read for a plain device
    copy of known size in the same run; lines ``VALU <launch> instructions=<n>`` hold
    SQ_INSTS_VALU per dispatch (wave-level vector instructions).  Returns (bytes per launch,
    vector instructions per launch); empty where the file has no such line."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    traffic, valu = {}, {}
    if os.path.exists(path):
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and parts[0] == "TRAFFIC":
                    kv = dict(p.split("=") for p in parts[2:])
                    traffic[parts[1]] = (float(kv["fetched_KiB"]) + float(kv["written_KiB"])) * 1024
                elif len(parts) == 3 and parts[0] == "VALU":
                    valu[parts[1]] = float(parts[2].split("=")[1])
    return traffic, valu


def stage_model(wl, m_bytes, y_bytes):
    """Algorithmic work of one launch of each kind (bytes, int8 ops)."""
    n = wl.m + 2
    T, C, K = wl.tiles, wl.C, wl.K
    model = _stage_bytes(wl, m_bytes, y_bytes, n, T, C, K)
    # a1 and a2 run as one launch
    model["operand_transforms"] = {
        "bound": "hbm",
        "work": model["weight_transform"]["work"] + model["input_transform"]["work"]}
    # a3 and a4 in one launch: the contraction's multiply-accumulates; U, V in and y out
    model["contraction_output"] = {
        "bound": "mfma", "work": model["contraction"]["work"],
        "bytes": n * n * (T * C + K * C) + T * K * wl.m * wl.m * y_bytes}
    # a2 + a3 + a4 in one launch: x, V in and y out
    model["fused_layer"] = {
        "bound": "mfma", "work": model["contraction"]["work"],
        "bytes": T * C * wl.m * wl.m + n * n * K * C + T * K * wl.m * wl.m * y_bytes}
    return model


def _stage_bytes(wl, m_bytes, y_bytes, n, T, C, K):
    return {
        # per (k, c): 9 filter bytes in, n*n transformed bytes out
        "weight_transform": {"bound": "hbm", "work": K * C * (9 + n * n)},
        # per (tile, c): m*m fresh input bytes in, n*n transformed bytes out
        "input_transform": {"bound": "hbm", "work": T * C * (wl.m * wl.m + n * n)},
        # Winograd-domain multiply-accumulates actually issued, 2 ops each
        "contraction": {"bound": "mfma", "work": 2 * n * n * T * C * K,
                        "bytes": n * n * (T * C + K * C + T * K * m_bytes)},
        # per (tile, k): n*n contraction results in, m*m outputs out
        "output_transform": {"bound": "hbm",
                             "work": T * K * (n * n * m_bytes + wl.m * wl.m * y_bytes)},
    }


def hip_runtime():
    """The HIP runtime already loaded into this process (by torch), for plain event calls."""
    path = None
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
    lib = ctypes.CDLL(path or "libamdhip64.so")
    lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                        ctypes.c_void_p]
    lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return lib


def timed(torch, fn, steps, min_launches=MIN_TIMED_LAUNCHES, warm_seconds=WARM_SECONDS,
          warmup=0):
    """Seconds per call of fn: warm-up by time (and at least `warmup` calls), then the mean
    over steps * inner back-to-back calls, inner chosen so that at least min_launches calls
    are timed.  Returns (seconds per call, inner, warm-up calls)."""
    warm, t_end = 0, time.perf_counter() + warm_seconds
    while warm < warmup or time.perf_counter() < t_end:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        warm += 10
    inner = max(1, -(-min_launches // max(1, steps)))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps * inner):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (steps * inner), inner, warm


def layer_times(wn, si, torch, dev, name, steps):
    """Step time of one whole layer (filters untransformed) through wino_conv2d."""
    wl = si.WORKLOADS[name]
    L = si.make_layer(wl)
    x = torch.from_numpy(L["xq"]).to(dev)
    w = torch.from_numpy(L["wq"]).to(dev)
    y = torch.empty((wl.N, wl.H, wl.W, wl.K), dtype=torch.float32, device=dev)
    base = wn.BASE_LEGENDRE if wl.base == "legendre" else wn.BASE_CANONICAL
    ops = 2.0 * wl.N * wl.H * wl.W * wl.C * wl.K * 9
    res = {}
    sc = None
    for label, mode in (("split", wn.FUSED_OFF), ("auto", wn.FUSED_AUTO)):
        desc = wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, m=wl.m, base=base,
                           bits_hadamard=wl.bits_hadamard, fused=mode)
        if sc is None:
            cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8,
                              device=dev)
            sc = wn.wino_calibrate(desc, x, w, None, float(L["s_x"]), float(L["s_w"]), cws)
            del cws
        ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        dt = timed(torch, lambda: wn.wino_conv2d(desc, x, w, y, sc, ws), steps)[0]
        res[label] = {"ms_per_step": dt * 1e3, "TOPS_direct_equiv": ops / dt / 1e12,
                      "launches": wn.wino_conv2d_launches(desc)}
    return res


def resnet18_stack(wn, si, torch, dev, steps, N=256):
    """The 14 stride-1 3x3 layers of the CIFAR ResNet18 (stem 3->64 at 32x32, 4 x 64 at 32x32,
    3 x 128 at 16x16, 3 x 256 at 8x8, 3 x 512 at 4x4), F(4x4,3x3) Legendre int8 with ReLU,
    int8 activations handed from layer to layer inside a resolution stage, filters transformed
    ahead of time, scales chosen by wino_calibrate, fused = AUTO.  Returns the time of one pass
    over all 14 layers."""
    import numpy as np
    layers, stage_in, ops = [], {}, 0.0
    for li, (C, K, HW) in enumerate(si.RESNET18_STACK):
        Cp = (C + 15) // 16 * 16                          # the stem's 3 channels are zero-padded
        if HW not in stage_in:                            # a stage starts from a fresh seeded tensor
            x0, _ = si.make_real(N, HW, HW, C, 1, seed=4)
            if Cp != C:
                x0 = np.concatenate([x0, np.zeros(x0.shape[:3] + (Cp - C,), np.float32)], axis=3)
            xq, s_x = si.cast_int8(x0)
            stage_in[HW] = (torch.from_numpy(xq).to(dev), float(s_x))
            x, s_in = stage_in[HW]
        _, w0 = si.make_real(1, 1, 1, C, K, seed=400 + HW + li)
        if Cp != C:
            w0 = np.concatenate([w0, np.zeros((K, Cp - C, 3, 3), np.float32)], axis=1)
        wq, s_w = si.cast_int8(w0)
        w = torch.from_numpy(wq).to(dev)
        desc = wn.ConvDesc(N, HW, HW, Cp, K, m=4, out_type=wn.OUT_I8, relu=1)
        y = torch.empty((N, HW, HW, K), dtype=torch.int8, device=dev)
        cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        sc = wn.wino_calibrate(desc, x, w, y, s_in, float(s_w), cws)
        del cws
        lay = wn.wino_preferred_operand_layout(desc)
        run = wn.ConvDesc(N, HW, HW, Cp, K, m=4, out_type=wn.OUT_I8, relu=1,
                          weights_pretransformed=1, fused=wn.FUSED_AUTO, operand_layout=lay)
        V = torch.empty((wn.wino_operand_bytes(run)[0],), dtype=torch.int8, device=dev)
        wn.wino_weight_transform(run, w, V, sc)
        ws = torch.empty(wn.wino_workspace_bytes(run), dtype=torch.uint8, device=dev)
        layers.append((run, x, V, y, sc, ws))
        ops += 2.0 * N * HW * HW * C * K * 9
        x, s_in = y, sc.s_y                               # this layer's codes feed the next one
    def once():
        for run, xi, V, y, sc, ws in layers:
            wn.wino_conv2d(run, xi, V, y, sc, ws)
    dt = timed(torch, once, steps, min_launches=40)[0]
    per_layer = []
    for (C, K, HW), (run, xi, V, y, sc, ws) in zip(si.RESNET18_STACK, layers):
        t = timed(torch, lambda: wn.wino_conv2d(run, xi, V, y, sc, ws), steps, min_launches=200)[0]
        per_layer.append({"C": C, "K": K, "HW": HW, "us": round(t * 1e6, 2),
                          "launches": wn.wino_conv2d_launches(run)})
    return {"ms_per_pass": dt * 1e3, "TOPS_direct_equiv": ops / dt / 1e12, "layers": len(layers),
            "N": N, "note": "int8 in, int8 + ReLU out, filters pretransformed, fused = AUTO",
            "per_layer": per_layer}


def cpu_baseline(wl, min_seconds=12.0):
    """The oracle, as it stands, timed on the host cores: whole passes over the full
    workload, repeated until about min_seconds of CPU work have been spent."""
    import synth_inputs as si
    from oracle import quantised as oq
    L = si.make_layer(wl)
    cfg = oq.LayerConfig(m=wl.m, base=wl.base, bits_hadamard=wl.bits_hadamard)
    scales = si.workload_scales(wl.name)
    passes, t0 = 0, time.perf_counter()
    while True:
        oq.run_layer(L["xq"], L["wq"], L["s_x"], L["s_w"], cfg, scales=scales)
        passes += 1
        total = time.perf_counter() - t0
        if total >= min_seconds or passes >= 64:
            break
    dt = total / passes
    ops = 2.0 * wl.N * wl.H * wl.W * wl.C * wl.K * 9
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": 1, "kind": "oracle",
            "sample": "full workload %s, %d passes in %.1f s, %.2f s per pass "
                      "(numpy int64, single thread)" % (wl.name, passes, total, dt),
            "host_cpus": len(os.sched_getaffinity(0))}


class Events:
    """Raw HIP events for the library's per-dispatch timing hook."""

    def __init__(self):
        self.hip = hip_runtime()

    def new(self):
        ev = ctypes.c_void_p()
        assert self.hip.hipEventCreate(ctypes.byref(ev)) == 0
        return ev

    def ms(self, a, b):
        out = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(out), a, b) == 0
        return out.value

    def free(self, evs):
        for ev in evs:
            self.hip.hipEventDestroy(ev)


def sample_launches(wn, torch, ev, call, n_launches, samples=STAGE_SAMPLES, gap=3):
    """Median duration (ms) of each of the n_launches kernels that `call` queues.  Every
    sampled call carries one event pair per launch, attached by the library to that very
    dispatch (wino_profile_next_launch -> hipExtLaunchKernel), so elapsed(start, stop) is the
    kernel's own begin-to-end time on its stream -- the interval rocprofv3 reports -- free of
    the marker overhead an event recorded between launches would add.  `gap` unsampled calls
    run between two sampled ones."""
    import numpy as np
    pairs = [[(ev.new(), ev.new()) for _ in range(n_launches)] for _ in range(samples)]
    for s in range(samples):
        for _ in range(gap):
            call()
        for a, b in pairs[s]:
            wn.wino_profile_next_launch(a.value, b.value)
        call()
    torch.cuda.synchronize()
    med = [float(np.median([ev.ms(*pairs[s][j]) for s in range(samples)]))
           for j in range(n_launches)]
    for row in pairs:
        for a, b in row:
            ev.free((a, b))
    return med


def price_stages(names, stage_ms, model, traffic, valu, measured_peaks):
    """Every launch against its ceilings.  Transforms are priced against HBM (algorithmic bytes
    over the kernel's duration), kernels that contain the contraction against the int8 MFMA
    peak (Winograd-domain multiply-accumulates actually issued).  Because the Legendre brackets
    are arithmetic-heavy, the rate at which the launch issued vector instructions is given
    beside it where the profile holds its instruction count (valu_issue_*: SQ_INSTS_VALU x 64
    lanes over the duration, against 256 CUs x 64 lanes x 2.4 GHz)."""
    stages = {}
    frag = "contraction_output" in names    # its operands are written in fragment order
    for nm in names:
        sec = stage_ms[nm] * 1e-3
        mdl = model[nm]
        st = {"ms": stage_ms[nm], "bound": mdl["bound"]}
        if mdl["bound"] == "hbm":
            hbm = mdl["work"] / sec / 1e9
            st.update({"achieved": hbm, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": hbm / HBM_PEAK_GBS, "algorithmic_bytes": mdl["work"],
                       "frac_of_measured_peak": hbm / measured_peaks["copy_GBps"]})
        elif "bytes" in mdl and (mdl["bytes"] / (HBM_PEAK_GBS * 1e9)
                                 > mdl["work"] / (INT8_MFMA_PEAK_TOPS * 1e12)):
            # the layer's arithmetic intensity is below the machine balance: moving the
            # algorithmic bytes at the HBM peak takes longer than the multiply-accumulates at
            # the MFMA peak, so HBM is the ceiling of this launch; the MFMA rate is given beside it
            hbm = mdl["bytes"] / sec / 1e9
            ach = mdl["work"] / sec / 1e12
            st.update({"bound": "hbm", "achieved": hbm, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": hbm / HBM_PEAK_GBS, "algorithmic_bytes": mdl["bytes"],
                       "frac_of_measured_peak": hbm / measured_peaks["copy_GBps"],
                       "algorithmic_ops": mdl["work"], "mfma_TOPs": ach,
                       "mfma_frac": ach / INT8_MFMA_PEAK_TOPS})
        else:
            ach = mdl["work"] / sec / 1e12
            st.update({"achieved": ach, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                       "frac": ach / INT8_MFMA_PEAK_TOPS, "algorithmic_ops": mdl["work"],
                       "frac_of_measured_peak": ach / measured_peaks["int8_mfma_TOPs"]})
            if "bytes" in mdl:
                st.update({"algorithmic_bytes": mdl["bytes"],
                           "hbm_GBps": mdl["bytes"] / sec / 1e9,
                           "hbm_frac": mdl["bytes"] / sec / 1e9 / HBM_PEAK_GBS})
        # counters of the fragment-order build of a transform, where the profile has them
        key = nm + "_fragments" if frag and (nm + "_fragments") in traffic else nm
        if key in valu:
            rate = valu[key] * 64 / sec / 1e12
            st.update({"valu_instructions": valu[key], "valu_issue_Tops": rate,
                       "valu_issue_frac": rate / VALU_PEAK_TOPS})
        st["traffic"] = traffic.get(key)
        stages[nm] = st
    return stages


def device_peaks(wn, torch, ev, dev, stream):
    """What this device sustains on the units the stages are priced against: register-only
    int8 / bf16 MFMA and 24-bit multiply-add loops (library probes, timed per dispatch) and a
    plain 256 MiB device copy (read + write bytes)."""
    def probe(kind, blocks, iters):
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        wn.wino_probe_peak(kind, blocks, iters, sink, stream)          # warm-up
        a, b = ev.new(), ev.new()
        wn.wino_profile_next_launch(a.value, b.value)
        work = wn.wino_probe_peak(kind, blocks, iters, sink, stream)
        torch.cuda.synchronize()
        ms = ev.ms(a, b)
        ev.free((a, b))
        return work / (ms * 1e-3) / 1e12
    src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return {"int8_mfma_TOPs": probe(wn.PROBE_MFMA_I8, 256 * 16, 2048),
            "valu_mad24_Tops": probe(wn.PROBE_VALU_MAD24, 256 * 16, 2048),
            "bf16_mfma_TFLOPs": probe(wn.PROBE_MFMA_BF16, 256 * 16, 2048),
            "copy_GBps": 2 * src.numel() * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9}


def measure_layer(wn, si, torch, ev, dev, wl_name, batch_scale, steps, warmup, mode, peaks,
                  copy_probe=False):
    """One whole-layer workload through wino_conv2d (filters untransformed): step time, the
    duration of each of its launches, and their roofline figures."""
    from fractions import Fraction
    base_wl = si.WORKLOADS[wl_name]
    wl = si.Workload(**{**base_wl.__dict__, "N": base_wl.N * batch_scale})
    L = si.make_layer(base_wl)
    x = torch.from_numpy(L["xq"]).to(dev).repeat(batch_scale, 1, 1, 1).contiguous()
    w = torch.from_numpy(L["wq"]).to(dev)
    base = wn.BASE_LEGENDRE if wl.base == "legendre" else wn.BASE_CANONICAL
    desc = wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, m=wl.m, base=base,
                       bits_hadamard=wl.bits_hadamard, out_type=wn.OUT_F32, fused=mode)
    # set-up, outside the timed region: the library chooses the layer's scales itself
    cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    sc = wn.wino_calibrate(desc, x, w, None, float(L["s_x"]), float(L["s_w"]), cws)
    del cws
    ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    y = torch.empty((wl.N, wl.H, wl.W, wl.K), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    names = wn.wino_conv2d_launches(desc)

    def step():
        wn.wino_conv2d(desc, x, w, y, sc, ws, stream)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step()                        # first launch of each kernel in this process
    torch.cuda.synchronize()
    cold_ms = (time.perf_counter() - t0) * 1e3
    sec, inner, warm = timed(torch, step, steps, warmup=warmup)
    if copy_probe:
        src = torch.ones(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    med = sample_launches(wn, torch, ev, step, len(names))
    stage_ms = dict(zip(names, med))
    pts = {2: [0, 1, -1], 4: [0, 1, -1, 2, -2], 6: [0, 1, -1, 2, -2, (1, 2), (-1, 2)]}[wl.m]
    mats = wn.wino_make_matrices(wl.m, 3, [Fraction(*p) if isinstance(p, tuple) else p
                                           for p in pts], base)
    m_bytes = {8: 1, 9: 2, 32: 4}[wl.bits_hadamard]
    model = stage_model(wl, m_bytes, 4)
    traffic, valu = profile_counters(base_wl.name)
    if batch_scale != 1:
        # byte counters are not carried over to another batch size; a wave's instruction
        # count does not depend on the batch, so the launch's count scales with it
        traffic, valu = {}, {k: v * batch_scale for k, v in valu.items()}
    stages = price_stages(names, stage_ms, model, traffic, valu, peaks)
    ops = 2.0 * wl.N * wl.H * wl.W * wl.C * wl.K * 9
    stage_sum = sum(med)
    res = {"workload": wl.name + ("" if batch_scale == 1 else "_batchx%d" % batch_scale),
           "wl": wl, "desc": desc, "x": x, "w": w, "y": y, "sc": sc, "L": L, "mats": mats,
           "ms_per_step": sec * 1e3, "value": ops / sec / 1e12, "ops": ops, "launches": names,
           "stages": stages, "stage_sum_ms": stage_sum,
           "stage_sum_exceeds_step": bool(stage_sum > 1.05 * sec * 1e3),
           "timing": {"timed_steps": steps * inner, "inner_repeats": inner, "warmup_steps": warm,
                      "stage_samples": STAGE_SAMPLES, "stage_statistic": "median"},
           "cold_step_ms": cold_ms}
    return res


def public(res):
    """The JSON-serialisable part of a measure_layer result."""
    keep = ("workload", "ms_per_step", "value", "launches", "stages", "stage_sum_ms",
            "stage_sum_exceeds_step", "timing", "cold_step_ms")
    out = {k: res[k] for k in keep}
    out["unit"] = "TOPS"
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg4a_f4_c256")
    ap.add_argument("--batch-scale", type=int, default=1,
                    help="multiply the batch size N (extra, labelled in config)")
    ap.add_argument("--mode", default="auto", choices=("auto", "split", "on"),
                    help="kernel selection of the headline step: the library's own choice "
                         "(fused = AUTO), one kernel per stage (OFF), or M kept on chip (ON)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the extra timings of the other layer configurations")
    ap.add_argument("--only-extra", default=None,
                    choices=("split", "batch64", "fused", "pretransformed", "per_point", "flex",
                             "backward", "others"),
                    help="run just this one of the extra measurements (for profiling it)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 64 MiB device copy after warm-up: the known-size "
                         "kernel against which rocprofv3 --pmc byte counters are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; a layer shards over the batch "
              "with no exchange step, so N GPUs would run N independent copies. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2004_11077_amd as wn

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    ev = Events()
    # a first burst of work so that the probes below do not see a cold device
    burn = torch.ones(64 << 20, dtype=torch.uint8, device=dev)
    for _ in range(20):
        burn.add_(1)
    torch.cuda.synchronize()
    del burn
    peaks = device_peaks(wn, torch, ev, dev, stream)

    mode = {"auto": wn.FUSED_AUTO, "split": wn.FUSED_OFF, "on": wn.FUSED_ON}[args.mode]
    head = measure_layer(wn, si, torch, ev, dev, args.workload, args.batch_scale, args.steps,
                         args.warmup, mode, peaks, copy_probe=args.copy_probe)
    wl, desc, x, w, y, sc, L, mats = (head[k] for k in ("wl", "desc", "x", "w", "y", "sc", "L",
                                                        "mats"))
    reps = args.batch_scale
    base = desc.base
    n2, T = desc.n ** 2, desc.tiles
    ops = head["ops"]
    stages = head["stages"]
    names = head["launches"]
    dominant = max(names, key=lambda nm: stages[nm]["ms"])
    roofline = {k: stages[dominant].get(k) for k in ("bound", "achieved", "peak", "unit", "frac",
                                                     "traffic")}
    roofline["kernel"] = dominant
    for k in ("frac_of_measured_peak", "algorithmic_bytes", "algorithmic_ops", "hbm_GBps",
              "hbm_frac", "mfma_TOPs", "mfma_frac", "valu_instructions", "valu_issue_Tops",
              "valu_issue_frac"):
        if k in stages[dominant]:
            roofline[k] = stages[dominant][k]

    out = {
        "metric": "int8 Winograd conv TOPS (direct-equiv)",
        "value": head["value"],
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": head["workload"],
                   "N": wl.N, "H": wl.H, "W": wl.W, "C": wl.C, "K": wl.K,
                   "algorithm": "F(%dx%d,3x3) %s base" % (wl.m, wl.m, wl.base),
                   "bits_hadamard": wl.bits_hadamard, "output": "fp32",
                   "step": "wino_conv2d, filters untransformed, fused = %s: %s"
                           % (args.mode.upper(), " + ".join(names))},
        "roofline": roofline,
        "stages": stages,
        "stage_sum_ms": head["stage_sum_ms"],
        "stage_sum_exceeds_step": head["stage_sum_exceeds_step"],
        "timing": head["timing"],
        "measured_peaks": peaks,
        "cold_step_ms": head["cold_step_ms"],
    }

    def want(name, always=False):
        if args.only_extra is not None:
            return args.only_extra == name
        return always or not args.no_extras

    steps = args.steps
    # extra: the same layer with one kernel per stage (a1 + a2 | a3 | a4): the contraction on
    # its own against the int8 MFMA peak, each transform on its own against HBM
    if want("split", always=True) and args.mode != "split" and "contraction" not in names:
        sp = measure_layer(wn, si, torch, ev, dev, args.workload, reps, steps, 0, wn.FUSED_OFF,
                           peaks)
        out["split_path"] = public(sp)
        del sp
    # extra: the same layer on 64 times the batch (x + U beyond twice the Infinity Cache), so
    # that kernel efficiency and launch effects can be told apart
    if want("batch64", always=True) and reps == 1:
        big = measure_layer(wn, si, torch, ev, dev, args.workload, 64, max(5, steps // 10), 0,
                            mode, peaks)
        out["batch_x64"] = public(big)
        del big
        torch.cuda.empty_cache()
    # extra: the same layer with its filters transformed ahead of time (a1 is a per-layer,
    # offline step in deployment)
    if want("pretransformed"):
        lay = wn.wino_preferred_operand_layout(desc) if mode == wn.FUSED_AUTO else wn.LAYOUT_ROWS
        pdesc = wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, m=wl.m, base=base,
                            bits_hadamard=wl.bits_hadamard, out_type=wn.OUT_F32, fused=mode,
                            weights_pretransformed=1, operand_layout=lay)
        V = torch.empty((wn.wino_operand_bytes(pdesc)[0],), dtype=torch.int8, device=dev)
        wn.wino_weight_transform(pdesc, w, V, sc, stream)
        pws = torch.empty(wn.wino_workspace_bytes(pdesc), dtype=torch.uint8, device=dev)
        vdt = timed(torch, lambda: wn.wino_conv2d(pdesc, x, V, y, sc, pws, stream), steps)[0]
        out["pretransformed_weights"] = {"ms_per_step": vdt * 1e3, "value": ops / vdt / 1e12,
                                         "unit": "TOPS", "launches": wn.wino_conv2d_launches(pdesc),
                                         "note": "V computed once beforehand"}
        del V, pws
    # extra: the single-kernel variant where it exists for this layer (C <= 64)
    if want("fused") and wl.C <= 64 and wl.m in (2, 4) and wl.bits_hadamard in (8, 9):
        fdesc = wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, m=wl.m, base=base,
                            bits_hadamard=wl.bits_hadamard, out_type=wn.OUT_F32, fused=wn.FUSED_ON)
        fws = torch.empty(wn.wino_workspace_bytes(fdesc), dtype=torch.uint8, device=dev)
        fdt = timed(torch, lambda: wn.wino_conv2d(fdesc, x, w, y, sc, fws, stream), steps)[0]
        out["fused_variant"] = {"ms_per_step": fdt * 1e3, "value": ops / fdt / 1e12,
                                "unit": "TOPS", "launches": wn.wino_conv2d_launches(fdesc)}
        del fws
    # extra: the same layer with per-Winograd-point scales (U, V per point, M with
    # power-of-two refinements), calibrated on the device
    if want("per_point") and wl.bits_hadamard in (8, 9):
        cws = torch.empty(wn.wino_calibrate_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        psc = wn.wino_calibrate(desc, x, w, None, float(L["s_x"]), float(L["s_w"]), cws,
                                per_point=True)
        del cws
        pws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        pdt = timed(torch, lambda: wn.wino_conv2d(desc, x, w, y, psc, pws, stream), steps)[0]
        out["per_point_variant"] = {"ms_per_step": pdt * 1e3, "value": ops / pdt / 1e12,
                                    "unit": "TOPS", "m_shift_max": max(psc.m_shift[:n2]),
                                    "note": "per-point scales for U, V and M"}
        del pws
    # extra: the flex layer (run-time fp32 G_P, B_P, A_P; here the static matrices rounded
    # to fp32, as at the start of training) on the same workload, whole-layer call
    if want("flex"):
        fm = wn.FlexMatrices(*[np.array([[float(v) for v in row] for row in getattr(mats, nm)],
                                        dtype=np.float32) for nm in ("GP", "BPT", "APT")])
        xdesc = wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, m=wl.m, base=base,
                            bits_hadamard=wl.bits_hadamard, out_type=wn.OUT_F32)
        cws = torch.empty(wn.wino_calibrate_workspace_bytes(xdesc), dtype=torch.uint8, device=dev)
        xsc = wn.wino_flex_calibrate(xdesc, fm, x, w, None, float(L["s_x"]), float(L["s_w"]), cws)
        del cws
        xws = torch.empty(wn.wino_workspace_bytes(xdesc), dtype=torch.uint8, device=dev)
        xdt = timed(torch, lambda: wn.wino_flex_conv2d(xdesc, fm, x, w, y, xsc, xws, stream),
                    steps)[0]
        out["flex_variant"] = {"ms_per_step": xdt * 1e3, "value": ops / xdt / 1e12,
                               "unit": "TOPS",
                               "note": "fp32 brackets with run-time matrices, three launches"}
        del xws
    # extra: backward pass of the same layer (gradients w.r.t. input and weights from a
    # synthetic output gradient, U and V of the forward pass), fp32; each of its launches
    # timed by its own event pair
    if want("backward") and reps == 1:
        sdesc = wn.ConvDesc(wl.N, wl.H, wl.W, wl.C, wl.K, m=wl.m, base=base,
                            bits_hadamard=wl.bits_hadamard, out_type=wn.OUT_F32)
        mdt = {8: torch.int8, 9: torch.int16, 32: torch.int32}[wl.bits_hadamard]
        V = torch.empty((n2, wl.K, wl.C), dtype=torch.int8, device=dev)
        U = torch.empty((n2, T, wl.C), dtype=torch.int8, device=dev)
        M = torch.empty((n2, T, wl.K), dtype=mdt, device=dev)
        wn.wino_transform_operands(sdesc, x, U, w, V, sc, stream)
        wn.wino_contract(sdesc, U, V, M, sc, stream)
        # up to 8 partial sums of dV are added by the kernel that reads dV; more cost a launch of their own
        parts = wn.wino_backward_dv_parts(sdesc)
        extra_launch = ("sum_dV_parts",) if parts > 8 else ()
        bnames = ("dY_to_dM", "gemm_dV_and_dU") + extra_launch + ("dU_to_dx_and_dV_to_dw",)
        g = torch.Generator(device="cpu").manual_seed(wl.seed + 1)
        dy = torch.randn((wl.N, wl.H, wl.W, wl.K), generator=g, dtype=torch.float32).to(dev)
        dx = torch.empty((wl.N, wl.H, wl.W, wl.C), dtype=torch.float32, device=dev)
        dw = torch.empty((wl.K, wl.C, 3, 3), dtype=torch.float32, device=dev)
        bws = torch.empty(wn.wino_backward_workspace_bytes(sdesc), dtype=torch.uint8, device=dev)

        def bstep():
            wn.wino_backward(sdesc, dy, U, V, sc, dx, dw, bws, stream)
        bdt = timed(torch, bstep, steps, min_launches=100)[0]
        bmed = sample_launches(wn, torch, ev, bstep, len(bnames), samples=16, gap=1)
        kus = {nm: v * 1e3 for nm, v in zip(bnames, bmed)}
        # Both contractions: 2*n^2*T*C*K fp32-equivalent flops each, run as three bf16 MFMAs per
        # product (dM cut into three exact bf16 pieces), so the matrix pipe issues three times
        # that; algorithmic bytes: dM read by both, U and V, dU and the parts of dV written.
        gemm_flops = 2 * 2.0 * n2 * T * wl.C * wl.K
        gemm_s = kus["gemm_dV_and_dU"] * 1e-6
        issued_tf = 3 * gemm_flops / gemm_s / 1e12
        gemm_bytes = n2 * (2 * 4 * T * wl.K + T * wl.C + wl.K * wl.C + 4 * T * wl.C + 4 * parts * wl.K * wl.C)
        out["backward_variant"] = {
            "ms_per_step": bdt * 1e3, "dtype": "f32", "kernel_us": kus,
            "roofline": {"bound": "hbm", "kernel": "gemm_dV_and_dU (both contractions, one launch)",
                         "achieved": gemm_bytes / gemm_s / 1e9, "peak": 8000.0, "unit": "GB/s",
                         "frac": gemm_bytes / gemm_s / 8e12, "traffic": None,
                         "algorithmic_bytes": gemm_bytes,
                         "bf16_mfma_issued_TFLOPs": issued_tf, "bf16_mfma_frac": issued_tf / 2500.0,
                         "bf16_mfma_frac_of_measured_peak": issued_tf / peaks["bf16_mfma_TFLOPs"],
                         "fp32_equivalent_TFLOPs": gemm_flops / gemm_s / 1e12,
                         "fp32_mfma_peak_TFLOPs": 157.3},
            "note": "straight-through gradients; the two contraction gradients are GEMMs of fp32 dM with "
                    "int8 codes, exact to fp32 accumulation, on the bf16 matrix pipe (3 MFMAs per product)"}
        # the same for the flex layer (run-time matrices: here the static ones rounded to
        # fp32), which also returns the gradients of G_P, B_P, A_P; first four of its five
        # launches timed (the last one sums the partial matrix gradients)
        fnames = ("dY_M_to_dM_dAPT", "gemm_dV_and_dU") + extra_launch + ("input_and_filter_brackets",
                                                                         "tile_dX_to_dx")
        bfm = wn.FlexMatrices(*[np.array([[float(v) for v in row] for row in getattr(mats, nm)],
                                         dtype=np.float32) for nm in ("GP", "BPT", "APT")])
        nn = desc.n
        dGP = torch.empty((nn, 3), dtype=torch.float32, device=dev)
        dBPT = torch.empty((nn, nn), dtype=torch.float32, device=dev)
        dAPT = torch.empty((wl.m, nn), dtype=torch.float32, device=dev)
        fws = torch.empty(wn.wino_flex_backward_workspace_bytes(sdesc), dtype=torch.uint8, device=dev)

        def fstep():
            wn.wino_flex_backward(sdesc, bfm, dy, x, w, U, V, M, sc, dx, dw, dGP, dBPT, dAPT, fws,
                                  stream)
        fdt = timed(torch, fstep, steps, min_launches=100)[0]
        fmed = sample_launches(wn, torch, ev, fstep, len(fnames), samples=16, gap=1)
        torch.cuda.synchronize()
        out["flex_backward_variant"] = {
            "ms_per_step": fdt * 1e3, "dtype": "f32",
            "kernel_us": {nm: v * 1e3 for nm, v in zip(fnames, fmed)},
            "note": "dx, dw and the gradients of the three trained matrices"}
        del dy, dx, dw, bws, fws, U, V, M
    # extra: whole-layer call (wino_conv2d) on the other single-layer configurations, one
    # kernel per stage and the library's own choice; not the headline figure
    if want("others") and reps == 1:
        out["other_workloads"] = {}
        for name in ("cfg2_f4_c64", "cfg3_f4_c128_h9", "cfg4b_f4_c512", "cfg4a_f6_c256",
                     "cfg4b_f6_c512"):
            if name == wl.name:
                continue
            out["other_workloads"][name] = layer_times(wn, si, torch, dev, name, 50)
        out["resnet18_stack"] = resnet18_stack(wn, si, torch, dev, 20)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(si.WORKLOADS[args.workload])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
