"""Shared plumbing of the parity tests: oracle run + library run on the same inputs."""
import numpy as np

import synth_inputs as si
from oracle import quantised as q

M_DTYPES = {8: np.int8, 9: np.int16, 32: np.int32}


def oracle_layer(xq, wq, s_x, s_w, m=4, base="legendre", bits_hadamard=8, inner_quant=True,
                 out_type="f32", relu=False, per_point=False):
    cfg = q.LayerConfig(m=m, base=base, bits_hadamard=bits_hadamard, inner_quant=inner_quant,
                        out_type=out_type, relu=relu, per_point=per_point)
    return q.run_layer(xq, wq, s_x, s_w, cfg)


def small_layer(N, H, W, C, K, seed, outliers=0.0):
    x, w = si.make_real(N, H, W, C, K, seed, outliers)
    xq, s_x = si.cast_int8(x)
    wq, s_w = si.cast_int8(w)
    return xq, wq, s_x, s_w


def gpu_layer(xq, wq, scales, m=4, base="legendre", bits_hadamard=8, inner_quant=True,
              out_type="f32", relu=False, whole=False, fused=False, per_point=False):
    """Runs the library stage by stage (or wino_conv2d when ``whole``) and
    returns numpy copies of V, U, M, y."""
    import torch
    import paper_2004_11077_amd as wn
    dev = torch.device("cuda:0")
    N, H, W, C = xq.shape
    K = wq.shape[0]
    base_id = {"canonical": wn.BASE_CANONICAL, "legendre": wn.BASE_LEGENDRE,
               "chebyshev": wn.BASE_CHEBYSHEV, "hermite": wn.BASE_HERMITE}[base]
    out_id = {"f32": wn.OUT_F32, "i32": wn.OUT_I32, "i8": wn.OUT_I8}[out_type]
    desc = wn.ConvDesc(N, H, W, C, K, m=m, base=base_id, bits_hadamard=bits_hadamard,
                       inner_quant=int(inner_quant), out_type=out_id, relu=int(relu))
    n2, T = desc.n ** 2, desc.tiles
    sc = wn.Scales.from_dict(scales)
    x = torch.from_numpy(np.ascontiguousarray(xq, dtype=np.int8)).to(dev)
    w = torch.from_numpy(np.ascontiguousarray(wq, dtype=np.int8)).to(dev)
    mdt = {8: torch.int8, 9: torch.int16, 32: torch.int32}[bits_hadamard]
    ydt = {"f32": torch.float32, "i32": torch.int32, "i8": torch.int8}[out_type]
    y = torch.full((N, H, W, K), 77, dtype=ydt, device=dev)
    if fused:
        # single-kernel variant: U and M stay on chip, only V and y can be read back
        desc.fused = 1
        ws = torch.empty(wn.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        wn.wino_conv2d(desc, x, w, y, sc, ws)
        torch.cuda.synchronize()
        if "contraction_output" in wn.wino_conv2d_launches(desc):
            # two-kernel form: the workspace holds V in fragment order
            fd = wn.ConvDesc(N, H, W, C, K, m=m, operand_layout=wn.LAYOUT_FRAGMENTS)
            vb = wn.wino_operand_bytes(fd)[0]
            Vn = wn.defragment(ws[:vb].view(torch.int8).cpu().numpy(), n2, K, C)
        else:
            Vn = ws[:n2 * K * C].view(torch.int8).reshape(n2, K, C).cpu().numpy()
        return {"V": Vn, "y": y.cpu().numpy()}
    if whole:
        nbytes = wn.wino_workspace_bytes(desc)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        wn.wino_conv2d(desc, x, w, y, sc, ws)
        torch.cuda.synchronize()
        r256 = lambda v: (v + 255) // 256 * 256
        o = 0
        V = ws[o:o + n2 * K * C].view(torch.int8).reshape(n2, K, C); o += r256(n2 * K * C)
        U = ws[o:o + n2 * T * C].view(torch.int8).reshape(n2, T, C); o += r256(n2 * T * C)
        mb = n2 * T * K * torch.empty((), dtype=mdt).element_size()
        M = ws[o:o + mb].view(mdt).reshape(n2, T, K)
    else:
        V = torch.full((n2, K, C), 77, dtype=torch.int8, device=dev)
        U = torch.full((n2, T, C), 77, dtype=torch.int8, device=dev)
        M = torch.full((n2, T, K), 77, dtype=mdt, device=dev)
        wn.wino_weight_transform(desc, w, V, sc)
        wn.wino_input_transform(desc, x, U, sc)
        wn.wino_contract(desc, U, V, M, sc)
        wn.wino_output_transform(desc, M, y, sc)
        torch.cuda.synchronize()
    return {"V": V.cpu().numpy(), "U": U.cpu().numpy(), "M": M.cpu().numpy(),
            "y": y.cpu().numpy()}


def assert_layer_parity(ora, got, out_type="f32"):
    """Integer stages bit-exact; fp32 output within 1e-5 of the output range."""
    for key in ("V", "U", "M"):
        if key not in got:
            continue
        assert got[key].shape == ora[key].shape, key
        bad = np.nonzero(got[key].astype(np.int64) != ora[key])
        assert bad[0].size == 0, "%s: %d mismatches, first at %s" % (
            key, bad[0].size, [int(b[0]) for b in bad])
    if out_type == "f32":
        ref = ora["y"]
        tol = 1e-5 * max(float(np.abs(ref).max()), 1e-30)
        err = float(np.abs(got["y"].astype(np.float64) - ref).max()) if ref.size else 0.0
        assert err <= tol, "y: max abs err %g > %g" % (err, tol)
    else:
        assert np.array_equal(got["y"].astype(np.int64), ora["y"]), "y codes differ"
