"""Shared plumbing of the GPU parity tests: build a case (seeded inputs, matrices
and scales from the oracle side), run it through the C ABI on the GPU, return every
tap as numpy.  No arithmetic of the method lives here."""
import numpy as np

from paper_2002_10711_amd import workloads


def make_case(oracle, layer, with_oracle=True):
    X, g = workloads.make_inputs(layer)
    BT, G, AT = oracle.cook_toom(layer.m, dtype=np.float32)
    if layer.flex_sigma > 0:
        BT, G, AT = workloads.perturb_transforms(BT, G, AT, layer.flex_sigma, layer.seed)
    case = dict(layer=layer, X=X, g=g, BT=BT, G=G, AT=AT)
    if layer.dtype == "i8":
        sc = oracle.calibrate(X, g, BT, G, AT, pad=layer.pad)
        case["scales"] = sc
        case["xq"] = oracle.quantize_tensor(X, sc["s_x"]).astype(np.int8)
        if with_oracle:
            case["ref"] = oracle.winograd_q(case["xq"], g, BT, G, AT, sc, pad=layer.pad)
    return case


def run_gpu(case, taps=True, scales=None):
    import torch
    from paper_2002_10711_amd import binding as wb
    L = case["layer"]
    dev = torch.device("cuda:0")
    i8 = L.dtype == "i8"
    bf = L.dtype == "bf16"
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m,
                   wb.WINO_I8 if i8 else wb.WINO_BF16 if bf else wb.WINO_F32,
                   BT=case["BT"], G=case["G"], AT=case["AT"])
    quant = None
    if i8:
        sc = scales or case["scales"]
        quant = wb.make_quant(sc["s_x"], sc.get("s_v", 1.0), sc.get("s_u", 1.0), sc["s_y"],
                              sc.get("s_m", 0.0), sc.get("qmax", 127),
                              s_v_pos=sc.get("s_v_pos"), s_u_pos=sc.get("s_u_pos"))
    x = torch.from_numpy(case["xq"] if i8 else case["X"]).to(dev)
    g = torch.from_numpy(case["g"]).to(dev)
    U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    Ho, Wo = L.H + 2 * L.pad - 2, L.W + 2 * L.pad - 2
    y = torch.full((L.N, L.K, Ho, Wo), 77, dtype=torch.int8 if i8 else torch.float32, device=dev)
    wb.wino_transform_weights(desc, quant, g, U)
    # the whole forward in one call (GEMM and output transform fused, M never stored)
    wb.wino_conv2d_fwd(desc, quant, x, U, y, ws)
    torch.cuda.synchronize()
    out = dict(Y=y.cpu().numpy())
    # the same forward with every kernel sequence that can run this problem, named explicitly
    out["Y_seq"] = {}
    if i8:
        for seq, name in wb.SEQ_NAMES.items():
            if wb.wino_fwd_sequence(desc, seq) != seq:
                continue
            ys = torch.full_like(y, 33)
            ws.zero_()
            wb.wino_conv2d_fwd_seq(desc, quant, x, U, ys, ws, seq)
            torch.cuda.synchronize()
            out["Y_seq"][name] = ys.cpu().numpy()
    if bf:
        return out                                  # one kernel only: no stages, no taps
    # stage by stage, which materialises V and M for the taps
    y2 = torch.full_like(y, 55)
    ws.zero_()
    for stage in (wb.WINO_STAGE_INPUT, wb.WINO_STAGE_GEMM, wb.WINO_STAGE_OUTPUT):
        wb.wino_conv2d_fwd_stages(desc, quant, x, U, y2, ws, stage)
    torch.cuda.synchronize()
    out["Y_staged"] = y2.cpu().numpy()
    if taps:
        n = L.m + 2
        P = n * n
        T = L.N * (-(-Ho // L.m)) * (-(-Wo // L.m))
        dt = torch.int8 if i8 else torch.float32
        Uo = torch.empty((P, L.K, L.C), dtype=dt, device=dev)
        Vo = torch.empty((P, T, L.C), dtype=dt, device=dev)
        Mo = torch.empty((P, T, L.K), dtype=torch.int32 if i8 else torch.float32, device=dev)
        wb.wino_debug_export(desc, wb.WINO_TAP_U, U, Uo)
        wb.wino_debug_export(desc, wb.WINO_TAP_V, ws, Vo)
        wb.wino_debug_export(desc, wb.WINO_TAP_M, ws, Mo)
        torch.cuda.synchronize()
        out.update(U=Uo.cpu().numpy(), V=Vo.cpu().numpy(), M=Mo.cpu().numpy())
    return out


def max_rel(a, ref):
    """max |a - ref| / max |ref| over the whole tensor."""
    return float(np.abs(a.astype(np.float64) - ref).max() / np.abs(ref).max())
