"""GPU-vs-oracle parity of the wider stages (Sec. 3.2 "quantization diversity", the INT10 /
INT16 pipelines of Sec. 5.1): every tap bit-exact -- 16-bit codes of the transformed
weights and input, the exact int64 accumulators, the output codes -- for one width
everywhere (WINO_I16) and for 8-bit activations around a 16-bit Winograd domain
(WINO_I8W16), with and without the Hadamard-stage quantizer, per-position scales, learned
("flex") matrices, ragged shapes and the longest reduction the digit arithmetic allows."""
import json
import os

import numpy as np
import pytest

from paper_2002_10711_amd import workloads
from paper_2002_10711_amd.workloads import Layer

from helpers import make_case

pytestmark = pytest.mark.gpu

INT16 = dict(x=32767, u=32767, v=32767, m=32767, y=32767)
INT10 = dict(x=511, u=511, v=511, m=511, y=511)
W16 = dict(x=127, u=32767, v=32767, m=32767, y=127)        # 8-bit data, 16-bit Winograd domain
MIXED = dict(x=127, u=2047, v=32767, m=8191, y=127)         # a different width at every stage


def run_wide(case, qm, sc):
    """Forward through the C ABI in a wide mode; every tap back as numpy."""
    import torch
    from paper_2002_10711_amd import binding as wb
    L = case["layer"]
    dev = torch.device("cuda:0")
    x16 = qm["y"] > 127 or qm["x"] > 127
    dt = wb.WINO_I16 if x16 else wb.WINO_I8W16
    tdt = torch.int16 if x16 else torch.int8
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, dt, BT=case["BT"], G=case["G"], AT=case["AT"])
    quant = wb.make_quant(sc["s_x"], sc.get("s_v", 1.0), sc.get("s_u", 1.0), sc["s_y"],
                          sc.get("s_m", 0.0), qm["y"], s_v_pos=sc.get("s_v_pos"),
                          s_u_pos=sc.get("s_u_pos"), qmax_u=qm["u"], qmax_v=qm["v"],
                          qmax_m=qm["m"], qmax_y=qm["y"])
    assert wb.wino_fwd_num_kernels(desc) in (2, 3)
    x = torch.from_numpy(case["xq"].astype(np.int16 if x16 else np.int8)).to(dev)
    g = torch.from_numpy(case["g"]).to(dev)
    U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    Ho, Wo = L.H + 2 * L.pad - 2, L.W + 2 * L.pad - 2
    y = torch.full((L.N, L.K, Ho, Wo), 77, dtype=tdt, device=dev)
    wb.wino_transform_weights(desc, quant, g, U)
    wb.wino_conv2d_fwd(desc, quant, x, U, y, ws)
    torch.cuda.synchronize()
    out = dict(Y=y.cpu().numpy())
    y2 = torch.full_like(y, 55)
    ws.zero_()
    for stage in (wb.WINO_STAGE_INPUT, wb.WINO_STAGE_GEMM, wb.WINO_STAGE_OUTPUT):
        wb.wino_conv2d_fwd_stages(desc, quant, x, U, y2, ws, stage)
    P = (L.m + 2) ** 2
    T = L.N * (-(-Ho // L.m)) * (-(-Wo // L.m))
    Uo = torch.empty((P, L.K, L.C), dtype=torch.int16, device=dev)
    Vo = torch.empty((P, T, L.C), dtype=torch.int16, device=dev)
    Mo = torch.empty((P, T, L.K), dtype=torch.int64, device=dev)
    wb.wino_debug_export(desc, wb.WINO_TAP_U, U, Uo)
    wb.wino_debug_export(desc, wb.WINO_TAP_V, ws, Vo)
    wb.wino_debug_export(desc, wb.WINO_TAP_M, ws, Mo)
    torch.cuda.synchronize()
    out.update(Y_staged=y2.cpu().numpy(), U=Uo.cpu().numpy(), V=Vo.cpu().numpy(), M=Mo.cpu().numpy())
    return out


def check(ref, out):
    for tap, key in (("U", "Uq"), ("V", "Vq"), ("M", "M"), ("Y_staged", "Yq"), ("Y", "Yq")):
        a, b = out[tap].astype(np.int64), ref[key].astype(np.int64)
        assert a.shape == b.shape, (tap, a.shape, b.shape)
        bad = int((a != b).sum())
        assert bad == 0, "%s: %d of %d differ, first at %s" % (
            tap, bad, a.size, np.argwhere(a != b)[:3].tolist())


def wide_case(oracle, layer, qm, with_m=False, pos=False):
    case = make_case(oracle, layer, with_oracle=False)
    if pos:
        sc = oracle.calibrate_pos(case["X"], case["g"], case["BT"], case["G"], case["AT"],
                                  pad=layer.pad, qmax=qm["v"])
        # calibrate_pos knows one width: rescale what it derived from it to the stage widths
        f32 = np.float32
        sc["s_x"] = float(f32(sc["s_x"]) * f32(qm["v"]) / f32(qm["x"]))
        sc["s_u_pos"] = (sc["s_u_pos"] * f32(qm["v"]) / f32(qm["u"])).astype(f32)
        sc["s_y"] = float(f32(sc["s_y"]) * f32(qm["v"]) / f32(qm["y"]))
    else:
        sc = oracle.calibrate(case["X"], case["g"], case["BT"], case["G"], case["AT"],
                              pad=layer.pad, qmax=qm, with_m=with_m)
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"], qm["x"])
    ref = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                            pad=layer.pad, qmax=qm)
    return case, sc, ref


LAYERS = [
    Layer("w_f4_16px", 2, 64, 64, 16, 16, m=4, seed=301),
    Layer("w_f2_ragged", 3, 37, 70, 9, 11, m=2, seed=302),
    Layer("w_f4_ragged_pad0", 2, 20, 33, 13, 10, m=4, pad=0, seed=303),
    Layer("w_f6_14px", 1, 48, 36, 14, 14, m=6, seed=304),
    Layer("w_f4_flex", 2, 40, 24, 12, 12, m=4, flex_sigma=0.03, seed=305),
    Layer("w_f4_c600", 1, 600, 40, 8, 8, m=4, seed=306),          # beyond 512 channels
    Layer("w_f2_1px", 5, 3, 5, 1, 1, m=2, seed=307),              # a single output pixel
    Layer("w_f2_16k_tiles", 64, 16, 24, 32, 32, m=2, seed=309),   # two tile groups per workgroup
    # enough tiles for the GEMM + output kernel (512; 1024 for F6), every reduction length
    Layer("w_f4_600tiles_ragged", 6, 37, 70, 38, 40, m=4, seed=310),
    Layer("w_f6_c100_1100tiles", 11, 100, 40, 60, 58, m=6, seed=311),
    Layer("w_f2_c200_630tiles", 3, 200, 40, 28, 30, m=2, seed=312),
    Layer("w_f4_c450_512tiles_flex", 2, 450, 24, 64, 64, m=4, flex_sigma=0.03, seed=313),
    Layer("w_f4_c100_576tiles", 4, 100, 24, 48, 48, m=4, seed=314),
    Layer("w_f4_c200_576tiles", 4, 200, 24, 48, 48, m=4, seed=315),
    Layer("w_f2_c100_576tiles", 4, 100, 24, 24, 24, m=2, seed=316),
    Layer("w_f6_c40_1024tiles", 16, 40, 24, 48, 48, m=6, seed=317),
]
FUSED = LAYERS[-8:-4]


@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: l.name)
@pytest.mark.parametrize("qm", [INT16, INT10, W16, MIXED], ids=["int16", "int10", "i8w16", "mixed"])
def test_wide_stages_all_taps(oracle, layer, qm):
    case, sc, ref = wide_case(oracle, layer, qm)
    assert np.abs(ref["Vq"]).max() == qm["v"] and np.abs(ref["Uq"]).max() == qm["u"]
    check(ref, run_wide(case, qm, sc))


@pytest.mark.parametrize("layer", LAYERS[:5] + FUSED[1:3], ids=lambda l: l.name)
@pytest.mark.parametrize("qm", [INT16, MIXED], ids=["int16", "mixed"])
def test_wide_stages_with_hadamard_quantizer(oracle, layer, qm):
    case, sc, ref = wide_case(oracle, layer, qm, with_m=True)
    assert sc["s_m"] > 0
    check(ref, run_wide(case, qm, sc))


@pytest.mark.parametrize("layer", LAYERS[:4] + FUSED[:2], ids=lambda l: l.name)
@pytest.mark.parametrize("qm", [INT16, W16], ids=["int16", "i8w16"])
def test_wide_stages_per_position_scales(oracle, layer, qm):
    case, sc, ref = wide_case(oracle, layer, qm, pos=True)
    check(ref, run_wide(case, qm, sc))
    sc = dict(sc, s_m=float(np.abs(ref["M"] * ref["scalars"]["w"][:, None, None]).max()) / qm["m"])
    ref = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                            pad=layer.pad, qmax=qm)
    check(ref, run_wide(case, qm, sc))


def test_every_code_saturated_over_1024_channels(oracle):
    """The worst case of the digit arithmetic: all codes at +-32767 (digits +-128, -+1) and
    the longest supported reduction, where the sums of digit products reach 2^24."""
    layer = Layer("w_sat", 1, 1024, 16, 4, 4, m=2, seed=308)
    case = make_case(oracle, layer, with_oracle=False)
    sc = dict(s_x=1.0, s_v=1e-6, s_u=1e-9, s_y=1.0, s_m=0.0)
    rng = np.random.default_rng(layer.seed)
    case["xq"] = rng.choice([-32767, 32767], size=case["X"].shape).astype(np.int32)
    case["xq"][0, :, :, :] = 32767
    case["g"] = np.abs(case["g"]) + np.float32(0.01)
    ref = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc, qmax=INT16)
    assert np.abs(ref["M"]).max() >= 1000 * 32767 * 32767
    check(ref, run_wide(case, INT16, sc))


@pytest.mark.parametrize("dtype", ["i16", "i8w16"])
def test_config2_wide_full_size_as_benchmarked(oracle, dtype):
    """The benchmark's wide workloads at full size, with the scales the benchmark reads
    (written by tests/golden/make_bench_scales.py through the oracle): every tap."""
    L = workloads.config2(dtype)[0]
    qm = workloads.STAGE_QMAX[dtype]
    sc = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "bench_scales.json")))[L.name]
    case = make_case(oracle, L, with_oracle=False)
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"], qm["x"])
    ref = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                            pad=L.pad, qmax=qm)
    assert np.abs(ref["Vq"]).max() == qm["v"] and np.abs(ref["Yq"]).max() == qm["y"]
    check(ref, run_wide(case, qm, sc))


def test_wide_argument_checks():
    import torch
    from paper_2002_10711_amd import binding as wb
    BT, G, AT = wb.wino_cook_toom(4)
    q = wb.make_quant(1.0, 1.0, 1.0, 1.0, 0.0, 32767)
    assert wb.wino_weights_bytes(wb.Desc(1, 1025, 8, 8, 8, 1, 4, wb.WINO_I16, BT=BT, G=G, AT=AT)) == 0
    d = wb.Desc(1, 8, 8, 8, 8, 1, 4, wb.WINO_I8W16, BT=BT, G=G, AT=AT)
    dev = torch.device("cuda:0")
    U = torch.empty(wb.wino_weights_bytes(d), dtype=torch.uint8, device=dev)
    g = torch.zeros((8, 8, 3, 3), device=dev)
    # 8-bit output container: qmax_y may not exceed 127
    with pytest.raises(wb.WinoError):
        wb.wino_transform_weights(d, q, g, U)
    wb.wino_transform_weights(d, wb.make_quant(1.0, 1.0, 1.0, 1.0, 0.0, 127, qmax_u=32767), g, U)
    # the int8 mode shares one range between its stages
    d8 = wb.Desc(1, 8, 8, 8, 8, 1, 4, wb.WINO_I8, BT=BT, G=G, AT=AT)
    with pytest.raises(wb.WinoError):
        wb.wino_transform_weights(d8, wb.make_quant(1.0, 1.0, 1.0, 1.0, 0.0, 127, qmax_u=63), g, U)
    torch.cuda.synchronize()
