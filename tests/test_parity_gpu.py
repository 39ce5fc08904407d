"""GPU-vs-oracle parity through the C ABI.  int8: every tap (transformed weights,
transformed input, int32 accumulators, int8 output) bit-exact against the pinned
quantized pipeline of the oracle.  fp32: max |diff| / max |ref| against the fp64
direct convolution <= 1e-4 (m = 2, 4) or 1e-3 (m = 6); with perturbed matrices the
reference is the fp64 literal Winograd with the same matrices."""
import numpy as np
import pytest

from paper_2002_10711_amd import workloads
from paper_2002_10711_amd.workloads import Layer

from helpers import make_case, max_rel, run_gpu

pytestmark = pytest.mark.gpu

FP32_TOL = {2: 1e-4, 4: 1e-4, 6: 1e-3}


def _check_i8(case, out, inexact_ok=False):
    ref = case["ref"]
    assert inexact_ok or ref["inexact"] == 0
    for tap, key in (("U", "Uq"), ("V", "Vq"), ("M", "M"), ("Y_staged", "Yq"), ("Y", "Yq")):
        a, b = out[tap].astype(np.int64), ref[key].astype(np.int64)
        assert a.shape == b.shape, (tap, a.shape, b.shape)
        bad = int((a != b).sum())
        assert bad == 0, "%s: %d of %d differ, first at %s" % (
            tap, bad, a.size, np.argwhere(a != b)[:3].tolist())
    # every kernel sequence that can run the shape gives the same codes
    assert out["Y_seq"], "no kernel sequence reported as supported"
    for name, ys in out["Y_seq"].items():
        bad = int((ys.astype(np.int64) != ref["Yq"].astype(np.int64)).sum())
        assert bad == 0, "sequence %s: %d of %d output codes differ" % (name, bad, ys.size)


def _check_f32(oracle, case, out):
    L = case["layer"]
    if L.flex_sigma > 0:
        ref = oracle.winograd_f64(case["X"], case["g"], case["BT"], case["G"], case["AT"], L.pad)
    else:
        ref = oracle.conv2d_direct_f64(case["X"], case["g"], 1, L.pad)
    assert out["Y"].shape == ref.shape
    err = max(max_rel(out["Y"], ref), max_rel(out["Y_staged"], ref))
    assert err <= FP32_TOL[L.m], err
    if "U" in out:
        # every stage on its own, against the same stage evaluated in fp64 (plain einsum over
        # the patches): transformed weights and input within 1e-5 of their max-abs (a few
        # fp32 roundings each), the channel sums within the tolerance of the output
        n = L.m + 2
        G64, BT64 = case["G"].astype(np.float64), case["BT"].astype(np.float64)
        U_ref = np.einsum("ia,kcab,jb->ijkc", G64, case["g"].astype(np.float64), G64)
        U_ref = U_ref.reshape(n * n, L.K, L.C)
        Ho, Wo = L.H + 2 * L.pad - 2, L.W + 2 * L.pad - 2
        TH, TW = -(-Ho // L.m), -(-Wo // L.m)
        Xp = np.zeros((L.N, L.C, L.pad + TH * L.m + n, L.pad + TW * L.m + n))
        Xp[:, :, L.pad:L.pad + L.H, L.pad:L.pad + L.W] = case["X"]
        d = np.stack([Xp[:, :, th * L.m:th * L.m + n, tw * L.m:tw * L.m + n]
                      for th in range(TH) for tw in range(TW)], axis=1)       # [N, TH*TW, C, n, n]
        d = d.reshape(L.N * TH * TW, L.C, n, n)
        V_ref = np.einsum("ij,tcjl,kl->iktc", BT64, d, BT64).reshape(n * n, -1, L.C)
        M_ref = np.einsum("ptc,pkc->ptk", V_ref, U_ref)
        assert max_rel(out["U"], U_ref) <= 1e-5, ("U", max_rel(out["U"], U_ref))
        assert max_rel(out["V"], V_ref) <= 1e-5, ("V", max_rel(out["V"], V_ref))
        assert max_rel(out["M"], M_ref) <= FP32_TOL[L.m], ("M", max_rel(out["M"], M_ref))
    return err


def test_config1_fp32_f2(oracle):
    case = make_case(oracle, workloads.config1()[0])
    _check_f32(oracle, case, run_gpu(case))


# Small shapes spanning several 64-row blocks, ragged tiles (m does not divide
# Ho), C and K that are not multiples of the padding granules, pad 0 and 1.
SMALL = [
    Layer("s_f2", 3, 20, 24, 9, 11, m=2, seed=101),
    Layer("s_f4", 2, 70, 33, 13, 10, m=4, seed=102),
    Layer("s_f6", 2, 12, 65, 16, 16, m=6, seed=103),
    Layer("s_f6_tiny", 5, 5, 3, 4, 4, m=6, seed=104),
    Layer("s_f4_pad0", 2, 16, 16, 10, 12, m=4, pad=0, seed=105),
    Layer("s_f2_1x1out", 1, 3, 2, 3, 3, m=2, pad=0, seed=106),
    Layer("s_f4_wide", 1, 130, 70, 6, 40, m=4, seed=107),
    Layer("s_f4_16px", 3, 64, 64, 16, 16, m=4, seed=112),       # 4 x 4 tiles per workgroup row block
    Layer("s_f4_narrow", 2, 8, 8, 5, 3, m=4, seed=113),         # image narrower than a dword
    Layer("s_f4_c128k128", 2, 128, 128, 8, 8, m=4, seed=114),   # two channel blocks, two k blocks
    Layer("s_f2_32px", 2, 64, 32, 32, 32, m=2, seed=115),
    Layer("s_f6_32px", 1, 64, 64, 32, 32, m=6, seed=116),
    Layer("s_f2_16px_c128", 2, 128, 128, 16, 16, m=2, seed=117),  # F2, two channel and k blocks
    Layer("s_f2_8px", 5, 64, 64, 8, 8, m=2, seed=118),            # 4 tiles per row
    Layer("s_f2_14px", 3, 48, 36, 14, 14, m=2, seed=119),         # 7 tiles per row: odd window offsets
    Layer("s_f4_8px", 9, 64, 64, 8, 8, m=4, seed=120),            # 2 tiles per row, ragged row blocks
    Layer("s_f4_64px", 1, 64, 64, 64, 64, m=4, seed=121),         # 16 tiles per row
    Layer("s_f4_7px", 5, 24, 20, 7, 7, m=4, seed=141),            # 2 x 2 ragged tiles, odd width
    Layer("s_f2_4px", 9, 64, 64, 4, 4, m=2, seed=142),            # rows of one dword
    Layer("s_f4_4px", 17, 70, 33, 4, 4, m=4, seed=143),           # one tile per image, ragged row blocks
    Layer("s_f2_36px", 1, 16, 16, 36, 36, m=2, seed=144),         # 18 tiles per row: two row pieces
    Layer("s_f4_k32", 3, 64, 32, 16, 16, m=4, seed=122),          # K below the 64-channel block
    Layer("s_f4_k100", 2, 64, 100, 16, 16, m=4, seed=123),        # K = 64 + 36
    # 65..128 output channels, at most 128 input channels: the eight-wavefront fused kernel
    Layer("s_f4_c128_k128", 3, 128, 128, 16, 16, m=4, seed=145),  # two LDS regions
    Layer("s_f4_c70_k100", 2, 70, 100, 8, 8, m=4, seed=146),      # ragged channels both ways
    Layer("s_f4_c40_k128_7px", 5, 40, 128, 7, 7, m=4, seed=147),  # one region, ragged tiles
    Layer("s_f2_c128_k72_32px", 1, 128, 72, 32, 32, m=2, seed=148),
    Layer("s_f2_c100_k128_6px", 7, 100, 128, 6, 6, m=2, seed=149),
    Layer("s_f4_c128_k128_64px", 1, 128, 128, 64, 64, m=4, seed=150),
    # long reductions: GEMM fused with the column-by-column output transform
    Layer("s_f2_c200_k300_ragged", 2, 200, 300, 9, 11, m=2, seed=151),
    Layer("s_f4_c256_k64_pad0", 2, 256, 64, 14, 10, m=4, pad=0, seed=152),
    Layer("s_f2_c512_k70_5px", 3, 512, 70, 5, 5, m=2, seed=153),
    Layer("s_f6_c128_k96_13px", 2, 128, 96, 13, 13, m=6, seed=154),
    Layer("s_f4_c450_k130_12px", 1, 450, 130, 12, 12, m=4, seed=155),   # 512 padded: tiled GEMM
    # images narrower than a dword: byte-wise staging in the one-kernel forward
    Layer("s_f2_2px", 33, 64, 64, 2, 2, m=2, seed=156),
    Layer("s_f4_2px_c70_k100", 9, 70, 100, 2, 2, m=4, seed=157),
    Layer("s_f2_3px_k128", 5, 128, 128, 3, 3, m=2, seed=158),
    Layer("s_f4_1px_wide", 3, 20, 40, 9, 1, m=4, seed=159),             # a single column
    Layer("s_f2_3px_k300", 4, 64, 300, 6, 3, m=2, seed=160),            # narrow, unfused
    Layer("s_f6_2px", 6, 64, 64, 2, 2, m=6, seed=161),
    # many tiles and long reductions: two tile blocks per wavefront in the GEMM + output kernel
    Layer("s_f2_c200_k40_8649tiles", 9, 200, 40, 62, 62, m=2, seed=162),
    Layer("s_f4_c450_k40_2048tiles", 2, 450, 40, 126, 126, m=4, seed=163),
    Layer("s_f4_c500_k70_600tiles", 6, 500, 70, 38, 40, m=4, seed=164),   # F4, 512 channels, one block
    Layer("s_f6_c200_k40_1100tiles", 11, 200, 40, 60, 58, m=6, seed=168),  # F6, long reduction, many tiles
    Layer("s_f6_c500_k70_1024tiles", 16, 500, 70, 48, 48, m=6, seed=169),
    Layer("s_f2_c200_k130_8649tiles", 9, 200, 130, 62, 62, m=2, seed=171),   # K > 128: two kernels
    # learned (dense) matrices with long reductions: the dense variants of the GEMM + output kernel
    Layer("s_flex_f4_c200_k70", 8, 200, 70, 16, 16, m=4, flex_sigma=0.02, seed=172),
    Layer("s_flex_f2_c500_k70", 2, 500, 70, 12, 12, m=2, flex_sigma=0.02, seed=173),
    Layer("s_flex_f6_c200_k40_1100tiles", 11, 200, 40, 60, 58, m=6, flex_sigma=0.01, seed=174),
    Layer("s_flex_f4_c450_k40_512tiles", 2, 450, 40, 64, 64, m=4, flex_sigma=0.02, seed=175),
    # reductions of 3, 5, 6 and 7 blocks of 64 channels
    Layer("s_f4_c150_k140", 4, 150, 140, 16, 16, m=4, seed=176),
    Layer("s_f2_c300_k140", 2, 300, 140, 12, 14, m=2, seed=177),
    Layer("s_f4_c370_k70_576tiles", 4, 370, 70, 48, 48, m=4, seed=178),
    Layer("s_f2_c420_k130", 3, 420, 130, 9, 11, m=2, seed=179),
    Layer("s_f6_c300_k40_1100tiles", 11, 300, 40, 60, 58, m=6, seed=180),
    Layer("s_flex_f2_c170_k40", 3, 170, 40, 10, 10, m=2, flex_sigma=0.02, seed=181),
    # F2, 512 padded channels, >= 1 k tiles: GEMM + output kernel with 32 x 64 workgroup tiles
    Layer("s_f2_c500_k72_7px_1024tiles", 64, 500, 72, 7, 7, m=2, seed=182),    # ragged tiles, K = 64 + 8
    Layer("s_f2_c512_k128_4px_1024tiles", 256, 512, 128, 4, 4, m=2, seed=183),  # whole images: staged stores
    Layer("s_f2_c450_k64_8px_1040tiles", 65, 450, 64, 8, 8, m=2, seed=184),     # last tile block half empty
    # F6 with the Cook-Toom B^T: input transform on the matrix cores (two int8 digits of W)
    Layer("s_f6_pad0_20px", 2, 70, 33, 20, 20, m=6, pad=0, seed=185),          # 3 x 3 whole tiles, two channel blocks
    Layer("s_f6_w5_h9", 3, 24, 20, 9, 5, m=6, seed=186),                       # odd width: unaligned dword loads
    Layer("s_f6_112px", 1, 8, 16, 30, 112, m=6, seed=187),                     # 19 tiles per row: two row pieces of 16
    Layer("s_f6_24px_c130", 2, 130, 64, 24, 24, m=6, seed=188),                # 4 tiles per row, ragged channel block
    Layer("s_flex_f2_c512_k70_1024tiles", 16, 512, 70, 16, 16, m=2, flex_sigma=0.02, seed=185),
]


@pytest.mark.parametrize("layer", SMALL, ids=lambda l: l.name)
def test_small_int8_all_taps(oracle, layer):
    case = make_case(oracle, layer)
    _check_i8(case, run_gpu(case))


@pytest.mark.parametrize("layer", SMALL, ids=lambda l: l.name)
def test_small_fp32(oracle, layer):
    from dataclasses import replace
    case = make_case(oracle, replace(layer, dtype="f32"))
    _check_f32(oracle, case, run_gpu(case))


def test_flex_small_int8_and_fp32(oracle):
    from dataclasses import replace
    L = Layer("flex_small", 2, 24, 40, 10, 10, m=6, flex_sigma=0.01, seed=108)
    case = make_case(oracle, L)
    _check_i8(case, run_gpu(case))
    case = make_case(oracle, replace(L, dtype="f32"))
    _check_f32(oracle, case, run_gpu(case))
    L4 = Layer("flex_small4", 2, 24, 40, 10, 10, m=4, flex_sigma=0.05, seed=109)
    case = make_case(oracle, L4)
    _check_i8(case, run_gpu(case))
    # two blocks of input channels through the vector-ALU one-kernel forward (F2, few tiles)
    L2 = Layer("flex_f2_c100", 2, 100, 40, 12, 12, m=2, flex_sigma=0.03, seed=170)
    case = make_case(oracle, L2)
    _check_i8(case, run_gpu(case))


def test_saturation_and_m_quantizer(oracle):
    """Deliberately small scales drive every stage into saturation; the optional
    quantizer after the Hadamard stage is switched on."""
    L = Layer("sat", 2, 32, 16, 12, 12, m=4, seed=110)
    case = make_case(oracle, L, with_oracle=False)
    sc = dict(case["scales"])
    sc["s_v"] *= 0.25
    sc["s_u"] *= 0.5
    sc["s_y"] *= 0.3
    sc["s_m"] = sc["s_u"] * sc["s_v"] * 400.0
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc)
    out = run_gpu(case, scales=sc)
    for tap, key in (("U", "Uq"), ("V", "Vq"), ("Y", "Yq")):
        assert np.abs(case["ref"][key]).max() == 127 and case["ref"][key].min() >= -127
    _check_i8(case, out)
    sc["qmax"] = 7                                  # a 4-bit-ish quantizer through the same path
    case["ref"] = oracle.winograd_q(case["xq"].astype(np.int32) // 19, case["g"], case["BT"],
                                    case["G"], case["AT"], sc, qmax=7)
    case["xq"] = (case["xq"].astype(np.int32) // 19).astype(np.int8)
    _check_i8(case, run_gpu(case, scales=sc))


@pytest.mark.parametrize("m", [2, 4])
def test_many_tiles_ragged_flex_and_m_quantizer(oracle, m):
    """Few channels, many tiles: large enough (>= 256 workgroups of 16 tiles x 64 output
    channels) for the kernels that are only chosen on big grids, with ragged tiles
    (30 = 7.5 tiles of 4), K not a multiple of 4, dense (perturbed) matrices, and the
    optional quantizer after the Hadamard stage; then the same with the default
    matrices in fp32."""
    from dataclasses import replace
    L = Layer("many_tiles_m%d" % m, 32 if m == 4 else 10, 16, 70, 30, 30, m=m, flex_sigma=0.02,
              seed=124 + m)
    case = make_case(oracle, L, with_oracle=False)
    sc = dict(case["scales"])
    sc["s_m"] = sc["s_u"] * sc["s_v"] * 3.0
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc)
    _check_i8(case, run_gpu(case, scales=sc))
    case = make_case(oracle, replace(L, flex_sigma=0.0))          # Cook-Toom pattern, no s_m
    _check_i8(case, run_gpu(case))
    case = make_case(oracle, replace(L, flex_sigma=0.0, dtype="f32"))
    _check_f32(oracle, case, run_gpu(case))


@pytest.mark.parametrize("layer", [
    Layer("pos_f4", 3, 40, 70, 16, 16, m=4, seed=131),            # matrix-core input stage
    Layer("pos_f2_ragged", 2, 20, 24, 9, 11, m=2, seed=132),      # vector-ALU input stage
    Layer("pos_f6", 2, 12, 33, 14, 14, m=6, seed=133),
    Layer("pos_f4_flex", 2, 24, 40, 10, 10, m=4, flex_sigma=0.05, seed=134),
    Layer("pos_f2_c256", 2, 256, 40, 8, 8, m=2, seed=135),        # long reduction, fused GEMM + output
    Layer("pos_f6_c128", 1, 128, 70, 16, 16, m=6, seed=136),
    # the one-kernel forward with per-position factors: eight-wavefront form (one and two
    # LDS regions), two channel blocks, ragged tiles, byte-wise staging
    Layer("pos_f4_c100_k128", 3, 100, 128, 16, 16, m=4, seed=137),
    Layer("pos_f2_k72_8px", 2, 64, 72, 8, 8, m=2, seed=138),
    Layer("pos_f2_c128_k64", 2, 128, 64, 12, 12, m=2, seed=139),
    Layer("pos_f4_7px", 5, 24, 20, 7, 7, m=4, seed=140),
    Layer("pos_f2_2px", 9, 64, 40, 2, 2, m=2, seed=165),
    Layer("pos_f2_c512_k64_1024tiles", 64, 512, 64, 8, 8, m=2, seed=186),   # 32 x 64 workgroup tiles
], ids=lambda l: l.name)
def test_per_position_scales_all_taps(oracle, layer):
    """One quantizer scale per Winograd position for V and U (Sec. 7), calibrated by the
    oracle; every tap bit-exact; then the same with the Hadamard-stage quantizer on."""
    case = make_case(oracle, layer, with_oracle=False)
    sc = oracle.calibrate_pos(case["X"], case["g"], case["BT"], case["G"], case["AT"], pad=layer.pad)
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"]).astype(np.int8)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                                    pad=layer.pad)
    assert np.abs(case["ref"]["Vq"]).reshape(case["ref"]["Vq"].shape[0], -1).max(axis=1).min() >= 100
    _check_i8(case, run_gpu(case, scales=sc))
    sc = dict(sc, s_m=float(np.abs(case["ref"]["M"] * case["ref"]["scalars"]["w"][:, None, None]).max()) / 100.0)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                                    pad=layer.pad)
    _check_i8(case, run_gpu(case, scales=sc))


@pytest.mark.parametrize("layer", [
    Layer("denseA_f4", 3, 64, 64, 16, 16, m=4, seed=166),
    Layer("denseA_f2_c70_k100", 2, 70, 100, 9, 11, m=2, seed=167),
], ids=lambda l: l.name)
def test_learned_output_matrix_with_exact_input_matrix(oracle, layer):
    """A^T and G learned (dense), B^T left at its Cook-Toom values: the matrix-core input
    transform feeds the one-kernel forward with a dense output transform; per-tensor scales,
    then per-position scales with the Hadamard-stage quantizer."""
    case = make_case(oracle, layer, with_oracle=False)
    _, G, AT = workloads.perturb_transforms(case["BT"], case["G"], case["AT"], 0.05, layer.seed)
    case["G"], case["AT"] = G, AT
    BT = case["BT"]
    assert np.count_nonzero(AT) == AT.size
    sc = oracle.calibrate(case["X"], case["g"], BT, G, AT, pad=layer.pad)
    case["scales"] = sc
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"]).astype(np.int8)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], BT, G, AT, sc, pad=layer.pad)
    _check_i8(case, run_gpu(case))
    sc = oracle.calibrate_pos(case["X"], case["g"], BT, G, AT, pad=layer.pad)
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"]).astype(np.int8)
    ref = oracle.winograd_q(case["xq"], case["g"], BT, G, AT, sc, pad=layer.pad)
    sc = dict(sc, s_m=float(np.abs(ref["M"] * ref["scalars"]["w"][:, None, None]).max()) / 100.0)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], BT, G, AT, sc, pad=layer.pad)
    _check_i8(case, run_gpu(case, scales=sc))


def _random_layers(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        m = int(rng.choice([2, 4, 6]))
        pad = int(rng.integers(0, 2))
        H, W = int(rng.integers(3, 41)), int(rng.integers(3, 41))
        if H + 2 * pad - 2 < 1 or W + 2 * pad - 2 < 1:
            continue
        out.append(Layer("rnd%d" % len(out), int(rng.integers(1, 5)), int(rng.integers(1, 141)),
                         int(rng.integers(1, 141)), H, W, m=m, pad=pad,
                         flex_sigma=float(rng.choice([0.0, 0.0, 0.03])), seed=1000 + len(out)))
    return out


@pytest.mark.parametrize("layer", _random_layers(36, 7), ids=lambda l: "%s_%dx%dx%dx%dx%d_m%d_p%d%s" % (
    l.name, l.N, l.C, l.K, l.H, l.W, l.m, l.pad, "_flex" if l.flex_sigma else ""))
def test_random_shapes_int8_and_fp32(oracle, layer):
    """Seeded random shapes across every dispatch path: all int8 taps bit-exact, fp32 within
    tolerance."""
    from dataclasses import replace
    case = make_case(oracle, layer)
    _check_i8(case, run_gpu(case))
    case = make_case(oracle, replace(layer, dtype="f32"))
    _check_f32(oracle, case, run_gpu(case))


@pytest.mark.parametrize("layer", _random_layers(24, 11), ids=lambda l: "%s_%dx%dx%dx%dx%d_m%d_p%d%s" % (
    l.name, l.N, l.C, l.K, l.H, l.W, l.m, l.pad, "_flex" if l.flex_sigma else ""))
def test_random_shapes_per_position_scales_and_m_quantizer(oracle, layer):
    """Seeded random shapes with one scale per Winograd position and the Hadamard-stage
    quantizer on: every int8 tap bit-exact on whichever kernel sequence the shape takes."""
    case = make_case(oracle, layer, with_oracle=False)
    sc = oracle.calibrate_pos(case["X"], case["g"], case["BT"], case["G"], case["AT"], pad=layer.pad)
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"]).astype(np.int8)
    ref = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                            pad=layer.pad)
    peak = float(np.abs(ref["M"] * ref["scalars"]["w"][:, None, None]).max())
    sc = dict(sc, s_m=max(peak, 1e-20) / 100.0)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                                    pad=layer.pad)
    _check_i8(case, run_gpu(case, scales=sc))


def test_input_at_an_odd_address(oracle):
    """x need not be aligned: the staging falls back to unaligned dword loads."""
    import torch
    from paper_2002_10711_amd import binding as wb
    L = Layer("odd_x", 2, 64, 64, 16, 16, m=4, seed=145)
    case = make_case(oracle, L)
    sc = case["scales"]
    dev = torch.device("cuda:0")
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8, BT=case["BT"], G=case["G"],
                   AT=case["AT"])
    quant = wb.make_quant(sc["s_x"], sc["s_v"], sc["s_u"], sc["s_y"])
    buf = torch.zeros(case["xq"].size + 3, dtype=torch.int8, device=dev)
    for shift in (1, 2):
        x = buf[shift:shift + case["xq"].size].view(case["xq"].shape)
        x.copy_(torch.from_numpy(case["xq"]))
        assert x.data_ptr() % 4 == shift
        U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
        ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        y = torch.zeros((L.N, L.K, 16, 16), dtype=torch.int8, device=dev)
        wb.wino_transform_weights(desc, quant, torch.from_numpy(case["g"]).to(dev), U)
        wb.wino_conv2d_fwd(desc, quant, x, U, y, ws)
        y2 = torch.zeros_like(y)
        for stage in (wb.WINO_STAGE_INPUT, wb.WINO_STAGE_GEMM, wb.WINO_STAGE_OUTPUT):
            wb.wino_conv2d_fwd_stages(desc, quant, x, U, y2, ws, stage)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), case["ref"]["Yq"])
        assert np.array_equal(y2.cpu().numpy(), case["ref"]["Yq"])


@pytest.mark.parametrize("flex", [0.0, 0.03], ids=["matrix_core_input", "vector_alu_input"])
def test_output_at_an_odd_address(oracle, flex):
    """y need not be aligned either: the one-kernel forwards then leave their branch-free
    output side (2- and 4-byte stores) for byte stores."""
    import torch
    from paper_2002_10711_amd import binding as wb
    L = Layer("odd_y", 2, 64, 64, 16, 16, m=4, flex_sigma=flex, seed=187)
    case = make_case(oracle, L)
    sc = case["scales"]
    dev = torch.device("cuda:0")
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8, BT=case["BT"], G=case["G"],
                   AT=case["AT"])
    assert wb.wino_fwd_num_kernels(desc) == 1
    quant = wb.make_quant(sc["s_x"], sc["s_v"], sc["s_u"], sc["s_y"])
    x = torch.from_numpy(case["xq"]).to(dev)
    U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wb.wino_transform_weights(desc, quant, torch.from_numpy(case["g"]).to(dev), U)
    numel = L.N * L.K * 16 * 16
    buf = torch.full((numel + 3,), 99, dtype=torch.int8, device=dev)
    for shift in (1, 2, 3):
        y = buf[shift:shift + numel].view(L.N, L.K, 16, 16)
        assert y.data_ptr() % 4 == shift
        buf.fill_(99)
        wb.wino_conv2d_fwd(desc, quant, x, U, y, ws)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), case["ref"]["Yq"])
        edge = buf.cpu().numpy()
        assert (edge[:shift] == 99).all() and (edge[shift + numel:] == 99).all()


# the one-kernel F(2x2,3x3) forward on grids of more than a thousand workgroups, with several
# blocks of output channels; the F(6x6,3x3) input stage with three tiles per wavefront where
# the tile rows leave tile slots of the workgroup empty (5 of 8, 11 of 16)
EXTRA = [
    Layer("f2_1120_workgroups", 70, 64, 64, 32, 32, m=2, seed=195),
    Layer("f2_k200_1280_workgroups", 20, 40, 200, 32, 32, m=2, seed=196),
    Layer("f6_tw5", 3, 64, 32, 20, 28, m=6, seed=197),
    Layer("f6_tw11", 1, 64, 32, 12, 64, m=6, seed=198),
]


@pytest.mark.parametrize("layer", EXTRA, ids=lambda l: l.name)
def test_large_grids_and_three_tile_input_stage(oracle, layer):
    case = make_case(oracle, layer)
    _check_i8(case, run_gpu(case))


NONUNIT = [
    # Cook-Toom matrices from point lists that keep A^T's zero pattern but not its leading
    # ones (first nonzero point 2 or 1/2 instead of 1): the kernels whose chains start with
    # the term itself must not be taken; every sequence still has to give the oracle's codes
    (Layer("nonunit_f2", 3, 40, 70, 12, 12, m=2, seed=230), (0, 2, -2)),
    (Layer("nonunit_f4", 2, 64, 64, 16, 16, m=4, seed=231), (0, "1/2", "-1/2", 1, -1)),
    (Layer("nonunit_f4_c256", 2, 256, 64, 8, 8, m=4, seed=232), (0, 2, -2, 1, -1)),
    (Layer("nonunit_f6", 2, 64, 40, 16, 16, m=6, seed=233), (0, 2, -2, 1, -1, "1/2", "-1/2")),
]


@pytest.mark.parametrize("layer,points", NONUNIT, ids=lambda v: v.name if hasattr(v, "name") else "pts")
def test_sparse_matrices_without_unit_leading_entries(oracle, layer, points):
    from fractions import Fraction
    X, g = workloads.make_inputs(layer)
    BT, G, AT = oracle.cook_toom(layer.m, points=[Fraction(p) for p in points], dtype=np.float32)
    n = layer.m + 2
    assert AT[1, 1] != 1.0 and np.count_nonzero(AT) == np.count_nonzero(oracle.cook_toom(layer.m)[2])
    case = dict(layer=layer, X=X, g=g, BT=BT, G=G, AT=AT)
    sc = oracle.calibrate(X, g, BT, G, AT, pad=layer.pad)
    case["scales"] = sc
    case["xq"] = oracle.quantize_tensor(X, sc["s_x"]).astype(np.int8)
    case["ref"] = oracle.winograd_q(case["xq"], g, BT, G, AT, sc, pad=layer.pad)
    _check_i8(case, run_gpu(case), inexact_ok=True)


TROW = [
    # F(6x6,3x3) GEMM + output kernel on whole rows of tiles (sequence "trow"): several
    # workgroups with a partly filled last one, output channels that do not fill a block of
    # 32, every reduction length it is built for, images whose last row of tiles is cut
    Layer("tr_32px", 3, 64, 64, 32, 32, m=6, seed=190),                 # 18 rows of 6 tiles, 5 per workgroup
    Layer("tr_16px_c128_k40", 7, 128, 40, 16, 16, m=6, seed=191),       # 21 rows of 3 tiles, 10 per workgroup
    Layer("tr_48x20_c200_k70", 2, 200, 70, 20, 48, m=6, seed=192),      # 8 tiles per row, 256 padded channels
    Layer("tr_pad0_34px_k33", 2, 40, 33, 34, 34, m=6, pad=0, seed=193),
    Layer("tr_flex_16px_c100", 5, 100, 64, 16, 16, m=6, flex_sigma=0.01, seed=194),   # dense A^T
]


@pytest.mark.parametrize("layer", TROW, ids=lambda l: l.name)
def test_rows_of_tiles_kernel_all_taps(oracle, layer):
    case = make_case(oracle, layer)
    out = run_gpu(case)
    assert "trow" in out["Y_seq"]
    _check_i8(case, out)
    # ... with one scale per position and the Hadamard-stage quantizer on
    case = make_case(oracle, layer, with_oracle=False)
    sc = oracle.calibrate_pos(case["X"], case["g"], case["BT"], case["G"], case["AT"], pad=layer.pad)
    case["xq"] = oracle.quantize_tensor(case["X"], sc["s_x"]).astype(np.int8)
    ref = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                            pad=layer.pad)
    peak = float(np.abs(ref["M"] * ref["scalars"]["w"][:, None, None]).max())
    sc = dict(sc, s_m=max(peak, 1e-20) / 100.0)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc,
                                    pad=layer.pad)
    out = run_gpu(case, scales=sc)
    assert "trow" in out["Y_seq"]
    _check_i8(case, out)


def test_rows_of_tiles_kernel_needs_16_byte_aligned_output(oracle):
    """The kernel stores 16-byte pieces; an output at any other address takes the
    column-wise kernel instead, named or not."""
    import torch
    from paper_2002_10711_amd import binding as wb
    L = TROW[0]
    case = make_case(oracle, L)
    sc = case["scales"]
    dev = torch.device("cuda:0")
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8, BT=case["BT"], G=case["G"],
                   AT=case["AT"])
    assert wb.wino_fwd_sequence(desc, wb.WINO_SEQ_TROW) == wb.WINO_SEQ_TROW
    quant = wb.make_quant(sc["s_x"], sc["s_v"], sc["s_u"], sc["s_y"])
    x = torch.from_numpy(case["xq"]).to(dev)
    U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wb.wino_transform_weights(desc, quant, torch.from_numpy(case["g"]).to(dev), U)
    numel = case["ref"]["Yq"].size
    buf = torch.full((numel + 16,), 99, dtype=torch.int8, device=dev)
    for shift in (0, 4, 9):
        base = (-buf.data_ptr()) % 16 + shift
        y = buf[base:base + numel].view(case["ref"]["Yq"].shape)
        assert y.data_ptr() % 16 == shift
        buf.fill_(99)
        wb.wino_conv2d_fwd_seq(desc, quant, x, U, y, ws, wb.WINO_SEQ_TROW)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), case["ref"]["Yq"]), shift
        got = buf.cpu().numpy()
        assert (got[:base] == 99).all() and (got[base + numel:] == 99).all(), shift


def test_quantizer_factor_too_small_for_the_exact_scaling(oracle):
    """The matrix-core input transform divides the quantizer factor s_x / s_v by 4^s, exactly;
    a factor that underflows there makes its launcher decline, and the call must take the
    vector-ALU kernels instead of failing (every code of V is then 0, like the oracle's)."""
    L = Layer("tiny_rv", 2, 64, 64, 16, 16, m=4, seed=188)
    case = make_case(oracle, L, with_oracle=False)
    sc = dict(case["scales"])
    sc["s_x"] = float(np.float32(2.0 ** -148))
    sc["s_v"] = 1.0
    assert np.float32(sc["s_x"]) / np.float32(sc["s_v"]) / np.float32(16) == 0
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc)
    assert not case["ref"]["Vq"].any()
    _check_i8(case, run_gpu(case, scales=sc))
    # the same with more output channels than one kernel handles without the exact transform
    L2 = Layer("tiny_rv_k128", 2, 64, 128, 16, 16, m=4, seed=189)
    case = make_case(oracle, L2, with_oracle=False)
    case["ref"] = oracle.winograd_q(case["xq"], case["g"], case["BT"], case["G"], case["AT"], sc)
    _check_i8(case, run_gpu(case, scales=sc))


def test_reductions_beyond_512_channels(oracle):
    """More than 512 input channels take the three-kernel sequence (tiled GEMM writing M).
    600 channels on config-shaped data; then 1100 channels with same-sign codes close to
    saturation, so that accumulators pass 2^24 and (float)M has to round (to nearest, ties to
    even) exactly as the oracle's conversion does -- the oracle counts such accumulators."""
    from paper_2002_10711_amd import binding as wb
    for L in (Layer("c600_f4", 2, 600, 70, 9, 11, m=4, seed=190),
              Layer("c600_f2", 3, 600, 40, 8, 8, m=2, seed=191)):
        case = make_case(oracle, L)
        desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8, BT=case["BT"], G=case["G"],
                       AT=case["AT"])
        assert wb.wino_fwd_num_kernels(desc) == 3
        _check_i8(case, run_gpu(case))
    L = Layer("c1100_f2_rounding", 2, 1100, 40, 6, 6, m=2, seed=192)
    rng = np.random.default_rng(L.seed)
    BT, G, AT = oracle.cook_toom(2, dtype=np.float32)
    xq = rng.integers(100, 128, (L.N, L.C, L.H, L.W)).astype(np.int8)
    g = rng.uniform(0.5, 1.0, (L.K, L.C, 3, 3)).astype(np.float32)
    sc = dict(s_x=1.0, s_v=3.5, s_u=0.0135, s_y=1.0, s_m=0.0, qmax=127)
    ref = oracle.winograd_q(xq, g, BT, G, AT, sc, pad=1)
    sc["s_y"] = float(np.abs(ref["M"]).max() * sc["s_u"] * sc["s_v"] / 100.0)
    ref = oracle.winograd_q(xq, g, BT, G, AT, sc, pad=1)
    odd_large = int(((np.abs(ref["M"]) > 2 ** 24) & (ref["M"] % 2 != 0)).sum())
    assert ref["inexact"] > 100 and odd_large > 100 and np.abs(ref["Yq"]).max() >= 99
    case = dict(layer=L, X=None, g=g, BT=BT, G=G, AT=AT, scales=sc, xq=xq, ref=ref)
    _check_i8(case, run_gpu(case), inexact_ok=True)


def test_config2_int8_full(oracle):
    case = make_case(oracle, workloads.config2("i8")[0])
    _check_i8(case, run_gpu(case))


def test_config2_fp32_full(oracle):
    case = make_case(oracle, workloads.config2("f32")[0])
    _check_f32(oracle, case, run_gpu(case))


@pytest.mark.parametrize("layer", workloads.config3(), ids=lambda l: l.name)
def test_config3_int8_full(oracle, layer):
    case = make_case(oracle, layer)
    _check_i8(case, run_gpu(case))


def test_config4_flex_int8_full(oracle):
    case = make_case(oracle, workloads.config4()[0])
    _check_i8(case, run_gpu(case))


@pytest.mark.parametrize("layer", [l for l in workloads.config5() if l.stride == 1],
                         ids=lambda l: l.name)
def test_config5_full_batch_first_and_last_images(oracle, layer):
    """The stack's Winograd layers at the benchmarked batch of 256, so that every kernel runs
    in the launch configuration that is timed; the oracle computes the first and the last
    eight images (tiles do not interact across the batch), scales calibrated on the first
    eight."""
    X, g = workloads.make_inputs(layer)
    BT, G, AT = oracle.cook_toom(layer.m, dtype=np.float32)
    sc = oracle.calibrate(X[:8], g, BT, G, AT, pad=layer.pad)
    xq = oracle.quantize_tensor(X, sc["s_x"]).astype(np.int8)
    case = dict(layer=layer, X=X, g=g, BT=BT, G=G, AT=AT, scales=sc, xq=xq)
    out = run_gpu(case, taps=False)
    for sl in (slice(0, 8), slice(layer.N - 8, layer.N)):
        ref = oracle.winograd_q(xq[sl], g, BT, G, AT, sc, pad=layer.pad)
        for key in ("Y", "Y_staged"):
            bad = int((out[key][sl] != ref["Yq"]).sum())
            assert bad == 0, "%s images %s: %d codes differ" % (key, sl, bad)
    assert np.abs(out["Y"]).max() >= 100


def test_determinism(oracle):
    case = make_case(oracle, Layer("det", 4, 64, 64, 16, 16, m=4, seed=111), with_oracle=False)
    a, b = run_gpu(case), run_gpu(case)
    for k in a:
        if k == "Y_seq":
            assert a[k].keys() == b[k].keys()
            for name in a[k]:
                assert np.array_equal(a[k][name], b[k][name]), (k, name)
        else:
            assert np.array_equal(a[k], b[k]), k
