"""Host-side tests of the C ABI: the library loads, exports every symbol the header
declares, and every error path is reachable without a GPU (argument checks happen
before the first HIP call).  No compute is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2002_10711_amd import binding as wb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(wb.LIB_PATH):
        from paper_2002_10711_amd import build
        build.build()
    return wb.lib()


def _declared_functions():
    txt = open(os.path.join(ROOT, "include", "wino.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b((?:wino|conv2d_ref)_[a-z0-9_]+)\s*\(", txt)))


def test_every_declared_symbol_is_exported(L):
    names = _declared_functions()
    assert set(names) == set(wb.EXPORTS), (names, wb.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def _desc(**kw):
    d = dict(N=1, C=16, K=16, H=8, W=8, pad=1, m=2, dtype=wb.WINO_F32)
    d.update(kw)
    m = d["m"] if d["m"] in (2, 4, 6) else 2
    n = m + 2
    return wb.Desc(d["N"], d["C"], d["K"], d["H"], d["W"], d["pad"], d["m"], d["dtype"],
                   BT=np.eye(n, dtype=np.float32), G=np.ones((n, 3), np.float32),
                   AT=np.ones((m, n), np.float32))


def test_sizes(L):
    d = _desc()
    # F2, T=16 -> Tp=64, C=16 -> Cp=16 (float), K -> Kp=64, P=16
    assert wb.wino_weights_bytes(d) == 16 * 64 * 16 * 4
    assert wb.wino_workspace_bytes(d) == 16 * 64 * 16 * 4 + 16 * 64 * 64 * 4
    d = _desc(N=64, C=64, K=64, H=32, W=32, m=4, dtype=wb.WINO_I8)
    assert wb.wino_weights_bytes(d) == 36 * 64 * 64
    assert wb.wino_workspace_bytes(d) == 36 * 4096 * 64 + 36 * 4096 * 64 * 4
    for bad in (dict(m=3), dict(N=0), dict(pad=2), dict(dtype=7), dict(H=1, W=1, pad=0)):
        assert wb.wino_weights_bytes(_desc(**bad)) == 0
        assert wb.wino_workspace_bytes(_desc(**bad)) == 0


def _fwd(L, d, q, x=0x1000, U=0x1000, y=0x1000, ws=0x1000, nbytes=1 << 40):
    qp = ctypes.byref(q) if q is not None else None
    return L.wino_conv2d_fwd(d.ref, qp, x, U, y, ws, nbytes, None)


def test_error_codes_without_gpu(L):
    q = wb.make_quant(0.1, 0.1, 0.1, 0.1)
    assert L.wino_conv2d_fwd(None, None, 1, 1, 1, 1, 0, None) == -1
    assert _fwd(L, _desc(m=3), None) == -2
    assert _fwd(L, _desc(m=8), None) == -2
    assert _fwd(L, _desc(C=0), None) == -3
    assert _fwd(L, _desc(pad=2), None) == -3
    assert _fwd(L, _desc(H=2, W=2, pad=0), None) == -3
    assert _fwd(L, _desc(N=1 << 20, C=1 << 10, H=64, W=64), None) == -3     # index range
    assert _fwd(L, _desc(dtype=5), None) == -4
    assert _fwd(L, _desc(), None, x=None) == -1
    assert _fwd(L, _desc(), None, ws=None) == -1
    d = _desc()
    d.c.BT = None
    assert _fwd(L, d, None) == -1
    assert _fwd(L, _desc(dtype=wb.WINO_I8), None) == -5                     # quant missing
    for bad in (dict(s_x=0.0), dict(s_v=-1.0), dict(s_u=float("nan")), dict(s_y=float("inf")),
                dict(s_m=-0.5), dict(qmax=0), dict(qmax=128)):
        kw = dict(s_x=0.1, s_v=0.1, s_u=0.1, s_y=0.1, s_m=0.0, qmax=127)
        kw.update(bad)
        assert _fwd(L, _desc(dtype=wb.WINO_I8), wb.make_quant(**kw)) == -5, bad
    d = _desc()
    d._keep[0][1, 1] = np.inf
    assert _fwd(L, d, None) == -5
    assert _fwd(L, _desc(), None, nbytes=100) == -6
    assert _fwd(L, _desc(), None, ws=0x1010) == -6                           # misaligned
    # weights entry point
    assert L.wino_transform_weights(_desc().ref, None, None, 0x1000, None) == -1
    assert L.wino_transform_weights(_desc(dtype=wb.WINO_I8).ref, None, 0x1000, 0x1000, None) == -5
    assert L.wino_transform_weights(_desc(m=5).ref, None, 0x1000, 0x1000, None) == -2
    assert L.wino_transform_weights(_desc().ref, None, 0x1000, 0x1004, None) == -6
    # taps
    assert L.wino_debug_export(_desc().ref, 9, 0x1000, 0x1000, None) == -8
    assert L.wino_debug_export(_desc().ref, 0, None, 0x1000, None) == -1
    assert q.qmax == 127
    for s in range(-9, 1):
        assert len(wb.status_string(s)) > 1


def test_ref_conv_error_codes_without_gpu(L):
    f = lambda **kw: L.conv2d_ref_gpu(*[kw.get(k, v) for k, v in (
        ("N", 1), ("C", 8), ("K", 8), ("H", 8), ("W", 8), ("stride", 1), ("pad", 1),
        ("dtype", wb.WINO_I8), ("x", 0x1000), ("wp", 0x1000), ("y", 0x1000), ("s_x", 0.1),
        ("s_w", 0.1), ("s_y", 0.1), ("qmax", 127), ("ws", 0x1000), ("nbytes", 1 << 40),
        ("stream", None))])
    assert f(stride=3) == -8
    assert f(dtype=3) == -4
    assert f(N=0) == -3
    assert f(pad=3) == -3
    assert f(H=1, W=1, pad=0) == -3
    assert f(x=None) == -1
    assert f(s_w=0.0) == -5
    assert f(qmax=200) == -5
    assert f(nbytes=10) == -6
    assert wb.conv2d_ref_workspace_bytes(1, 8, 8, 8, 8, 1, 1, wb.WINO_I8) == 64 * 9 * 64 + 64 * 64 * 4
    assert wb.conv2d_ref_workspace_bytes(1, 8, 8, 8, 8, 2, 1, wb.WINO_F32) == 64 * 9 * 16 * 4 + 64 * 64 * 4
    # int8: the tap-major rows and the copy in MFMA operand order
    assert wb.conv2d_ref_packed_weights_bytes(8, 8, wb.WINO_I8) == 2 * 64 * 9 * 64
    assert wb.conv2d_ref_packed_weights_bytes(0, 8, wb.WINO_I8) == 0
    assert L.conv2d_ref_pack_weights(8, 8, wb.WINO_I8, None, 0x1000, None) == -1
    assert L.conv2d_ref_pack_weights(8, 8, 9, 0x1000, 0x1000, None) == -4


@pytest.mark.parametrize("m", [2, 4, 6])
def test_library_cook_toom_matches_oracle(L, oracle, m):
    """The library's own generator (host code, independent implementation) gives the
    correctly rounded fp32 matrices of the exact construction."""
    BT, G, AT = wb.wino_cook_toom(m)
    oBT, oG, oAT = oracle.cook_toom(m, dtype=np.float32)
    assert np.array_equal(BT, oBT) and np.array_equal(G, oG) and np.array_equal(AT, oAT)


def test_library_cook_toom_custom_points_and_errors(L, oracle):
    from fractions import Fraction
    pts = [0.0, 1.0, -1.0, 2.0, -2.0]
    BT, G, AT = wb.wino_cook_toom(4, pts)
    oBT, oG, oAT = oracle.cook_toom(4, [Fraction(p) for p in pts], dtype=np.float32)
    assert np.array_equal(BT, oBT) and np.array_equal(G, oG) and np.array_equal(AT, oAT)
    assert L.wino_cook_toom(3, None, 1, 1, 1) == -2
    assert L.wino_cook_toom(2, None, None, 1, 1) == -1
    dup = np.array([0.0, 1.0, 1.0])
    b = np.zeros(64, np.float32)
    assert L.wino_cook_toom(2, dup.ctypes.data, b.ctypes.data, b.ctypes.data, b.ctypes.data) == -8


def test_mfma_probe_argument_checks():
    """Argument errors of the matrix-core probe come back before any HIP call."""
    from paper_2002_10711_amd import binding as wb
    L = wb.lib()
    import ctypes
    assert L.wino_debug_mfma_loop(wb.WINO_I8, 8, 10, None, None, None) == -1        # WINO_E_NULL
    buf = (ctypes.c_float * 4)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert L.wino_debug_mfma_loop(wb.WINO_I8, 0, 10, p, None, None) == -3           # bad shape
    assert L.wino_debug_mfma_loop(wb.WINO_I8, 8, 0, p, None, None) == -3
    assert L.wino_debug_mfma_loop(7, 8, 10, p, None, None) == -4                    # bad dtype
    # the memory-path probe: pointers, then mode / wavefronts, then sizes
    assert L.wino_debug_load_loop(0, 4, 8, 4096, 10, None, p, None, None) == -1
    assert L.wino_debug_load_loop(4, 4, 8, 4096, 10, p, p, None, None) == -8
    assert L.wino_debug_load_loop(0, 5, 8, 4096, 10, p, p, None, None) == -8
    assert L.wino_debug_load_loop(0, 4, 8, 4000, 10, p, p, None, None) == -3          # not whole chunks
    assert L.wino_debug_load_loop(0, 4, 0, 4096, 10, p, p, None, None) == -3


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: any other --gpus value ends with a message, before
    anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)


def test_per_position_scale_argument_checks(L):
    """Both per-position arrays or neither; every entry finite and positive -- checked
    before any HIP call."""
    import ctypes
    import numpy as np
    from paper_2002_10711_amd import binding as wb
    BT, G, AT = wb.wino_cook_toom(4)
    d = wb.Desc(1, 8, 8, 8, 8, 1, 4, wb.WINO_I8, BT=BT, G=G, AT=AT)
    fake = ctypes.c_void_p(256)          # never dereferenced: the checks come first
    ok = np.full(36, 0.5, np.float32)
    q = wb.make_quant(0.1, 1.0, 1.0, 0.2, s_v_pos=ok, s_u_pos=ok)
    q.s_u_pos = None                                      # only one of the two
    assert L.wino_transform_weights(d.ref, ctypes.byref(q), fake, fake, None) == -5
    bad = ok.copy()
    bad[7] = 0.0
    q = wb.make_quant(0.1, 1.0, 1.0, 0.2, s_v_pos=ok, s_u_pos=bad)
    assert L.wino_transform_weights(d.ref, ctypes.byref(q), fake, fake, None) == -5
    bad[7] = np.inf
    q = wb.make_quant(0.1, 1.0, 1.0, 0.2, s_v_pos=bad, s_u_pos=ok)
    assert L.wino_transform_weights(d.ref, ctypes.byref(q), fake, fake, None) == -5


def test_wide_mode_sizes_and_argument_checks(L):
    """The modes with 16-bit codes in the Winograd domain: buffer sizes (two int8 digit planes
    per code of U and V, int64 M), the channel limit of the exact digit arithmetic, one code
    range per quantizer with the limit of its container -- all checked before any HIP call."""
    d = _desc(N=64, C=64, K=64, H=32, W=32, m=4, dtype=wb.WINO_I16)
    assert wb.wino_weights_bytes(d) == 36 * 64 * 64 * 2
    assert wb.wino_workspace_bytes(d) == 36 * 4096 * 64 * 2 + 36 * 4096 * 64 * 8
    assert wb.wino_workspace_bytes(_desc(C=3, dtype=wb.WINO_I8W16)) == 16 * 64 * 64 * 2 + 16 * 64 * 64 * 8
    assert wb.wino_weights_bytes(_desc(C=1024, dtype=wb.WINO_I16)) > 0
    assert wb.wino_weights_bytes(_desc(C=1025, dtype=wb.WINO_I16)) == 0
    assert _fwd(L, _desc(C=1025, dtype=wb.WINO_I8W16), wb.make_quant(1, 1, 1, 1)) == -3
    assert _fwd(L, _desc(dtype=wb.WINO_I16), None) == -5                    # quant missing
    kw = dict(s_x=0.1, s_v=0.1, s_u=0.1, s_y=0.1, s_m=0.0)
    for dtype, q, want in (
            (wb.WINO_I16, dict(qmax=32768), -5),
            (wb.WINO_I16, dict(qmax=127, qmax_v=40000), -5),
            (wb.WINO_I16, dict(qmax=127, qmax_m=-1), -5),
            (wb.WINO_I8W16, dict(qmax=32767), -5),               # output codes live in int8
            (wb.WINO_I8W16, dict(qmax=127, qmax_y=128), -5),
            (wb.WINO_I8, dict(qmax=127, qmax_v=63), -5),         # int8 mode: one range for all
            (wb.WINO_I8, dict(qmax=127, qmax_u=127, qmax_v=127, qmax_m=127, qmax_y=127), -6),
            (wb.WINO_I8W16, dict(qmax=127, qmax_u=32767, qmax_v=511, qmax_m=8191), -6),
            (wb.WINO_I16, dict(qmax=32767), -6)):
        # (-6: every argument check passed, the 100-byte workspace is what is refused)
        assert _fwd(L, _desc(dtype=dtype), wb.make_quant(**kw, **q), nbytes=100) == want, (dtype, q)
    # int16 tensors must be 2-byte aligned
    q = wb.make_quant(**kw, qmax=32767)
    assert _fwd(L, _desc(dtype=wb.WINO_I16), q, x=0x1001) == -8
    assert _fwd(L, _desc(dtype=wb.WINO_I16), q, y=0x1001) == -8


def test_bench_algorithmic_work_of_config2():
    """The bytes and operations the benchmark prices its kernels with, for the headline layer
    (N=64, 64->64, 32x32, F(4x4,3x3), int8), against values worked out by hand from Eq. 1 and
    the GEMM formulation of Sec. 5.3: 4096 tiles, 36 positions; X and Y 64*64*32*32 bytes,
    V 36*4096*64, U 36*64*64, M 4*36*4096*64; GEMM 2*36*4096*64*64 operations; direct
    convolution 2*64*64*32*32*64*9."""
    import os
    import sys
    import numpy as np
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    from paper_2002_10711_amd import binding as wb, workloads
    L = workloads.config2("i8")[0]
    BT, G, AT = wb.wino_cook_toom(4)
    a = bench.algorithmic(L, np.asarray(BT), np.asarray(AT))
    x = y = 4194304
    v, u, m = 9437184, 147456, 37748736
    assert a["input_transform"]["bytes"] == x + v
    assert a["gemm"]["bytes"] == v + u + m and a["gemm"]["ops"] == 1207959552
    assert a["output_transform"]["bytes"] == m + y
    assert a["gemm_output"]["bytes"] == v + u + y
    assert a["fused_forward"]["bytes"] == x + u + y and a["fused_forward"]["ops"] == 1207959552
    assert a["weight_transform"]["bytes"] == 9 * 64 * 64 * 4 + u
    assert 2 * L.N * L.K * L.Ho * L.Wo * L.C * 9 == 4831838208
    # the input transform of this layer runs on the matrix cores: three 16x16x64 MFMAs per 16
    # windows (36 positions in groups of 16) are matrix-core work, only the quantizer's four
    # operations per element remain vector-ALU work
    kron = 4096 * 64 * 3 * 16 * 64 * 2
    assert a["input_transform"]["mfma_issued"] == kron and a["input_transform"]["ops"] == 0
    assert a["fused_forward"]["mfma_issued"] == 1207959552 + kron
    assert a["input_transform"]["alu"] == 4096 * 64 * 36 * 4
    # which roofline bounds a kernel: bytes at 8 TB/s against GEMM operations at 5 POP/s
    e = bench.roofline_entry("fused_forward", a["fused_forward"], 10.0, "i8", None)
    assert e["bound"] == "hbm" and abs(e["hbm_frac"] - (x + u + y) / 10e-6 / 8e12) < 1e-12
    assert abs(e["mfma_frac"] - 1207959552 / 10e-6 / 5e15) < 1e-12 and e["frac"] == e["hbm_frac"]
    L5 = [l for l in workloads.config5() if l.name == "cfg5_l15_512to512_s4_F2"][0]
    BT2, _, AT2 = wb.wino_cook_toom(2)
    a5 = bench.algorithmic(L5, np.asarray(BT2), np.asarray(AT2))
    e5 = bench.roofline_entry("gemm_output", a5["gemm_output"], 10.0, "i8", None)
    # (V 16*1024*512 + U 16*512*512 + Y 256*512*16 bytes need 1.835 us at 8 TB/s, the
    # 8.59 G operations 1.718 us at 5 POP/s: the two roofs of this layer all but coincide)
    assert a5["gemm_output"]["ops"] == 2 * 16 * 1024 * 512 * 512
    assert a5["gemm_output"]["bytes"] == 16 * 1024 * 512 + 16 * 512 * 512 + 256 * 512 * 16
    assert e5["bound"] == "hbm" and 0.9 < e5["mfma_frac"] / e5["hbm_frac"] < 1.0
    # the 16-bit-stage workload: two bytes per code of X, Y, U, V, eight per accumulator
    # taken to memory, four int8 digit products per 16-bit product
    Lw = workloads.config2("i16")[0]
    w = bench.algorithmic(Lw, np.asarray(BT), np.asarray(AT))
    assert w["gemm_output"]["bytes"] == 2 * (v + u + y) and w["gemm"]["bytes"] == 2 * (v + u) + 2 * m
    assert w["gemm"]["ops"] == 4 * 1207959552


def test_kernel_sequences_of_the_named_workloads():
    """Which kernel sequence the forward takes for the benchmark's workloads (decided on the
    host from the descriptor alone, so no GPU is needed): one kernel for the 64- and
    128-channel F2/F4 layers, two (input stage, GEMM + output) for long reductions and for
    the 16-bit stages, three where few tiles or F(6x6,3x3) leave the tiled GEMM ahead."""
    from paper_2002_10711_amd import binding as wb, workloads
    dt = {"i8": wb.WINO_I8, "f32": wb.WINO_F32, "i16": wb.WINO_I16, "i8w16": wb.WINO_I8W16}

    def nk(L):
        BT, G, AT = wb.wino_cook_toom(L.m)
        return wb.wino_fwd_num_kernels(wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, dt[L.dtype],
                                               BT=BT, G=G, AT=AT))
    assert nk(workloads.config1()[0]) == 1
    assert nk(workloads.config2("i8")[0]) == 1 and nk(workloads.config2("f32")[0]) == 1
    assert nk(workloads.config2("i16")[0]) == 2 and nk(workloads.config2("i8w16")[0]) == 2
    c3 = {L.name: nk(L) for L in workloads.config3()}
    assert c3 == {"cfg3_c256_s8_F2": 2, "cfg3_c256_s8_F4": 2, "cfg3_c512_s4_F2": 2,
                  "cfg3_c512_s4_F4": 3}
    c5 = {L.name: nk(L) for L in workloads.config5() if L.stride == 1}
    assert [c5[k] for k in sorted(c5)] == [1, 2, 1, 1, 2, 1, 1, 2, 2, 2, 3, 3, 2]


def test_bf16_mode_is_limited_to_the_one_kernel_forward():
    """WINO_BF16 (float path, bf16 GEMM operands) is built for m in {2, 4}: m = 6 is an error
    of the descriptor, stage-by-stage calls and taps are refused, all before any HIP call."""
    import ctypes
    BT, G, AT = wb.wino_cook_toom(6)
    d6 = wb.Desc(1, 16, 16, 12, 12, 1, 6, wb.WINO_BF16, BT=BT, G=G, AT=AT)
    assert wb.wino_fwd_num_kernels(d6) == 0 and wb.wino_weights_bytes(d6) == 0
    lib = wb.lib()
    assert lib.wino_transform_weights(d6.ref, None, 0x1000, 0x1000, None) == -2
    BT, G, AT = wb.wino_cook_toom(4)
    d4 = wb.Desc(2, 16, 16, 12, 12, 1, 4, wb.WINO_BF16, BT=BT, G=G, AT=AT)
    assert wb.wino_fwd_num_kernels(d4) == 1
    assert wb.wino_weights_bytes(d4) > 0 and wb.wino_workspace_bytes(d4) > 0
    ws = wb.wino_workspace_bytes(d4)
    for stage in (wb.WINO_STAGE_INPUT, wb.WINO_STAGE_GEMM, wb.WINO_STAGE_OUTPUT):
        assert lib.wino_conv2d_fwd_stages(d4.ref, None, 0x1000, 0x1000, 0x1000, 0x1000, ws, stage, None) == -8
    assert lib.wino_debug_export(d4.ref, wb.WINO_TAP_U, 0x1000, 0x1000, None) == -4
    assert wb.wino_fwd_sequence(d4, wb.WINO_SEQ_AUTO) == 0
