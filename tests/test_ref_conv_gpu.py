"""The im2row baseline against the oracle's direct convolution: int8 bit-exact
(integer accumulation, one requantization), fp32 within 1e-5 of fp64."""
import numpy as np
import pytest

from paper_2002_10711_amd.workloads import Layer, make_inputs

from helpers import max_rel

pytestmark = pytest.mark.gpu

CASES = [
    Layer("r1", 2, 20, 24, 9, 11, stride=1, seed=201),
    Layer("r2", 3, 64, 128, 16, 16, stride=2, seed=202),
    Layer("r3", 2, 7, 5, 7, 5, stride=2, seed=203),
    Layer("r4", 1, 130, 70, 6, 10, stride=1, pad=0, seed=204),
    Layer("r5", 8, 64, 64, 32, 32, stride=1, seed=205),
    # several whole images per workgroup, the last group ragged; two chunks of channels
    Layer("r6_4x4_out", 5, 100, 128, 8, 8, stride=2, seed=206),
    Layer("r7_4x4_in", 7, 64, 130, 4, 4, stride=1, seed=207),
    # more than 64 output columns: two column blocks; rows not a multiple of four wide
    Layer("r8_wide", 1, 8, 16, 5, 70, stride=1, seed=208),
    Layer("r9_wide_s2", 1, 8, 16, 7, 141, stride=2, seed=209),
    # one output pixel per image
    Layer("r10_1x1", 70, 9, 12, 3, 3, stride=1, pad=0, seed=210),
    Layer("r11_30", 2, 16, 64, 30, 30, stride=1, seed=211),
    # whole images of 4 or 8 columns (gathered plane by plane): one image per workgroup, no
    # padding with an odd row count of pieces, 48 pixels per image, stride 2 on 4 columns
    Layer("r12_8x8", 3, 70, 64, 8, 8, stride=1, seed=212),
    Layer("r13_6x8_pad0", 6, 64, 128, 6, 8, stride=1, pad=0, seed=213),
    Layer("r14_12x4", 3, 130, 64, 12, 4, stride=1, seed=214),
    Layer("r15_8x4_s2", 9, 64, 192, 8, 4, stride=2, seed=215),
]
ENTRY = ["conv2d_ref_gpu", "conv2d_ref_gpu_rows"]


def _run(L, x_np, w_np, i8, s=(1.0, 1.0, 1.0), entry="conv2d_ref_gpu", odd=False):
    import torch
    from paper_2002_10711_amd import binding as wb
    dev = torch.device("cuda:0")
    dt = wb.WINO_I8 if i8 else wb.WINO_F32
    x, w = torch.from_numpy(x_np).to(dev), torch.from_numpy(w_np).to(dev)
    wp = torch.empty(wb.conv2d_ref_packed_weights_bytes(L.C, L.K, dt), dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.conv2d_ref_workspace_bytes(L.N, L.C, L.K, L.H, L.W, L.stride, L.pad, dt),
                     dtype=torch.uint8, device=dev)
    y = torch.full((L.N, L.K, L.Ho, L.Wo), 77, dtype=torch.int8 if i8 else torch.float32, device=dev)
    if odd:                                  # both tensors one element off their allocation
        xb = torch.empty(x.numel() + 1, dtype=x.dtype, device=dev)
        yb = torch.full((y.numel() + 2,), 77, dtype=y.dtype, device=dev)
        xb[1:].copy_(x.reshape(-1))
        x, y = xb[1:], yb[1:-1].view(y.shape)
    wb.conv2d_ref_pack_weights(L.C, L.K, dt, w, wp)
    getattr(wb, entry)(L.N, L.C, L.K, L.H, L.W, L.stride, L.pad, dt, x, wp, y, s[0], s[1], s[2],
                       127, ws)
    torch.cuda.synchronize()
    if odd:
        assert int(yb[0]) == 77 and int(yb[-1]) == 77        # nothing written outside y
    return y.cpu().numpy()


@pytest.mark.parametrize("entry,odd", [("conv2d_ref_gpu", False), ("conv2d_ref_gpu", True),
                                       ("conv2d_ref_gpu_rows", False)],
                         ids=["one_kernel", "one_kernel_odd_addresses", "three_kernels"])
@pytest.mark.parametrize("L", CASES, ids=lambda l: l.name)
def test_ref_conv_int8(oracle, L, entry, odd):
    X, g = make_inputs(L)
    s_x, s_w = np.float32(np.abs(X).max() / 127), np.float32(np.abs(g).max() / 127)
    xq, wq = oracle.quantize_tensor(X, s_x), oracle.quantize_tensor(g, s_w)
    acc, _ = oracle.conv2d_direct_q(xq, wq, 1.0, stride=L.stride, pad=L.pad)
    s_y = np.float32(s_x * s_w * np.abs(acc).max() / 127 * 0.8)      # a little saturation
    r_y = np.float32(np.float32(s_x * s_w) / s_y)
    _, Yq = oracle.conv2d_direct_q(xq, wq, r_y, stride=L.stride, pad=L.pad)
    print("case", L.name, entry, "odd" if odd else "aligned", flush=True)
    y = _run(L, xq.astype(np.int8), wq.astype(np.int8), True, (float(s_x), float(s_w), float(s_y)),
             entry, odd)
    assert np.abs(Yq).max() == 127
    assert np.array_equal(y.astype(np.int32), Yq)


@pytest.mark.parametrize("L", CASES, ids=lambda l: l.name)
def test_ref_conv_fp32(oracle, L):
    X, g = make_inputs(L)
    ref = oracle.conv2d_direct_f64(X, g, L.stride, L.pad)
    y = _run(L, X, g, False)
    assert y.shape == ref.shape and max_rel(y, ref) <= 1e-5


@pytest.mark.gpu
def test_mfma_probe_runs_and_counts_its_operations():
    import torch
    from paper_2002_10711_amd import binding as wb
    out = torch.zeros(64 * 256, dtype=torch.float32, device="cuda:0")
    ops = wb.wino_debug_mfma_loop(wb.WINO_I8, 64, 10, out)
    torch.cuda.synchronize()
    assert ops == 2.0 * 16 * 16 * 64 * 8 * 10 * 4 * 64
    ops = wb.wino_debug_mfma_loop(wb.WINO_F32, 64, 10, out)
    torch.cuda.synchronize()
    assert ops == 2.0 * 16 * 16 * 4 * 8 * 10 * 4 * 64
    assert torch.isfinite(out).all()


@pytest.mark.gpu
def test_memory_path_probe_runs_and_counts_its_bytes():
    import torch
    from paper_2002_10711_amd import binding as wb
    wgs, kb = 32, 64
    buf = torch.ones(wgs * (kb << 10), dtype=torch.uint8, device="cuda:0")
    out = torch.zeros(wgs * 1024, dtype=torch.float32, device="cuda:0")
    for mode, bpl in ((0, 16), (1, 8), (2, 4), (3, 16)):
        for waves in (4, 8, 16):
            nbytes = wb.wino_debug_load_loop(mode, waves, wgs, kb << 10, 5, buf, out)
            torch.cuda.synchronize()
            assert nbytes == wgs * waves * 64 * bpl * 8 * 5
    assert torch.isfinite(out).all()
