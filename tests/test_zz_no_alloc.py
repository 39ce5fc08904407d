"""The allocation-free forward (wino_conv2d_fwd_noalloc) against wino_conv2d_fwd, through the
C ABI: same output codes on two calls in a row, the second on a smaller problem (the
built-in scratch buffer then still holds the first call's V and M), and the size limit."""
import numpy as np
import pytest

from paper_2002_10711_amd.workloads import Layer

pytestmark = pytest.mark.gpu


def _problem(L, seed):
    import torch
    from paper_2002_10711_amd import binding as wb
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed)
    BT, G, AT = wb.wino_cook_toom(L.m)
    i8 = L.dtype == "i8"
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8 if i8 else wb.WINO_F32,
                   BT=BT, G=G, AT=AT)
    if i8:
        x = torch.from_numpy(rng.integers(-127, 128, size=(L.N, L.C, L.H, L.W)).astype(np.int8)).to(dev)
        quant = wb.make_quant(1.0, 6.0, 2e-3, 30.0 * (L.C / 256) ** 0.5)
    else:
        x = torch.from_numpy(rng.standard_normal((L.N, L.C, L.H, L.W)).astype(np.float32)).to(dev)
        quant = None
    g = torch.from_numpy((rng.standard_normal((L.K, L.C, 3, 3)) * 0.05).astype(np.float32)).to(dev)
    U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
    wb.wino_transform_weights(desc, quant, g, U)
    return desc, quant, x, U


def _both(L, seed):
    import torch
    from paper_2002_10711_amd import binding as wb
    desc, quant, x, U = _problem(L, seed)
    dev = x.device
    Ho, Wo = L.H + 2 * L.pad - 2, L.W + 2 * L.pad - 2
    dt = torch.int8 if L.dtype == "i8" else torch.float32
    y_ref = torch.full((L.N, L.K, Ho, Wo), 77, dtype=dt, device=dev)
    y_new = torch.full((L.N, L.K, Ho, Wo), 55, dtype=dt, device=dev)
    ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    wb.wino_conv2d_fwd(desc, quant, x, U, y_ref, ws)
    wb.wino_conv2d_fwd_noalloc(desc, quant, x, U, y_new)
    torch.cuda.synchronize()
    a, b = y_ref.cpu().numpy(), y_new.cpu().numpy()
    assert np.abs(a.astype(np.float64)).max() > 0
    return a, b, wb.wino_fwd_num_kernels(desc)


def _pick(cands, kernels):
    """The first of the candidate layers that the measured dispatch table runs as `kernels`
    kernels (which sequence a shape takes is the table's business and changes when it is
    re-measured; the scratch buffer's uses are what this test is after)."""
    from paper_2002_10711_amd import binding as wb
    for L in cands:
        BT, G, AT = wb.wino_cook_toom(L.m)
        desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8, BT=BT, G=G, AT=AT)
        if wb.wino_fwd_num_kernels(desc) == kernels:
            return L
    raise AssertionError("no candidate runs as %d kernels" % kernels)


def test_two_calls_in_a_row_the_second_smaller():
    # first: F4, 256 or 512 channels, few tiles: three kernels, V and M both in the scratch buffer
    big = _pick([Layer("na_big", 8, 256, 256, 8, 8, m=4), Layer("na_big", 4, 512, 256, 8, 8, m=4),
                 Layer("na_big", 8, 600, 128, 8, 8, m=4)], 3)
    a, b, nk = _both(big, 1)
    assert nk == 3
    assert np.array_equal(a, b)
    # then a smaller one on the same buffer: F2, two kernels (V only), ragged tiles
    small = _pick([Layer("na_small", 3, 120, 140, 13, 11, m=2), Layer("na_small", 3, 200, 140, 13, 11, m=2),
                   Layer("na_small", 5, 300, 140, 13, 11, m=2)], 2)
    a, b, nk = _both(small, 2)
    assert nk == 2
    assert np.array_equal(a, b)
    # one kernel (no scratch at all) and fp32 (bit-identical: same kernels, same order)
    a, b, nk = _both(_pick([Layer("na_fused", 3, 64, 64, 16, 16, m=4),
                            Layer("na_fused", 8, 64, 64, 32, 32, m=4)], 1), 3)
    assert nk == 1
    assert np.array_equal(a, b)
    a, b, _ = _both(Layer("na_f32", 2, 160, 160, 12, 12, m=6, dtype="f32"), 4)
    assert np.array_equal(a, b)


def test_size_limit_and_argument_checks():
    from paper_2002_10711_amd import binding as wb
    # 64 -> 64 channels at 32 x 32, F6, batch 256: two kernels, and V alone (64 positions x
    # 9216 tiles x 64 channels = 37.7 MB) is beyond the buffer
    L = Layer("na_too_big", 256, 64, 64, 32, 32, m=6)
    BT, G, AT = wb.wino_cook_toom(L.m)
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, wb.WINO_I8, BT=BT, G=G, AT=AT)
    assert wb.wino_fwd_num_kernels(desc) == 2
    assert 64 * 9216 * 64 > wb.NOALLOC_SCRATCH_BYTES
    quant = wb.make_quant(1.0, 6.0, 2e-3, 30.0)
    lib = wb.lib()
    import ctypes
    assert lib.wino_conv2d_fwd_noalloc(desc.ref, ctypes.byref(quant), 0x1000, 0x1000, 0x1000, None) == -9
    assert "scratch" in wb.status_string(-9)
    # the ordinary argument checks come first and need no GPU
    assert lib.wino_conv2d_fwd_noalloc(desc.ref, ctypes.byref(quant), None, 0x1000, 0x1000, None) == -1
    assert lib.wino_conv2d_fwd_noalloc(desc.ref, None, 0x1000, 0x1000, 0x1000, None) == -5
    assert lib.wino_conv2d_fwd_noalloc(None, None, 0x1000, 0x1000, 0x1000, None) == -1
