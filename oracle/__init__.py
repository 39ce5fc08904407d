"""CPU oracle for the Winograd-aware convolution forward path (Python face).

TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the
CPU-baseline leg of the benchmark may import this package.  It never imports the
HIP library or its binding, and the library never imports it.

The arithmetic lives in ``wino_oracle.cpp`` (plain C++, compiled with g++ into
``liboracle.so`` next to this file) and in ``cook_toom.py`` (exact rationals).
This module only marshals numpy arrays across ctypes and strings the stages of
the quantized pipeline together in the order of the paper's Fig. 2 / Sec. 3.2:
quantize input -> B^T d B -> quantize ; G g G^T -> quantize ; Hadamard product
summed over input channels -> (optional quantizer) ; A^T M A -> quantize.
"""
import ctypes
import os
import subprocess

import numpy as np

from .cook_toom import DEFAULT_POINTS, cook_toom, cook_toom_exact  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wino_oracle.cpp")
# WINO_ORACLE_LIB names an already built copy (the sanitizer test passes an
# instrumented build of the same source); it is loaded as it is, not rebuilt.
_PREBUILT = os.environ.get("WINO_ORACLE_LIB")
_LIB = _PREBUILT or os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with g++ (no fast-math, no contraction)."""
    if _PREBUILT:
        return _LIB
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["g++", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_q_output.restype = ctypes.c_int64
        L.oracle_q_output_pos.restype = ctypes.c_int64
        L.oracle_q_output_bits.restype = ctypes.c_int64
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def num_threads():
    return int(lib().oracle_num_threads())


def set_num_threads(nt):
    lib().oracle_set_num_threads(ctypes.c_int(int(nt)))


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def geometry(N, H, W, pad, m):
    """Ho, Wo, TH, TW, T, n, P for stride-1 F(m x m, 3 x 3)."""
    Ho, Wo = H + 2 * pad - 2, W + 2 * pad - 2
    TH, TW = -(-Ho // m), -(-Wo // m)
    n = m + 2
    return dict(Ho=Ho, Wo=Wo, TH=TH, TW=TW, T=N * TH * TW, n=n, P=n * n)


# ------------------------------------------------------------------ O1 -----
def conv2d_direct_f64(X, g, stride=1, pad=1):
    X = _c(X, np.float64)
    g = _c(g, np.float64)
    N, C, H, W = X.shape
    K = g.shape[0]
    assert g.shape == (K, C, 3, 3)
    Ho = (H + 2 * pad - 3) // stride + 1
    Wo = (W + 2 * pad - 3) // stride + 1
    Y = np.zeros((N, K, Ho, Wo), np.float64)
    rc = lib().oracle_conv2d_direct_f64(N, C, K, H, W, stride, pad, _p(X), _p(g), _p(Y))
    assert rc == 0
    return Y


def conv2d_direct_q(Xq, gq, r_y, qmax=127, stride=1, pad=1):
    """Integer direct convolution + one requantization; returns (acc int64, y int32)."""
    Xq = _c(Xq, np.int32)
    gq = _c(gq, np.int32)
    N, C, H, W = Xq.shape
    K = gq.shape[0]
    assert gq.shape == (K, C, 3, 3)
    Ho = (H + 2 * pad - 3) // stride + 1
    Wo = (W + 2 * pad - 3) // stride + 1
    acc = np.zeros((N, K, Ho, Wo), np.int64)
    Yq = np.zeros((N, K, Ho, Wo), np.int32)
    rc = lib().oracle_conv2d_direct_q(N, C, K, H, W, stride, pad, _p(Xq), _p(gq),
                                      ctypes.c_float(r_y), int(qmax), _p(acc), _p(Yq))
    assert rc == 0
    return acc, Yq


# ------------------------------------------------------------------ O2 -----
def winograd_f64(X, g, BT, G, AT, pad=1):
    X = _c(X, np.float64)
    g = _c(g, np.float64)
    BT = _c(BT, np.float64)
    G = _c(G, np.float64)
    AT = _c(AT, np.float64)
    N, C, H, W = X.shape
    K = g.shape[0]
    m = AT.shape[0]
    n = m + 2
    assert BT.shape == (n, n) and G.shape == (n, 3) and AT.shape == (m, n)
    Y = np.zeros((N, K, H + 2 * pad - 2, W + 2 * pad - 2), np.float64)
    rc = lib().oracle_winograd_f64(N, C, K, H, W, pad, m, _p(BT), _p(G), _p(AT),
                                   _p(X), _p(g), _p(Y))
    assert rc == 0
    return Y


# ------------------------------------------------------------------ O3 -----
def bf16_round(a):
    """fp32 values rounded to the nearest bf16 (8 significant bits), ties to even, returned
    as fp32.  Finite inputs only."""
    bits = np.ascontiguousarray(a, np.float32).view(np.uint32)
    bits = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return bits.view(np.float32)


def _fma32(a, b, c):
    """fp32 fused multiply-add on arrays: the product of two fp32 numbers is exact in fp64,
    the fp64 sum is then rounded once to fp32 (the fp64 sum itself rounds only when the terms
    are more than 2^5 apart in magnitude, and a wrong final bit then needs an exact fp32 tie
    after that rounding: about one case in 2^29)."""
    return (np.asarray(a, np.float64) * np.asarray(b, np.float64) + np.asarray(c, np.float64)).astype(np.float32)


def input_f32(X, BT, pad=1):
    """V = B^T d B of every tile of a FLOAT input in the pinned fp32 arithmetic (chains
    acc = +0; acc = fma(B^T[i][j], d[j][l], acc) over ascending j, left product first):
    what oracle_q_input computes for integer codes, here for any fp32 X.  Returns
    V [P, T, C] fp32, t = (img*TH + th)*TW + tw."""
    X = np.asarray(X, np.float32)
    BT = np.asarray(BT, np.float32)
    N, C, H, W = X.shape
    n = BT.shape[0]
    m = n - 2
    geo = geometry(N, H, W, pad, m)
    TH, TW = geo["TH"], geo["TW"]
    Xp = np.zeros((N, C, pad + TH * m + n, pad + TW * m + n), np.float32)
    Xp[:, :, pad:pad + H, pad:pad + W] = X
    d = np.stack([Xp[:, :, th * m:th * m + n, tw * m:tw * m + n]
                  for th in range(TH) for tw in range(TW)], axis=1)          # [N, TH*TW, C, n, n]
    d = d.reshape(N * TH * TW, C, n, n)
    w = np.zeros_like(d)
    for i in range(n):
        acc = np.zeros(d[:, :, 0, :].shape, np.float32)
        for j in range(n):
            acc = _fma32(BT[i, j], d[:, :, j, :], acc)
        w[:, :, i, :] = acc
    V = np.zeros_like(d)
    for k in range(n):
        acc = np.zeros(d[:, :, :, 0].shape, np.float32)
        for l in range(n):
            acc = _fma32(w[:, :, :, l], BT[k, l], acc)
        V[:, :, :, k] = acc
    return np.ascontiguousarray(V.transpose(2, 3, 0, 1).reshape(n * n, N * TH * TW, C))


def winograd_bf16(X, g, BT, G, AT, pad=1):
    """The float path with bf16 operands in the per-position GEMM (the speed variant of the
    GEMM stage, Sec. 5.3): U = G g G^T and V = B^T d B in the pinned fp32 arithmetic, each
    rounded to bf16 (nearest even), multiplied and summed over the input channels exactly
    (fp64), and transformed back with A^T in fp64.  Returns Y [N, K, Ho, Wo] in fp64."""
    AT = np.asarray(AT, np.float64)
    N, C, H, W = np.shape(X)
    K = np.shape(g)[0]
    m = AT.shape[0]
    n = m + 2
    geo = geometry(N, H, W, pad, m)
    TH, TW, Ho, Wo = geo["TH"], geo["TW"], geo["Ho"], geo["Wo"]
    Uf, _ = q_weights(g, G, want_q=False)                       # [P, K, C] fp32, pinned chains
    Ub = bf16_round(Uf).astype(np.float64)
    Vb = bf16_round(input_f32(X, BT, pad)).astype(np.float64)   # [P, T, C]
    Mt = np.einsum("ptc,pkc->ptk", Vb, Ub).reshape(n, n, N, TH, TW, K)
    Yt = np.einsum("ai,ijnhwk,bj->nkhawb", AT, Mt, AT).reshape(N, K, TH * m, TW * m)
    return np.ascontiguousarray(Yt[:, :, :Ho, :Wo])


def q_scalars(s_x, s_v, s_u, s_y, s_m=0.0):
    out = [ctypes.c_float() for _ in range(4)]
    lib().oracle_q_scalars(ctypes.c_float(s_x), ctypes.c_float(s_v), ctypes.c_float(s_u),
                           ctypes.c_float(s_y), ctypes.c_float(s_m),
                           *[ctypes.byref(o) for o in out])
    r_u, r_v, r_m, r_y = [np.float32(o.value) for o in out]
    return dict(r_u=r_u, r_v=r_v, r_m=r_m, r_y=r_y)


def q_scalars_pos(s_x, s_v_pos, s_u_pos, s_y, s_m=0.0):
    """Host scalars of the per-position variant: arrays r_u, r_v, w (one entry per
    Winograd position) and the two scalars r_m, r_y."""
    sv = _c(s_v_pos, np.float32)
    su = _c(s_u_pos, np.float32)
    P = sv.size
    assert su.size == P
    r_u, r_v, w = (np.zeros(P, np.float32) for _ in range(3))
    r_m, r_y = ctypes.c_float(), ctypes.c_float()
    lib().oracle_q_scalars_pos(P, ctypes.c_float(s_x), _p(sv), _p(su), ctypes.c_float(s_y),
                               ctypes.c_float(s_m), _p(r_u), _p(r_v), _p(w),
                               ctypes.byref(r_m), ctypes.byref(r_y))
    return dict(r_u=r_u, r_v=r_v, w=w, r_m=np.float32(r_m.value), r_y=np.float32(r_y.value))


def _per_position(r, P):
    a = np.asarray(r, np.float32)
    return np.ascontiguousarray(np.broadcast_to(a, (P,)) if a.ndim == 0 else a.reshape(P))


def q_weights(g, G, r_u=1.0, qmax=127, want_f32=True, want_q=True):
    """U = G g G^T in pinned fp32; returns (U_f32 [P,K,C] or None, Uq int32 or None).
    r_u: one factor, or one per Winograd position."""
    g = _c(g, np.float32)
    G = _c(G, np.float32)
    K, C = g.shape[:2]
    n = G.shape[0]
    m = n - 2
    P = n * n
    Uf = np.zeros((P, K, C), np.float32) if want_f32 else None
    Uq = np.zeros((P, K, C), np.int32) if want_q else None
    if np.ndim(r_u) == 0:
        rc = lib().oracle_q_weights(K, C, m, _p(G), _p(g), ctypes.c_float(r_u), int(qmax),
                                    _p(Uf), _p(Uq))
    else:
        rc = lib().oracle_q_weights_pos(K, C, m, _p(G), _p(g), _p(_per_position(r_u, P)),
                                        int(qmax), _p(Uf), _p(Uq))
    assert rc == 0
    return Uf, Uq


def q_input(xq, BT, pad=1, r_v=1.0, qmax=127, want_f32=True, want_q=True):
    """V = B^T d B per tile in pinned fp32; returns (V_f32 [P,T,C] or None, Vq or None).
    r_v: one factor, or one per Winograd position."""
    xq = _c(xq, np.int32)
    BT = _c(BT, np.float32)
    N, C, H, W = xq.shape
    n = BT.shape[0]
    m = n - 2
    geo = geometry(N, H, W, pad, m)
    Vf = np.zeros((geo["P"], geo["T"], C), np.float32) if want_f32 else None
    Vq = np.zeros((geo["P"], geo["T"], C), np.int32) if want_q else None
    if np.ndim(r_v) == 0:
        rc = lib().oracle_q_input(N, C, H, W, pad, m, _p(BT), _p(xq), ctypes.c_float(r_v),
                                  int(qmax), _p(Vf), _p(Vq))
    else:
        rc = lib().oracle_q_input_pos(N, C, H, W, pad, m, _p(BT), _p(xq),
                                      _p(_per_position(r_v, geo["P"])), int(qmax), _p(Vf), _p(Vq))
    assert rc == 0
    return Vf, Vq


def q_hadamard(Vq, Uq):
    """M[p,t,k] = sum_c Vq[p,t,c] Uq[p,k,c], exact int64."""
    Vq = _c(Vq, np.int32)
    Uq = _c(Uq, np.int32)
    P, T, C = Vq.shape
    K = Uq.shape[1]
    assert Uq.shape == (P, K, C)
    M = np.zeros((P, T, K), np.int64)
    rc = lib().oracle_q_hadamard(P, ctypes.c_int64(T), C, K, _p(Vq), _p(Uq), _p(M))
    assert rc == 0
    return M


def q_output(M, AT, N, H, W, pad=1, r_m=0.0, r_y=1.0, qmax=127, want_f32=True, want_q=True,
             w_pos=None, qmax_m=None):
    """Y tile = A^T M A in pinned fp32; returns (Y_f32 unscaled or None, Yq or None, inexact).
    w_pos: per-position factors that bring M to real units first (per-position scales).
    qmax is the range of the output codes; qmax_m (default: the same) that of the
    Hadamard-stage quantizer."""
    M = _c(M, np.int64)
    AT = _c(AT, np.float32)
    m, n = AT.shape
    geo = geometry(N, H, W, pad, m)
    P, T, K = M.shape
    assert P == geo["P"] and T == geo["T"]
    Yf = np.zeros((N, K, geo["Ho"], geo["Wo"]), np.float32) if want_f32 else None
    Yq = np.zeros((N, K, geo["Ho"], geo["Wo"]), np.int32) if want_q else None
    inexact = lib().oracle_q_output_bits(
        N, K, H, W, pad, m, _p(AT), _p(M), _p(None if w_pos is None else _per_position(w_pos, P)),
        ctypes.c_float(r_m), ctypes.c_float(r_y), int(qmax if qmax_m is None else qmax_m),
        int(qmax), _p(Yf), _p(Yq))
    assert inexact >= 0
    return Yf, Yq, int(inexact)


def stage_qmax(qmax):
    """Code ranges of the five quantizers (input x, transformed weights u, transformed
    input v, Hadamard stage m, output y) from one integer or a dict with those keys
    (missing keys: 127) -- Sec. 3.2 lets every stage have its own bit-width."""
    if isinstance(qmax, dict):
        return {k: int(qmax.get(k, 127)) for k in "xuvmy"}
    return {k: int(qmax) for k in "xuvmy"}


def quantize_tensor(x, scale, qmax=127):
    """Per-tensor symmetric quantizer of Sec. 5.1: sat(rne(x / scale)), in fp32."""
    v = np.asarray(x, np.float32) / np.float32(scale)
    return np.clip(np.rint(v), -qmax, qmax).astype(np.int32)


def calibrate(X, g, BT, G, AT, pad=1, qmax=127, with_m=False):
    """Static max-abs scales for the quantizers (stand-in for the paper's warmed-up moving
    averages, Table 1 caption).  Each scale is the max-abs of the stage's value range
    divided by that stage's qmax (an integer, or per stage as in stage_qmax), over the
    whole tensor (per-layer scale, Sec. 5.1), computed with the pipeline's own arithmetic,
    stage after stage.  with_m: also a scale for the quantizer after the Hadamard stage."""
    f32 = np.float32
    qm = stage_qmax(qmax)
    s_x = f32(np.abs(np.asarray(X, f32)).max() / f32(qm["x"]))
    xq = quantize_tensor(X, s_x, qm["x"])
    Vf, _ = q_input(xq, BT, pad=pad, want_q=False)
    s_v = f32(s_x * f32(np.abs(Vf).max()) / f32(qm["v"]))
    Uf, _ = q_weights(g, G, want_q=False)
    s_u = f32(np.abs(Uf).max() / f32(qm["u"]))
    sc = q_scalars(s_x, s_v, s_u, 1.0)
    _, Vq = q_input(xq, BT, pad=pad, r_v=sc["r_v"], qmax=qm["v"], want_f32=False)
    _, Uq = q_weights(g, G, r_u=sc["r_u"], qmax=qm["u"], want_f32=False)
    M = q_hadamard(Vq, Uq)
    N, _, H, W = xq.shape
    s_m = f32(0)
    if with_m:
        s_m = f32(f32(s_u * s_v) * f32(np.abs(M).max()) / f32(qm["m"]))
        scm = q_scalars(s_x, s_v, s_u, 1.0, s_m)
        Yf, _, _ = q_output(M, AT, N, H, W, pad=pad, r_m=scm["r_m"], qmax_m=qm["m"], want_q=False)
        s_y = f32(s_m * f32(np.abs(Yf).max()) / f32(qm["y"]))
    else:
        Yf, _, _ = q_output(M, AT, N, H, W, pad=pad, want_q=False)
        s_y = f32(f32(s_u * s_v) * f32(np.abs(Yf).max()) / f32(qm["y"]))
    return dict(s_x=float(s_x), s_v=float(s_v), s_u=float(s_u), s_y=float(s_y), s_m=float(s_m))


def calibrate_pos(X, g, BT, G, AT, pad=1, qmax=127):
    """As calibrate, with one max-abs scale per Winograd position for the transformed
    input and the transformed weights ("s_v_pos", "s_u_pos"; a position that is zero
    everywhere gets the scale 1)."""
    f32 = np.float32
    s_x = f32(np.abs(np.asarray(X, f32)).max() / f32(qmax))
    xq = quantize_tensor(X, s_x, qmax)
    Vf, _ = q_input(xq, BT, pad=pad, want_q=False)
    Uf, _ = q_weights(g, G, want_q=False)
    P = Vf.shape[0]
    vmax = np.abs(Vf).reshape(P, -1).max(axis=1).astype(f32)
    umax = np.abs(Uf).reshape(P, -1).max(axis=1).astype(f32)
    s_v = np.where(vmax > 0, s_x * vmax / f32(qmax), f32(1)).astype(f32)
    s_u = np.where(umax > 0, umax / f32(qmax), f32(1)).astype(f32)
    sc = q_scalars_pos(s_x, s_v, s_u, 1.0)
    _, Vq = q_input(xq, BT, pad=pad, r_v=sc["r_v"], qmax=qmax, want_f32=False)
    _, Uq = q_weights(g, G, r_u=sc["r_u"], qmax=qmax, want_f32=False)
    M = q_hadamard(Vq, Uq)
    N, _, H, W = xq.shape
    Yf, _, _ = q_output(M, AT, N, H, W, pad=pad, want_q=False, w_pos=sc["w"])
    s_y = f32(f32(np.abs(Yf).max()) / f32(qmax))
    return dict(s_x=float(s_x), s_v_pos=s_v, s_u_pos=s_u, s_y=float(s_y), s_m=0.0)


def winograd_q(xq, g, BT, G, AT, scales, pad=1, qmax=127):
    """The whole quantized forward, every tap returned.  xq: int input at scale s_x.
    With "s_v_pos" / "s_u_pos" in scales: the per-position variant.  qmax: one code range
    for every stage, or one per stage (stage_qmax)."""
    qm = stage_qmax(qmax)
    N, _, H, W = np.asarray(xq).shape
    if "s_v_pos" in scales:
        sc = q_scalars_pos(scales["s_x"], scales["s_v_pos"], scales["s_u_pos"], scales["s_y"],
                           scales.get("s_m", 0.0))
        w_pos = sc["w"]
    else:
        sc = q_scalars(scales["s_x"], scales["s_v"], scales["s_u"], scales["s_y"],
                       scales.get("s_m", 0.0))
        w_pos = None
    _, Uq = q_weights(g, G, r_u=sc["r_u"], qmax=qm["u"], want_f32=False)
    _, Vq = q_input(xq, BT, pad=pad, r_v=sc["r_v"], qmax=qm["v"], want_f32=False)
    M = q_hadamard(Vq, Uq)
    _, Yq, inexact = q_output(M, AT, N, H, W, pad=pad, r_m=sc["r_m"], r_y=sc["r_y"],
                              qmax=qm["y"], qmax_m=qm["m"], want_f32=False, w_pos=w_pos)
    return dict(Uq=Uq, Vq=Vq, M=M, Yq=Yq, inexact=inexact, scalars=sc)
