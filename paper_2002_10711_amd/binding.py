"""ctypes binding of libwino.so: the same names as ``include/wino.h``, argument
marshalling only.  Device buffers are torch tensors (used for memory and streams,
nothing else); matrices are numpy/host arrays.  There is no fallback: if the
library has not been built, loading raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# WINO_LIB names another build of the same library (the sanitizer test loads one whose
# host code is instrumented); it is still this library, never a substitute path.
LIB_PATH = os.environ.get("WINO_LIB") or os.path.join(_HERE, "libwino.so")

WINO_F32, WINO_I8, WINO_I16, WINO_I8W16, WINO_BF16 = 0, 1, 2, 3, 4
WINO_TAP_U, WINO_TAP_V, WINO_TAP_M = 0, 1, 2
WINO_STAGE_INPUT, WINO_STAGE_GEMM, WINO_STAGE_OUTPUT, WINO_STAGE_ALL = 1, 2, 4, 7

EXPORTS = [
    "wino_status_string", "wino_weights_bytes", "wino_workspace_bytes",
    "wino_transform_weights", "wino_conv2d_fwd", "wino_conv2d_fwd_noalloc",
    "wino_conv2d_fwd_stages", "wino_fwd_num_kernels", "wino_fwd_sequence", "wino_conv2d_fwd_seq",
    "wino_debug_export", "wino_debug_mfma_loop", "wino_debug_load_loop", "wino_cook_toom",
    "conv2d_ref_packed_weights_bytes", "conv2d_ref_workspace_bytes",
    "conv2d_ref_pack_weights", "conv2d_ref_gpu", "conv2d_ref_gpu_rows",
]


class WinoDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("C", ctypes.c_int), ("K", ctypes.c_int),
                ("H", ctypes.c_int), ("W", ctypes.c_int), ("pad", ctypes.c_int),
                ("m", ctypes.c_int), ("dtype", ctypes.c_int),
                ("BT", ctypes.c_void_p), ("G", ctypes.c_void_p), ("AT", ctypes.c_void_p)]


class WinoQuant(ctypes.Structure):
    _fields_ = [("s_x", ctypes.c_float), ("s_v", ctypes.c_float), ("s_u", ctypes.c_float),
                ("s_y", ctypes.c_float), ("s_m", ctypes.c_float), ("qmax", ctypes.c_int),
                ("s_v_pos", ctypes.c_void_p), ("s_u_pos", ctypes.c_void_p),
                ("qmax_u", ctypes.c_int), ("qmax_v", ctypes.c_int), ("qmax_m", ctypes.c_int),
                ("qmax_y", ctypes.c_int)]


class WinoError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, status_string(status)))


_lib = None


def lib():
    """Loads libwino.so; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libwino.so is missing: build it with `python -m paper_2002_10711_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path")
        # PyTorch first: it brings its own copy of the HIP runtime, and the device pointers the
        # callers pass come from it -- loaded the other way round, the library would bind to a
        # second runtime and its first kernel launch fails (hipErrorInvalidDeviceFunction)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        L.wino_status_string.restype = ctypes.c_char_p
        for f in ("wino_weights_bytes", "wino_workspace_bytes",
                  "conv2d_ref_packed_weights_bytes", "conv2d_ref_workspace_bytes"):
            getattr(L, f).restype = ctypes.c_size_t
        L.wino_weights_bytes.argtypes = [ctypes.POINTER(WinoDesc)]
        L.wino_fwd_num_kernels.argtypes = [ctypes.POINTER(WinoDesc)]
        L.wino_workspace_bytes.argtypes = [ctypes.POINTER(WinoDesc)]
        L.wino_transform_weights.argtypes = [ctypes.POINTER(WinoDesc), ctypes.POINTER(WinoQuant),
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.wino_conv2d_fwd.argtypes = [ctypes.POINTER(WinoDesc), ctypes.POINTER(WinoQuant),
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        L.wino_conv2d_fwd_seq.argtypes = [ctypes.POINTER(WinoDesc), ctypes.POINTER(WinoQuant),
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                          ctypes.c_void_p]
        L.wino_fwd_sequence.argtypes = [ctypes.POINTER(WinoDesc), ctypes.c_int]
        L.wino_conv2d_fwd_noalloc.argtypes = [ctypes.POINTER(WinoDesc), ctypes.POINTER(WinoQuant),
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_void_p]
        L.wino_conv2d_fwd_stages.argtypes = [ctypes.POINTER(WinoDesc), ctypes.POINTER(WinoQuant),
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                             ctypes.c_void_p]
        L.wino_debug_export.argtypes = [ctypes.POINTER(WinoDesc), ctypes.c_int, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_void_p]
        L.wino_debug_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                           ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
        L.wino_debug_load_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                                           ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
        L.wino_cook_toom.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_void_p]
        L.conv2d_ref_packed_weights_bytes.argtypes = [ctypes.c_int] * 3
        L.conv2d_ref_workspace_bytes.argtypes = [ctypes.c_int] * 8
        L.conv2d_ref_pack_weights.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 3
        for f in (L.conv2d_ref_gpu, L.conv2d_ref_gpu_rows):
            f.argtypes = ([ctypes.c_int] * 8 + [ctypes.c_void_p] * 3 + [ctypes.c_float] * 3 +
                          [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p])
        _lib = L
    return _lib


def status_string(status):
    return lib().wino_status_string(int(status)).decode()


def _ptr(t):
    """Device (torch) or host (numpy) buffer -> integer address; None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status, where):
    if status != 0:
        raise WinoError(status, where)


class Desc:
    """Owns the host copies of the matrices a wino_desc points to."""

    def __init__(self, N, C, K, H, W, pad, m, dtype, BT=None, G=None, AT=None):
        self._keep = []
        self.c = WinoDesc(N, C, K, H, W, pad, m, dtype, None, None, None)
        for name, arr in (("BT", BT), ("G", G), ("AT", AT)):
            if arr is not None:
                a = np.ascontiguousarray(arr, dtype=np.float32)
                self._keep.append(a)
                setattr(self.c, name, a.ctypes.data)

    @property
    def ref(self):
        return ctypes.byref(self.c)


def make_quant(s_x, s_v, s_u, s_y, s_m=0.0, qmax=127, s_v_pos=None, s_u_pos=None,
               qmax_u=0, qmax_v=0, qmax_m=0, qmax_y=0):
    """wino_quant; with s_v_pos / s_u_pos (one scale per Winograd position, host arrays)
    s_v and s_u are ignored.  The arrays are kept alive by the returned object.
    qmax_*: code range of one stage (0 = qmax)."""
    q = WinoQuant(s_x, s_v, s_u, s_y, s_m, qmax, None, None, qmax_u, qmax_v, qmax_m, qmax_y)
    if s_v_pos is not None or s_u_pos is not None:
        q._sv = np.ascontiguousarray(s_v_pos, dtype=np.float32)
        q._su = np.ascontiguousarray(s_u_pos, dtype=np.float32)
        q.s_v_pos = q._sv.ctypes.data
        q.s_u_pos = q._su.ctypes.data
    return q


def wino_weights_bytes(desc):
    return int(lib().wino_weights_bytes(desc.ref))


def wino_workspace_bytes(desc):
    return int(lib().wino_workspace_bytes(desc.ref))


def wino_transform_weights(desc, quant, g_dev, U_dev, stream=None):
    q = ctypes.byref(quant) if quant is not None else None
    _check(lib().wino_transform_weights(desc.ref, q, _ptr(g_dev), _ptr(U_dev), _stream(stream)),
           "wino_transform_weights")


def wino_conv2d_fwd(desc, quant, x_dev, U_dev, y_dev, workspace_dev, workspace_bytes=None,
                    stream=None):
    q = ctypes.byref(quant) if quant is not None else None
    if workspace_bytes is None:
        workspace_bytes = workspace_dev.numel() * workspace_dev.element_size()
    _check(lib().wino_conv2d_fwd(desc.ref, q, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev),
                                 _ptr(workspace_dev), workspace_bytes, _stream(stream)),
           "wino_conv2d_fwd")


# kernel sequences of the int8 forward (wino.h)
(WINO_SEQ_AUTO, WINO_SEQ_FUSED, WINO_SEQ_COL, WINO_SEQ_COL2, WINO_SEQ_LDS, WINO_SEQ_REGS,
 WINO_SEQ_STAGED, WINO_SEQ_TROW) = range(8)
SEQ_NAMES = {WINO_SEQ_FUSED: "fused", WINO_SEQ_COL: "col", WINO_SEQ_COL2: "col2", WINO_SEQ_LDS: "lds",
             WINO_SEQ_REGS: "regs", WINO_SEQ_STAGED: "staged", WINO_SEQ_TROW: "trow"}


def wino_fwd_sequence(desc, seq=WINO_SEQ_AUTO):
    return int(lib().wino_fwd_sequence(desc.ref, seq))


def wino_conv2d_fwd_seq(desc, quant, x_dev, U_dev, y_dev, workspace_dev, seq, workspace_bytes=None,
                        stream=None):
    q = ctypes.byref(quant) if quant is not None else None
    if workspace_bytes is None:
        workspace_bytes = workspace_dev.numel() * workspace_dev.element_size()
    _check(lib().wino_conv2d_fwd_seq(desc.ref, q, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev),
                                     _ptr(workspace_dev), workspace_bytes, seq, _stream(stream)),
           "wino_conv2d_fwd_seq")


NOALLOC_SCRATCH_BYTES = 32 << 20


def wino_conv2d_fwd_noalloc(desc, quant, x_dev, U_dev, y_dev, stream=None):
    q = ctypes.byref(quant) if quant is not None else None
    _check(lib().wino_conv2d_fwd_noalloc(desc.ref, q, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev),
                                         _stream(stream)), "wino_conv2d_fwd_noalloc")


def wino_fwd_num_kernels(desc):
    return int(lib().wino_fwd_num_kernels(desc.ref))


def wino_conv2d_fwd_stages(desc, quant, x_dev, U_dev, y_dev, workspace_dev, stages,
                           workspace_bytes=None, stream=None):
    q = ctypes.byref(quant) if quant is not None else None
    if workspace_bytes is None:
        workspace_bytes = workspace_dev.numel() * workspace_dev.element_size()
    _check(lib().wino_conv2d_fwd_stages(desc.ref, q, _ptr(x_dev), _ptr(U_dev), _ptr(y_dev),
                                        _ptr(workspace_dev), workspace_bytes, stages,
                                        _stream(stream)), "wino_conv2d_fwd_stages")


def wino_debug_export(desc, which, src_dev, out_dev, stream=None):
    _check(lib().wino_debug_export(desc.ref, which, _ptr(src_dev), _ptr(out_dev), _stream(stream)),
           "wino_debug_export")


def wino_debug_mfma_loop(dtype, workgroups, iters, out_dev, stream=None):
    """Launches the matrix-core peak probe; returns the operations one launch performs."""
    ops = ctypes.c_double(0.0)
    _check(lib().wino_debug_mfma_loop(dtype, workgroups, iters, _ptr(out_dev), ctypes.byref(ops),
                                      _stream(stream)), "wino_debug_mfma_loop")
    return ops.value


def wino_debug_load_loop(mode, waves, workgroups, workgroup_bytes, iters, buf_dev, out_dev, stream=None):
    """Launches the vector-memory-path probe; returns the bytes one launch loads."""
    nbytes = ctypes.c_double(0.0)
    _check(lib().wino_debug_load_loop(mode, waves, workgroups, ctypes.c_size_t(workgroup_bytes), iters,
                                      _ptr(buf_dev), _ptr(out_dev), ctypes.byref(nbytes),
                                      _stream(stream)), "wino_debug_load_loop")
    return nbytes.value


def wino_cook_toom(m, points=None):
    """Host-only: returns (BT, G, AT) float32 arrays."""
    n = m + 2
    if m not in (2, 4, 6):
        _check(lib().wino_cook_toom(m, None, None, None, None), "wino_cook_toom")
    BT = np.zeros((n, n), np.float32)
    G = np.zeros((n, 3), np.float32)
    AT = np.zeros((m, n), np.float32)
    pts = None
    if points is not None:
        pts = np.ascontiguousarray(points, dtype=np.float64)
        assert pts.size == n - 1
    _check(lib().wino_cook_toom(m, _ptr(pts), BT.ctypes.data, G.ctypes.data, AT.ctypes.data),
           "wino_cook_toom")
    return BT, G, AT


def conv2d_ref_packed_weights_bytes(C, K, dtype):
    return int(lib().conv2d_ref_packed_weights_bytes(C, K, dtype))


def conv2d_ref_workspace_bytes(N, C, K, H, W, stride, pad, dtype):
    return int(lib().conv2d_ref_workspace_bytes(N, C, K, H, W, stride, pad, dtype))


def conv2d_ref_pack_weights(C, K, dtype, w_dev, wp_dev, stream=None):
    _check(lib().conv2d_ref_pack_weights(C, K, dtype, _ptr(w_dev), _ptr(wp_dev), _stream(stream)),
           "conv2d_ref_pack_weights")


def conv2d_ref_gpu(N, C, K, H, W, stride, pad, dtype, x_dev, wp_dev, y_dev, s_x, s_w, s_y, qmax,
                   workspace_dev, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace_dev.numel() * workspace_dev.element_size()
    _check(lib().conv2d_ref_gpu(N, C, K, H, W, stride, pad, dtype, _ptr(x_dev), _ptr(wp_dev),
                                _ptr(y_dev), s_x, s_w, s_y, qmax, _ptr(workspace_dev),
                                workspace_bytes, _stream(stream)), "conv2d_ref_gpu")


def conv2d_ref_gpu_rows(N, C, K, H, W, stride, pad, dtype, x_dev, wp_dev, y_dev, s_x, s_w, s_y, qmax,
                   workspace_dev, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace_dev.numel() * workspace_dev.element_size()
    _check(lib().conv2d_ref_gpu_rows(N, C, K, H, W, stride, pad, dtype, _ptr(x_dev), _ptr(wp_dev),
                                _ptr(y_dev), s_x, s_w, s_y, qmax, _ptr(workspace_dev),
                                workspace_bytes, _stream(stream)), "conv2d_ref_gpu_rows")
