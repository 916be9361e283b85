"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE, not product code).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
The functions here marshal numpy arrays into oracle/fq_oracle.c and hold none
of the method's arithmetic.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

CRIT_NONE, CRIT_ABSMAX_GT, CRIT_ALL, CRIT_L1_GT, CRIT_L1REL_GT = 0, 1, 2, 3, 4
OP_NT, OP_NN, OP_TN = 0, 1, 2


class _Operand(C.Structure):
    _fields_ = [("rows", C.c_int), ("cols", C.c_int),
                ("codes", C.c_void_p), ("scales", C.c_void_p), ("mask", C.c_void_p),
                ("res_codes", C.c_void_p), ("res_scales", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.fqo_quantize.restype = C.c_int
        _lib.fqo_quantize.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_long, C.c_int, C.c_int,
                                      C.c_float] + [C.c_void_p] * 7
        _lib.fqo_quantize_topk.restype = C.c_int
        _lib.fqo_quantize_topk.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_long, C.c_int,
                                           C.c_int] + [C.c_void_p] * 7
        _lib.fqo_gemm.restype = C.c_int
        _lib.fqo_gemm.argtypes = [C.c_int, C.POINTER(_Operand), C.POINTER(_Operand), C.c_int,
                                  C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _lib.fqo_gemm_partials.restype = C.c_int
        _lib.fqo_gemm_partials.argtypes = [C.c_int, C.POINTER(_Operand), C.POINTER(_Operand),
                                           C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.c_int, C.c_void_p]
        _lib.fqo_num_threads.restype = C.c_int
        _lib.fqo_philox4x32_10.restype = None
        _lib.fqo_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.fqo_quantize_sr.restype = C.c_int
        _lib.fqo_quantize_sr.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_long, C.c_int,
                                         C.c_uint64, C.c_void_p, C.c_void_p]
        _lib.fqo_ctx_quantize.restype = C.c_int
        _lib.fqo_ctx_quantize.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_long, C.c_void_p,
                                          C.c_void_p]
        _lib.fqo_ctx_dequantize.restype = C.c_int
        _lib.fqo_ctx_dequantize.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                            C.c_long]
        _lib.fqo_glu_forward.restype = C.c_int
        _lib.fqo_glu_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_long,
                                         C.c_void_p, C.c_long]
        _lib.fqo_glu_backward.restype = C.c_int
        _lib.fqo_glu_backward.argtypes = [C.c_void_p, C.c_long] + [C.c_void_p] * 4 + \
                                         [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_long]
        _lib.fqo_rmsnorm_forward.restype = C.c_int
        _lib.fqo_rmsnorm_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_long,
                                             C.c_double, C.c_void_p, C.c_long, C.c_void_p]
        _lib.fqo_rmsnorm_backward.restype = C.c_int
        _lib.fqo_rmsnorm_backward.argtypes = [C.c_void_p, C.c_long] + [C.c_void_p] * 4 + \
                                             [C.c_int, C.c_int, C.c_void_p, C.c_long, C.c_void_p]
        _lib.fqo_threshold_update.restype = C.c_float
        _lib.fqo_threshold_update.argtypes = [C.c_float, C.c_int, C.c_int, C.c_float, C.c_float,
                                              C.c_float]
    return _lib


def num_threads() -> int:
    return int(lib().fqo_num_threads())


class QTensor:
    """Outputs of the oracle quantizer for one matrix (all numpy, row-major)."""

    def __init__(self, rows, cols, g):
        self.rows, self.cols, self.g = rows, cols, g
        self.nbr, self.nbc = -(-rows // g), -(-cols // g)
        self.codes = np.zeros((rows, cols), np.int8)
        self.scales = np.zeros((self.nbr, self.nbc), np.float32)
        self.mask = np.zeros((self.nbr, self.nbc), np.uint8)
        self.res_codes = np.zeros((rows, cols), np.int8)
        self.res_scales = np.zeros((self.nbr, self.nbc), np.float32)
        self.fb_list = np.full((max(1, self.nbr * self.nbc),), -1, np.int32)
        self.fb_count = np.zeros((1,), np.int32)

    def operand(self, with_fallback=True):
        o = _Operand()
        o.rows, o.cols = self.rows, self.cols
        o.codes = self.codes.ctypes.data
        o.scales = self.scales.ctypes.data
        if with_fallback:
            o.mask = self.mask.ctypes.data
            o.res_codes = self.res_codes.ctypes.data
            o.res_scales = self.res_scales.ctypes.data
        else:
            o.mask = o.res_codes = o.res_scales = None
        return o


def quantize(x_bf16: np.ndarray, g: int, crit: int, theta: float) -> QTensor:
    """x_bf16: 2-D uint16 array of bf16 bit patterns (row stride may exceed cols)."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    assert x_bf16.strides[1] == 2 and x_bf16.strides[0] % 2 == 0
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2 if rows > 1 else max(cols, 1)
    q = QTensor(rows, cols, g)
    rc = lib().fqo_quantize(x_bf16.ctypes.data, rows, cols, ld, g, crit, C.c_float(theta),
                            q.codes.ctypes.data, q.scales.ctypes.data, q.mask.ctypes.data,
                            q.res_codes.ctypes.data, q.res_scales.ctypes.data,
                            q.fb_list.ctypes.data, q.fb_count.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_quantize failed: {rc}")
    return q


def quantize_topk(x_bf16: np.ndarray, g: int, k: int) -> QTensor:
    """TopK AbsMax selection (Sec. 4.4): the k blocks with the largest abs-max fall back."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2
    assert x_bf16.strides[1] == 2 and x_bf16.strides[0] % 2 == 0
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2 if rows > 1 else max(cols, 1)
    q = QTensor(rows, cols, g)
    rc = lib().fqo_quantize_topk(x_bf16.ctypes.data, rows, cols, ld, g, int(k),
                                 q.codes.ctypes.data, q.scales.ctypes.data, q.mask.ctypes.data,
                                 q.res_codes.ctypes.data, q.res_scales.ctypes.data,
                                 q.fb_list.ctypes.data, q.fb_count.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_quantize_topk failed: {rc}")
    return q


def out_shape(op, A: QTensor, B: QTensor):
    if op == OP_NT:
        return A.rows, B.rows
    if op == OP_NN:
        return A.rows, B.cols
    if op == OP_TN:
        return A.cols, B.cols
    raise ValueError(op)


def gemm(op, A: QTensor, B: QTensor, window=None, want_bf16=False, a_fallback=True):
    """Alg. 1 on the window (i0, i1, j0, j1) of the output (default: all of it).

    Returns the full-shape fp32 array (zeros outside the window) and, if asked,
    the bf16 bit patterns."""
    Mo, No = out_shape(op, A, B)
    i0, i1, j0, j1 = window if window is not None else (0, Mo, 0, No)
    c = np.zeros((Mo, No), np.float32)
    cb = np.zeros((Mo, No), np.uint16) if want_bf16 else None
    oa, ob = A.operand(a_fallback), B.operand(False)
    rc = lib().fqo_gemm(op, C.byref(oa), C.byref(ob), A.g, i0, i1, j0, j1, c.ctypes.data,
                        cb.ctypes.data if cb is not None else None)
    if rc != 0:
        raise RuntimeError(f"fqo_gemm failed: {rc}")
    return (c, cb) if want_bf16 else c


def gemm_window(op, A: QTensor, B: QTensor, window, want_bf16=False):
    """Alg. 1 on the window (i0, i1, j0, j1) of the output, returning only the window's rows
    (arrays of shape [i1 - i0, No] whose columns outside [j0, j1) are zero): the same call as
    gemm() without materializing the whole output."""
    Mo, No = out_shape(op, A, B)
    i0, i1, j0, j1 = window
    assert 0 <= i0 <= i1 <= Mo and 0 <= j0 <= j1 <= No
    c = np.zeros((i1 - i0, No), np.float32)
    cb = np.zeros((i1 - i0, No), np.uint16) if want_bf16 else None
    oa, ob = A.operand(True), B.operand(False)
    # the C routine addresses element (i, j) at base + i*No + j: hand it the base that puts
    # row i0 at the start of the window buffer
    rc = lib().fqo_gemm(op, C.byref(oa), C.byref(ob), A.g, i0, i1, j0, j1,
                        C.c_void_p(c.ctypes.data - i0 * No * 4),
                        C.c_void_p(cb.ctypes.data - i0 * No * 2) if cb is not None else None)
    if rc != 0:
        raise RuntimeError(f"fqo_gemm failed: {rc}")
    return (c, cb) if want_bf16 else c


def gemm_partials(op, A: QTensor, B: QTensor, kb: int, residual_term: bool, window=None):
    Mo, No = out_shape(op, A, B)
    i0, i1, j0, j1 = window if window is not None else (0, Mo, 0, No)
    p = np.zeros((Mo, No), np.int32)
    oa, ob = A.operand(True), B.operand(False)
    rc = lib().fqo_gemm_partials(op, C.byref(oa), C.byref(ob), A.g, kb, int(residual_term),
                                 i0, i1, j0, j1, p.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_gemm_partials failed: {rc}")
    return p


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, np.uint32)
    k = np.asarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().fqo_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def quantize_sr(x_bf16: np.ndarray, g: int, seed: int) -> QTensor:
    """Block INT8 with stochastic rounding (no fallback): Sec. 3.1 / 5.1."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2 and x_bf16.strides[1] == 2
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2 if rows > 1 else max(cols, 1)
    q = QTensor(rows, cols, g)
    rc = lib().fqo_quantize_sr(x_bf16.ctypes.data, rows, cols, ld, g, C.c_uint64(seed),
                               q.codes.ctypes.data, q.scales.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_quantize_sr failed: {rc}")
    return q


def threshold_update(theta, n_fallback, n_blocks, r_min=0.1, r_max=0.3, alpha=1.3) -> float:
    return float(lib().fqo_threshold_update(C.c_float(theta), int(n_fallback), int(n_blocks),
                                            C.c_float(r_min), C.c_float(r_max), C.c_float(alpha)))


def ctx_quantize(x_bf16: np.ndarray):
    """1 x 128 group INT10 context compression (Sec. 5.2): returns (packed uint8 [rows, ng, 160],
    scales float32 [rows, ng])."""
    assert x_bf16.dtype == np.uint16 and x_bf16.ndim == 2 and x_bf16.strides[1] == 2
    rows, cols = x_bf16.shape
    ld = x_bf16.strides[0] // 2 if rows > 1 else max(cols, 1)
    ng = -(-cols // 128)
    packed = np.zeros((rows, ng, 160), np.uint8)
    scales = np.zeros((rows, ng), np.float32)
    rc = lib().fqo_ctx_quantize(x_bf16.ctypes.data, rows, cols, ld, packed.ctypes.data,
                                scales.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_ctx_quantize failed: {rc}")
    return packed, scales


def ctx_dequantize(packed: np.ndarray, scales: np.ndarray, rows: int, cols: int) -> np.ndarray:
    out = np.zeros((rows, cols), np.uint16)
    rc = lib().fqo_ctx_dequantize(packed.ctypes.data, scales.ctypes.data, rows, cols,
                                  out.ctypes.data, max(cols, 1))
    if rc != 0:
        raise RuntimeError(f"fqo_ctx_dequantize failed: {rc}")
    return out


def glu_forward(x1_bf16: np.ndarray, x2_bf16: np.ndarray):
    """y = silu(x1) * x2 (Sec. 4.1) as a non-linear layer of Sec. 5.2: returns (y bf16 bits,
    context of x1, context of x2), each context a (packed, scales) pair of ctx_quantize."""
    assert x1_bf16.shape == x2_bf16.shape and x1_bf16.dtype == x2_bf16.dtype == np.uint16
    x1 = np.ascontiguousarray(x1_bf16)
    x2 = np.ascontiguousarray(x2_bf16)
    rows, cols = x1.shape
    y = np.zeros((rows, cols), np.uint16)
    rc = lib().fqo_glu_forward(x1.ctypes.data, x2.ctypes.data, rows, cols, max(cols, 1),
                               y.ctypes.data, max(cols, 1))
    if rc != 0:
        raise RuntimeError(f"fqo_glu_forward failed: {rc}")
    return y, ctx_quantize(x1), ctx_quantize(x2)


def glu_backward(dy_bf16: np.ndarray, ctx1, ctx2):
    """(dx1, dx2) bf16 bits from dy and the two INT10 contexts of glu_forward."""
    dy = np.ascontiguousarray(dy_bf16)
    rows, cols = dy.shape
    dx1 = np.zeros((rows, cols), np.uint16)
    dx2 = np.zeros((rows, cols), np.uint16)
    rc = lib().fqo_glu_backward(dy.ctypes.data, max(cols, 1), ctx1[0].ctypes.data,
                                ctx1[1].ctypes.data, ctx2[0].ctypes.data, ctx2[1].ctypes.data,
                                rows, cols, dx1.ctypes.data, dx2.ctypes.data, max(cols, 1))
    if rc != 0:
        raise RuntimeError(f"fqo_glu_backward failed: {rc}")
    return dx1, dx2


def rmsnorm_forward(x_bf16: np.ndarray, w_bf16: np.ndarray, eps: float):
    """y = x * rstd * w per row (non-linear layer of Sec. 5.2): returns (y bf16 bits, rstd float32
    [rows], INT10 context of x as a (packed, scales) pair)."""
    x = np.ascontiguousarray(x_bf16)
    w = np.ascontiguousarray(w_bf16)
    rows, cols = x.shape
    assert w.shape == (cols,) and x.dtype == w.dtype == np.uint16
    y = np.zeros((rows, cols), np.uint16)
    rstd = np.zeros(rows, np.float32)
    rc = lib().fqo_rmsnorm_forward(x.ctypes.data, w.ctypes.data, rows, cols, cols, float(eps),
                                   y.ctypes.data, cols, rstd.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_rmsnorm_forward failed: {rc}")
    return y, rstd, ctx_quantize(x)


def rmsnorm_backward(dy_bf16: np.ndarray, ctx, rstd: np.ndarray, w_bf16: np.ndarray):
    """(dx bf16 bits, dw float32 [cols]) from dy, the INT10 context of x, rstd and the gain."""
    dy = np.ascontiguousarray(dy_bf16)
    w = np.ascontiguousarray(w_bf16)
    rs = np.ascontiguousarray(rstd, dtype=np.float32)
    rows, cols = dy.shape
    dx = np.zeros((rows, cols), np.uint16)
    dw = np.zeros(cols, np.float32)
    rc = lib().fqo_rmsnorm_backward(dy.ctypes.data, cols, ctx[0].ctypes.data, ctx[1].ctypes.data,
                                    rs.ctypes.data, w.ctypes.data, rows, cols, dx.ctypes.data, cols,
                                    dw.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"fqo_rmsnorm_backward failed: {rc}")
    return dx, dw
