"""Python binding of libfq (Fallback Quantization on MI355X).

Thin ctypes layer over the C ABI declared in include/fq.h: same names, argument
marshalling only.  PyTorch supplies device memory and the current stream; every
step of the path runs in the library's HIP kernels.  If the compiled library is
missing, importing this package's functions raises -- there is no fallback.
"""
import ctypes as C
import os

FQ_BLOCK = 128
FQ_BLOCK_BYTES = 16384
FQ_CTX_GROUP = 128
FQ_CTX_GROUP_BYTES = 160

FQ_OK, FQ_ERR_NULL, FQ_ERR_SHAPE, FQ_ERR_BLOCK, FQ_ERR_ENUM, FQ_ERR_CAPACITY, FQ_ERR_HIP, \
    FQ_ERR_SCRATCH = 0, -1, -2, -3, -4, -5, -6, -7
FQ_STATIC_SCRATCH_FLOATS = 4 * 1024 * 1024
FQ_CRIT_NONE, FQ_CRIT_ABSMAX_GT, FQ_CRIT_ALL, FQ_CRIT_L1_GT, FQ_CRIT_L1REL_GT, FQ_CRIT_TOPK = \
    0, 1, 2, 3, 4, 5
FQ_OP_NT, FQ_OP_NN, FQ_OP_TN = 0, 1, 2
FQ_OUT_F32, FQ_OUT_BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
# FQ_LIBRARY: another build of the same library to load instead (the benchmark's ablation builds)
LIB_PATH = os.environ.get("FQ_LIBRARY") or os.path.join(_HERE, "libfq.so")

EXPORTS = ["fq_qtensor_bytes", "fq_qtensor_bind", "fq_quantize", "fq_quantize_sr", "fq_quantize_topk",
           "fq_threshold_update", "fq_gemm", "fq_gemm_plain", "fq_gemm_biased",
           "fq_gemm_debug_partials", "fq_codes_to_rowmajor", "fq_qtensor_check",
           "fq_status_string", "fq_ctx_packed_bytes", "fq_ctx_scales_bytes", "fq_ctx_quantize",
           "fq_ctx_dequantize", "fq_gemm_tile_plan", "fq_glu_forward", "fq_glu_backward", "fq_rmsnorm_forward",
           "fq_rmsnorm_backward", "fq_rmsnorm_backward_static"]


class fq_qtensor(C.Structure):
    """Mirror of the C struct fq_qtensor."""
    _fields_ = [("rows", C.c_int32), ("cols", C.c_int32), ("block", C.c_int32),
                ("capacity", C.c_int32), ("criterion", C.c_int32), ("epoch", C.c_int32),
                ("codes", C.c_void_p), ("codes_t", C.c_void_p), ("scales", C.c_void_p),
                ("mask", C.c_void_p), ("fb_count", C.c_void_p), ("fb_counters", C.c_void_p),
                ("fb_list", C.c_void_p),
                ("fb_slot", C.c_void_p), ("res_codes", C.c_void_p), ("res_codes_t", C.c_void_p),
                ("res_scales", C.c_void_p)]


class FqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2503_08040_amd.build` (needs hipcc)")
        L = C.CDLL(LIB_PATH)
        L.fq_qtensor_bytes.restype = C.c_size_t
        L.fq_qtensor_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int]
        L.fq_qtensor_bind.restype = C.c_int
        L.fq_qtensor_bind.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int, C.POINTER(fq_qtensor)]
        L.fq_quantize.restype = C.c_int
        L.fq_quantize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_int,
                                  C.c_float, C.POINTER(fq_qtensor), C.c_void_p]
        L.fq_quantize_sr.restype = C.c_int
        L.fq_quantize_sr.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int32,
                                     C.c_uint64, C.POINTER(fq_qtensor), C.c_void_p]
        L.fq_quantize_topk.restype = C.c_int
        L.fq_quantize_topk.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int32,
                                       C.c_int32, C.POINTER(fq_qtensor), C.c_void_p]
        L.fq_threshold_update.restype = C.c_float
        L.fq_threshold_update.argtypes = [C.c_float, C.c_int32, C.c_int32, C.c_float, C.c_float,
                                          C.c_float]
        L.fq_gemm.restype = C.c_int
        L.fq_gemm.argtypes = [C.c_int, C.POINTER(fq_qtensor), C.POINTER(fq_qtensor), C.c_void_p,
                              C.c_int, C.c_int64, C.c_void_p]
        L.fq_gemm_plain.restype = C.c_int
        L.fq_gemm_plain.argtypes = L.fq_gemm.argtypes
        L.fq_gemm_biased.restype = C.c_int
        L.fq_gemm_biased.argtypes = L.fq_gemm.argtypes
        L.fq_gemm_debug_partials.restype = C.c_int
        L.fq_gemm_debug_partials.argtypes = [C.c_int, C.POINTER(fq_qtensor), C.POINTER(fq_qtensor),
                                             C.c_int32, C.c_int, C.c_void_p, C.c_void_p]
        L.fq_codes_to_rowmajor.restype = C.c_int
        L.fq_codes_to_rowmajor.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.fq_qtensor_check.restype = C.c_int
        L.fq_qtensor_check.argtypes = [C.POINTER(fq_qtensor), C.POINTER(C.c_int32), C.c_void_p]
        L.fq_status_string.restype = C.c_char_p
        L.fq_status_string.argtypes = [C.c_int]
        for f in (L.fq_ctx_packed_bytes, L.fq_ctx_scales_bytes):
            f.restype = C.c_size_t
            f.argtypes = [C.c_int32, C.c_int32]
        L.fq_ctx_quantize.restype = C.c_int
        L.fq_ctx_quantize.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        L.fq_ctx_dequantize.restype = C.c_int
        L.fq_ctx_dequantize.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                        C.c_int64, C.c_void_p]
        L.fq_glu_forward.restype = C.c_int
        L.fq_glu_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                                     C.c_void_p, C.c_int64] + [C.c_void_p] * 5
        L.fq_glu_backward.restype = C.c_int
        L.fq_glu_backward.argtypes = [C.c_void_p, C.c_int64] + [C.c_void_p] * 4 + \
                                     [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64,
                                      C.c_void_p]
        L.fq_rmsnorm_forward.restype = C.c_int
        L.fq_rmsnorm_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                                         C.c_float, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
        L.fq_rmsnorm_backward.restype = C.c_int
        L.fq_rmsnorm_backward.argtypes = [C.c_void_p, C.c_int64] + [C.c_void_p] * 4 + \
                                         [C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                                          C.c_void_p, C.c_int32, C.c_void_p]
        L.fq_rmsnorm_backward_static.restype = C.c_int
        L.fq_rmsnorm_backward_static.argtypes = [C.c_void_p, C.c_int64] + [C.c_void_p] * 4 + \
                                                [C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_int32, C.c_void_p]
        L.fq_gemm_tile_plan.restype = C.c_int
        L.fq_gemm_tile_plan.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fq_status_string(int(status)).decode()


def _check(status, where):
    if status != FQ_OK:
        raise FqError(status, where)


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def fq_qtensor_bytes(rows, cols, capacity, want_transposed=False, block=FQ_BLOCK) -> int:
    return int(lib().fq_qtensor_bytes(rows, cols, block, capacity, int(want_transposed)))


class QTensor:
    """Device buffers of one quantized matrix: a torch byte tensor carved up by
    fq_qtensor_bind, plus typed views of its pieces for inspection."""

    def __init__(self, rows, cols, capacity=None, want_transposed=False, device="cuda",
                 block=FQ_BLOCK):
        import torch
        self.rows, self.cols, self.block = int(rows), int(cols), int(block)
        # grids of per-block values (scales, mask, slots); codes are always stored in 128-tiles
        self.nbr, self.nbc = -(-self.rows // self.block), -(-self.cols // self.block)
        self.n_tiles = (-(-self.rows // FQ_BLOCK)) * (-(-self.cols // FQ_BLOCK))
        if capacity is None:
            capacity = self.nbr * self.nbc if self.block == FQ_BLOCK else 0
        self.capacity = int(capacity)
        self.want_transposed = bool(want_transposed)
        nbytes = fq_qtensor_bytes(self.rows, self.cols, self.capacity, self.want_transposed,
                                  self.block)
        if nbytes == 0:
            raise FqError(FQ_ERR_SHAPE, "fq_qtensor_bytes")
        self.storage = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        self._base = (self.storage.data_ptr() + 255) & ~255
        self.c = fq_qtensor()
        _check(lib().fq_qtensor_bind(C.c_void_p(self._base), self.rows, self.cols, self.block,
                                     self.capacity, int(self.want_transposed), C.byref(self.c)),
               "fq_qtensor_bind")

    def _view(self, ptr, nbytes, dtype, shape):
        import torch
        off = ptr - self.storage.data_ptr()
        return self.storage[off:off + nbytes].view(dtype).view(shape)

    def view(self, field):
        """Typed torch view of one buffer (device memory, no copy)."""
        import torch
        spec = {
            "codes": (torch.int8, (self.n_tiles, FQ_BLOCK_BYTES), 1),
            "codes_t": (torch.int8, (self.n_tiles, FQ_BLOCK_BYTES), 1),
            "scales": (torch.float32, (self.nbr, self.nbc), 4),
            "mask": (torch.uint8, (self.nbr, self.nbc), 1),
            "fb_count": (torch.int32, (1,), 4),
            "fb_list": (torch.int32, (self.capacity,), 4),
            "fb_slot": (torch.int32, (self.nbr, self.nbc), 4),
            "res_codes": (torch.int8, (self.capacity, FQ_BLOCK_BYTES), 1),
            "res_codes_t": (torch.int8, (self.capacity, FQ_BLOCK_BYTES), 1),
            "res_scales": (torch.float32, (self.capacity,), 4),
        }[field]
        ptr = getattr(self.c, field)
        if not ptr:
            return None
        n = 1
        for d in spec[1]:
            n *= d
        return self._view(ptr, n * spec[2], spec[0], spec[1])


def fq_quantize(x, crit, theta, out: QTensor = None, capacity=None, want_transposed=False,
                stream=None, block=FQ_BLOCK) -> QTensor:
    """x: 2-D torch.bfloat16 CUDA tensor with unit column stride."""
    import torch
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda
    assert x.stride(1) == 1 or x.shape[1] <= 1
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else max(cols, 1)
    if out is None:
        out = QTensor(rows, cols, capacity, want_transposed, x.device, block=block)
    _check(lib().fq_quantize(C.c_void_p(x.data_ptr()), rows, cols, ld, out.block, int(crit),
                             C.c_float(theta), C.byref(out.c), _stream_ptr(stream)), "fq_quantize")
    return out


def fq_quantize_sr(x, seed, out: QTensor = None, want_transposed=False, stream=None) -> QTensor:
    """Block INT8 with stochastic rounding (no fallback); x as for fq_quantize."""
    import torch
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda
    assert x.stride(1) == 1 or x.shape[1] <= 1
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else max(cols, 1)
    if out is None:
        out = QTensor(rows, cols, 0, want_transposed, x.device)
    _check(lib().fq_quantize_sr(C.c_void_p(x.data_ptr()), rows, cols, ld, FQ_BLOCK,
                                C.c_uint64(seed), C.byref(out.c), _stream_ptr(stream)),
           "fq_quantize_sr")
    return out


def fq_quantize_topk(x, k, out: QTensor = None, capacity=None, want_transposed=False,
                     stream=None) -> QTensor:
    """As fq_quantize, with the k blocks of largest abs-max falling back (Sec. 4.4)."""
    import torch
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda
    assert x.stride(1) == 1 or x.shape[1] <= 1
    rows, cols = x.shape
    ld = x.stride(0) if rows > 1 else max(cols, 1)
    if out is None:
        out = QTensor(rows, cols, capacity, want_transposed, x.device)
    _check(lib().fq_quantize_topk(C.c_void_p(x.data_ptr()), rows, cols, ld, FQ_BLOCK, int(k),
                                  C.byref(out.c), _stream_ptr(stream)), "fq_quantize_topk")
    return out


def fq_threshold_update(theta, n_fallback, n_blocks, r_min=0.1, r_max=0.3, alpha=1.3) -> float:
    """Alg. 2 of the paper: next step's threshold from this step's fallback count (host only)."""
    return float(lib().fq_threshold_update(C.c_float(theta), int(n_fallback), int(n_blocks),
                                           C.c_float(r_min), C.c_float(r_max), C.c_float(alpha)))


def gemm_out_shape(op, A: QTensor, B: QTensor):
    if op == FQ_OP_NT:
        return A.rows, B.rows
    if op == FQ_OP_NN:
        return A.rows, B.cols
    if op == FQ_OP_TN:
        return A.cols, B.cols
    raise FqError(FQ_ERR_ENUM, "fq_gemm")


def fq_gemm_plain(op, A: QTensor, B: QTensor, out=None, out_dtype=None, stream=None):
    """Eq. (1) on the plain kernel (any block size, no fallback); see fq.h."""
    return fq_gemm(op, A, B, out, out_dtype, stream, _entry="fq_gemm_plain")


def fq_gemm_biased(op, A: QTensor, B: QTensor, out=None, out_dtype=None, stream=None):
    """fq_gemm within a tolerance (about 2e-4 of max |C|) with half the dequantization work; see fq.h."""
    return fq_gemm(op, A, B, out, out_dtype, stream, _entry="fq_gemm_biased")


def fq_gemm(op, A: QTensor, B: QTensor, out=None, out_dtype=None, stream=None, _entry="fq_gemm"):
    """C = A (op) B per Alg. 1; out is a 2-D float32 or bfloat16 CUDA tensor."""
    import torch
    Mo, No = gemm_out_shape(op, A, B)
    if out is None:
        out = torch.empty((Mo, No), dtype=out_dtype or torch.float32, device=A.storage.device)
    assert out.shape == (Mo, No) and (out.stride(1) == 1 or No <= 1)
    cdt = {torch.float32: FQ_OUT_F32, torch.bfloat16: FQ_OUT_BF16}[out.dtype]
    ldc = out.stride(0) if Mo > 1 else max(No, 1)
    _check(getattr(lib(), _entry)(int(op), C.byref(A.c), C.byref(B.c), C.c_void_p(out.data_ptr()),
                                  cdt, ldc, _stream_ptr(stream)), _entry)
    return out


def fq_gemm_debug_partials(op, A: QTensor, B: QTensor, k_block, residual_term, stream=None):
    import torch
    Mo, No = gemm_out_shape(op, A, B)
    out = torch.zeros((Mo, No), dtype=torch.int32, device=A.storage.device)
    _check(lib().fq_gemm_debug_partials(int(op), C.byref(A.c), C.byref(B.c), int(k_block),
                                        int(bool(residual_term)), C.c_void_p(out.data_ptr()),
                                        _stream_ptr(stream)), "fq_gemm_debug_partials")
    return out


def fq_codes_to_rowmajor(tiled, rows, cols, stream=None):
    """tiled: int8 CUDA tensor in tile order (a QTensor 'codes' view)."""
    import torch
    dense = torch.empty((rows, cols), dtype=torch.int8, device=tiled.device)
    _check(lib().fq_codes_to_rowmajor(C.c_void_p(tiled.data_ptr()), rows, cols,
                                      C.c_void_p(dense.data_ptr()), _stream_ptr(stream)),
           "fq_codes_to_rowmajor")
    return dense


def fq_qtensor_check(t: QTensor, stream=None) -> int:
    """Synchronizes; returns the number of flagged blocks, raises on capacity overflow."""
    n = C.c_int32(0)
    _check(lib().fq_qtensor_check(C.byref(t.c), C.byref(n), _stream_ptr(stream)), "fq_qtensor_check")
    return int(n.value)


def fq_ctx_packed_bytes(rows, cols) -> int:
    return int(lib().fq_ctx_packed_bytes(rows, cols))


def fq_ctx_scales_bytes(rows, cols) -> int:
    return int(lib().fq_ctx_scales_bytes(rows, cols))


def fq_ctx_quantize(x, packed=None, scales=None, stream=None):
    """1 x 128 group INT10 compression of a 2-D bf16 CUDA tensor (Sec. 5.2 of the paper).
    Returns (packed uint8 [rows, ng, 160], scales float32 [rows, ng])."""
    import torch
    assert x.dtype == torch.bfloat16 and x.dim() == 2 and x.is_cuda
    assert x.stride(1) == 1 or x.shape[1] <= 1
    rows, cols = x.shape
    ng = -(-cols // FQ_CTX_GROUP)
    ld = x.stride(0) if rows > 1 else max(cols, 1)
    if packed is None:
        packed = torch.empty((rows, ng, FQ_CTX_GROUP_BYTES), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, ng), dtype=torch.float32, device=x.device)
    assert packed.is_contiguous() and packed.numel() == fq_ctx_packed_bytes(rows, cols)
    assert scales.is_contiguous() and scales.numel() * 4 == fq_ctx_scales_bytes(rows, cols)
    _check(lib().fq_ctx_quantize(C.c_void_p(x.data_ptr()), rows, cols, ld,
                                 C.c_void_p(packed.data_ptr()), C.c_void_p(scales.data_ptr()),
                                 _stream_ptr(stream)), "fq_ctx_quantize")
    return packed, scales


def fq_ctx_dequantize(packed, scales, rows, cols, out=None, stream=None):
    """Inverse of fq_ctx_quantize: a bf16 [rows, cols] CUDA tensor."""
    import torch
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.bfloat16, device=packed.device)
    assert out.dtype == torch.bfloat16 and out.shape == (rows, cols)
    assert out.stride(1) == 1 or cols <= 1
    assert packed.is_contiguous() and packed.numel() == fq_ctx_packed_bytes(rows, cols)
    assert scales.is_contiguous() and scales.numel() * 4 == fq_ctx_scales_bytes(rows, cols)
    ldo = out.stride(0) if rows > 1 else max(cols, 1)
    _check(lib().fq_ctx_dequantize(C.c_void_p(packed.data_ptr()), C.c_void_p(scales.data_ptr()),
                                   rows, cols, C.c_void_p(out.data_ptr()), ldo,
                                   _stream_ptr(stream)), "fq_ctx_dequantize")
    return out


def fq_gemm_tile_plan(rows_out, cols_out, compute_units=0):
    """(workgroups with 256x256 tiles, tile columns they cover, columns of 128x384 tiles)."""
    out = (C.c_int32 * 3)()
    _check(lib().fq_gemm_tile_plan(int(rows_out), int(cols_out), int(compute_units), out),
           "fq_gemm_tile_plan")
    return int(out[0]), int(out[1]), int(out[2])


def _pitch(t):
    rows, cols = t.shape
    assert t.stride(1) == 1 or cols <= 1
    return t.stride(0) if rows > 1 else max(cols, 1)


def fq_glu_forward(x1, x2, stream=None):
    """y = silu(x1) * x2 with the INT10 contexts of x1 and x2 written in the same pass.
    Returns (y bf16, (packed1, scales1), (packed2, scales2))."""
    import torch
    assert x1.dtype == x2.dtype == torch.bfloat16 and x1.shape == x2.shape and x1.dim() == 2
    assert _pitch(x1) == _pitch(x2)
    rows, cols = x1.shape
    ng = -(-cols // FQ_CTX_GROUP)
    y = torch.empty((rows, cols), dtype=torch.bfloat16, device=x1.device)
    ctx = [(torch.empty((rows, ng, FQ_CTX_GROUP_BYTES), dtype=torch.uint8, device=x1.device),
            torch.empty((rows, ng), dtype=torch.float32, device=x1.device)) for _ in range(2)]
    _check(lib().fq_glu_forward(C.c_void_p(x1.data_ptr()), C.c_void_p(x2.data_ptr()), rows, cols,
                                _pitch(x1), C.c_void_p(y.data_ptr()), _pitch(y),
                                C.c_void_p(ctx[0][0].data_ptr()), C.c_void_p(ctx[0][1].data_ptr()),
                                C.c_void_p(ctx[1][0].data_ptr()), C.c_void_p(ctx[1][1].data_ptr()),
                                _stream_ptr(stream)), "fq_glu_forward")
    return y, ctx[0], ctx[1]


def fq_glu_backward(dy, ctx1, ctx2, stream=None):
    """(dx1, dx2) bf16 from dy and the two contexts of fq_glu_forward."""
    import torch
    assert dy.dtype == torch.bfloat16 and dy.dim() == 2
    rows, cols = dy.shape
    dx1 = torch.empty((rows, cols), dtype=torch.bfloat16, device=dy.device)
    dx2 = torch.empty_like(dx1)
    _check(lib().fq_glu_backward(C.c_void_p(dy.data_ptr()), _pitch(dy),
                                 C.c_void_p(ctx1[0].data_ptr()), C.c_void_p(ctx1[1].data_ptr()),
                                 C.c_void_p(ctx2[0].data_ptr()), C.c_void_p(ctx2[1].data_ptr()),
                                 rows, cols, C.c_void_p(dx1.data_ptr()), C.c_void_p(dx2.data_ptr()),
                                 _pitch(dx1), _stream_ptr(stream)), "fq_glu_backward")
    return dx1, dx2


def fq_rmsnorm_forward(x, w, eps, stream=None):
    """y = x * rstd * w per row with the INT10 context of x and rstd written in the same pass.
    Returns (y bf16, rstd float32 [rows], (packed, scales))."""
    import torch
    assert x.dtype == w.dtype == torch.bfloat16 and x.dim() == 2 and w.shape == (x.shape[1],)
    assert w.is_contiguous()
    rows, cols = x.shape
    ng = -(-cols // FQ_CTX_GROUP)
    y = torch.empty((rows, cols), dtype=torch.bfloat16, device=x.device)
    rstd = torch.empty((rows,), dtype=torch.float32, device=x.device)
    packed = torch.empty((rows, ng, FQ_CTX_GROUP_BYTES), dtype=torch.uint8, device=x.device)
    scales = torch.empty((rows, ng), dtype=torch.float32, device=x.device)
    _check(lib().fq_rmsnorm_forward(C.c_void_p(x.data_ptr()), C.c_void_p(w.data_ptr()), rows, cols,
                                    _pitch(x), C.c_float(eps), C.c_void_p(y.data_ptr()), _pitch(y),
                                    C.c_void_p(packed.data_ptr()), C.c_void_p(scales.data_ptr()),
                                    C.c_void_p(rstd.data_ptr()), _stream_ptr(stream)),
           "fq_rmsnorm_forward")
    return y, rstd, (packed, scales)


def fq_rmsnorm_backward_static(dy, ctx, rstd, w, dx, dw, n_parts=64, stream=None):
    """fq_rmsnorm_backward into caller-provided dx (bf16 [rows, cols]) and dw (float32 [cols])
    with the library's built-in scratch buffer: the call allocates nothing."""
    rows, cols = dy.shape
    _check(lib().fq_rmsnorm_backward_static(C.c_void_p(dy.data_ptr()), _pitch(dy),
                                            C.c_void_p(ctx[0].data_ptr()), C.c_void_p(ctx[1].data_ptr()),
                                            C.c_void_p(rstd.data_ptr()), C.c_void_p(w.data_ptr()),
                                            rows, cols, C.c_void_p(dx.data_ptr()), _pitch(dx),
                                            C.c_void_p(dw.data_ptr()), int(n_parts), _stream_ptr(stream)),
           "fq_rmsnorm_backward_static")
    return dx, dw


def fq_rmsnorm_backward(dy, ctx, rstd, w, n_parts=256, stream=None):
    """(dx bf16, dw float32 [cols]) from dy, the context and rstd of fq_rmsnorm_forward, and w."""
    import torch
    assert dy.dtype == w.dtype == torch.bfloat16 and dy.dim() == 2 and w.is_contiguous()
    rows, cols = dy.shape
    dx = torch.empty((rows, cols), dtype=torch.bfloat16, device=dy.device)
    dw = torch.empty((cols,), dtype=torch.float32, device=dy.device)
    parts = torch.empty((n_parts * cols + rows,), dtype=torch.float32, device=dy.device)
    _check(lib().fq_rmsnorm_backward(C.c_void_p(dy.data_ptr()), _pitch(dy),
                                     C.c_void_p(ctx[0].data_ptr()), C.c_void_p(ctx[1].data_ptr()),
                                     C.c_void_p(rstd.data_ptr()), C.c_void_p(w.data_ptr()), rows, cols,
                                     C.c_void_p(dx.data_ptr()), _pitch(dx), C.c_void_p(dw.data_ptr()),
                                     C.c_void_p(parts.data_ptr()), int(n_parts), _stream_ptr(stream)),
           "fq_rmsnorm_backward")
    return dx, dw
