/*
 * fq.h -- C ABI of libfq: Fallback Quantization for AMD MI355X (gfx950).
 *
 * The library implements the linear-layer hot path of "Accurate INT8 Training
 * Through Dynamic Block-Level Fallback" (arXiv 2503.08040):
 *
 *   fq_quantize  block INT8 quantization of a bf16 matrix with per-block scale
 *                (Sec. 3.1), run-time outlier detection u = [max|G| > theta]
 *                (Sec. 4.4) and, for flagged blocks, the second quantization
 *                step on the residual (Sec. 4.3);
 *   fq_gemm      the fallback block GEMM (Sec. 4.2 Eq. (1), Sec. 4.3 Alg. 1) for
 *                the three products of a linear layer (Sec. 3.2):
 *                Y = X W^T, dX = dY W, dW = dY^T X.
 *
 * General rules
 *   - Every data pointer is caller-owned DEVICE memory (hipMalloc'ed or a
 *     PyTorch CUDA/HIP tensor's storage) unless a comment says "host".  The
 *     library never allocates, frees or retains device memory: all that is
 *     carried from one call to the next lives in the caller's fq_qtensor (its
 *     `epoch` field and `fb_counters` buffer).
 *     fq_qtensor structs themselves live in host memory.
 *   - Calls enqueue kernels on `hip_stream` (a hipStream_t passed as void*;
 *     NULL is the default stream) and return without waiting.
 *   - Arguments are validated on the host before anything is launched; a
 *     failed validation returns a negative fq_status and launches nothing.
 *     HIP launch failures are returned as FQ_ERR_HIP.  No exception crosses
 *     this boundary.
 *   - Threads and streams: calls on different tensors and buffers may run concurrently from
 *     any threads and on any streams.  Calls that write the same fq_qtensor (its struct is
 *     updated on the host and its buffers on the device) or the same output buffer must be
 *     ordered by the caller, and a tensor must not be consumed (fq_gemm, fq_qtensor_check) on a
 *     stream that is not ordered after the quantize call that filled it.  The only state the
 *     library keeps by itself is a per-device cache of the compute-unit count and of a kernel
 *     attribute, both written once and safe to race on.
 *   - The quantization block is 128 x 128 (FQ_BLOCK), the size the paper settles on
 *     (Sec. 4.5).  Blocks of 64 x 64 and 32 x 32 are accepted for plain block INT8
 *     (FQ_CRIT_NONE, round to nearest; no fallback, no transposed residuals), which is what
 *     the group-size curve of Fig. 1b needs; any other use of them, and any other size,
 *     returns FQ_ERR_BLOCK.  Matrix dimensions need not be multiples of the block: an edge
 *     block consists of the elements that exist, the rest counts as zero.
 *     Whatever the block size, codes are stored in 128 x 128 tiles (below); the scale, mask
 *     and slot grids have one entry per block, nbr = ceil(rows/block) by nbc = ceil(cols/block).
 *
 * Storage order of INT8 codes ("tile order")
 *   Codes are not stored row-major.  A rows x cols matrix is cut into
 *   nbr x nbc blocks (nbr = ceil(rows/128), nbc = ceil(cols/128)); block
 *   (bi, bk) occupies the 16384 bytes starting at (bi*nbc + bk)*16384, and
 *   element (r, c) of the block (0 <= r, c < 128) is the byte at
 *       ((r/32)*4 + c/32)*1024 + ((r%32) + 32*((c%32)/16))*16 + c%16 .
 *   Every 16-byte run holds 16 contraction-contiguous codes of one row, and rows follow each
 *   other at 16-byte steps inside a 1 KiB run of 32 rows x 32 contraction positions: the
 *   operands of the gfx950 INT8 matrix instructions (16 contraction-contiguous bytes per lane,
 *   consecutive lanes = consecutive rows) are whole 256- or 512-byte runs of this order, so the
 *   GEMM moves blocks with
 *   perfectly coalesced 16-byte accesses and no shuffling.  Padding elements
 *   of edge blocks are stored as 0.  `codes_t` holds the transposed matrix
 *   (cols x rows) in the same order; it is what the backward products read
 *   when the contraction runs along the rows of the stored matrix.
 *   fq_codes_to_rowmajor converts back to a plain row-major array.
 */
#ifndef FQ_H_
#define FQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FQ_BLOCK 128
#define FQ_BLOCK_BYTES 16384

typedef enum {
  FQ_OK = 0,
  FQ_ERR_NULL = -1,     /* a required pointer is NULL                          */
  FQ_ERR_SHAPE = -2,    /* negative / inconsistent dimensions or strides       */
  FQ_ERR_BLOCK = -3,    /* unsupported block size, or a block of 64 / 32 with fallback */
  FQ_ERR_ENUM = -4,     /* unknown enum value, or B operand quantized with fallback */
  FQ_ERR_CAPACITY = -5, /* more flagged blocks than `capacity` (fq_qtensor_check) */
  FQ_ERR_HIP = -6,      /* a HIP call failed                                   */
  FQ_ERR_SCRATCH = -7   /* fq_rmsnorm_backward_static: the call needs more scratch
                           memory than the library's built-in buffer holds         */
} fq_status;

/* Fallback criterion.  NONE: u = 0 everywhere (plain block INT8, Eq. (1)).
 * ABSMAX_GT: u(i,k) = [max|G_ik| > theta], strict; the selector the paper adopts (Sec. 4.4).
 * ALL: u = 1.
 * L1_GT, L1REL_GT: the two error-based selectors Sec. 4.4 compares it with,
 *   u = [L1 > theta] with L1 = sum |G_ik - Q(G_ik)| over the block, and
 *   u = [L1 / sum |G_ik| > theta] (an all-zero block is never flagged).
 *   G - Q(G) is the same binary32 residual the second quantization step uses; the two sums
 *   are binary64 accumulations of the binary32 terms in unspecified order and the comparison
 *   is binary64, so a block whose metric is within about 2^-40 (relative) of theta may be
 *   decided either way.  These two cost one extra pass over the block in registers.
 *   FQ_CRIT_TOPK       the k blocks with the largest max|G| (Sec. 4.4): not accepted by
 *                      fq_quantize, which has no k; it is what fq_quantize_topk records in
 *                      the tensor.  It needs a tensor-wide selection, which is why the paper
 *                      replaces it by the delayed threshold of App. D (fq_threshold_update). */
typedef enum {
  FQ_CRIT_NONE = 0, FQ_CRIT_ABSMAX_GT = 1, FQ_CRIT_ALL = 2, FQ_CRIT_L1_GT = 3, FQ_CRIT_L1REL_GT = 4,
  FQ_CRIT_TOPK = 5
} fq_criterion;

/* Which product of the linear layer (Sec. 3.2).  A is the operand that may
 * carry fallback blocks (Alg. 1 defines fallback for A only).
 *   NT: C[M,N] = A[M,K] * B[N,K]^T     Y  = X  W^T
 *   NN: C[M,K] = A[M,N] * B[N,K]       dX = dY W      (needs B->codes_t)
 *   TN: C[N,K] = A[M,N]^T * B[M,K]     dW = dY^T X    (needs A->codes_t,
 *                                       A->res_codes_t if A has fallback, B->codes_t) */
typedef enum { FQ_OP_NT = 0, FQ_OP_NN = 1, FQ_OP_TN = 2 } fq_op;

typedef enum { FQ_OUT_F32 = 0, FQ_OUT_BF16 = 1 } fq_out_dtype;

/*
 * A quantized matrix.  The struct is host memory; every pointer in it is
 * device memory owned by the caller.  fq_qtensor_bind fills the pointers from
 * one allocation of fq_qtensor_bytes bytes; a caller may also set them itself.
 */
typedef struct {
  int32_t rows, cols;    /* shape of the source matrix                           */
  int32_t block;         /* 128 (or 64 / 32: plain block INT8, capacity 0)      */
  int32_t capacity;      /* number of residual slots the res_* buffers hold      */
  int32_t criterion;     /* host: fq_criterion of the last fq_quantize into this */
  int32_t epoch;         /* host: fq_quantize calls made into this tensor (library-managed;
                            fq_qtensor_bind sets 0; selects the live counter; -1 once a
                            call into the tensor has been recorded under stream capture) */
  int8_t *codes;         /* [nbr*nbc][16384] tile order, Q^(G)        (Sec. 3.1) */
  int8_t *codes_t;       /* [nbc*nbr][16384] tile order of G^T, or NULL          */
  float *scales;         /* [nbr, nbc]  a_{i,k} = max|G_ik| / 127     (Sec. 3.1) */
  uint8_t *mask;         /* [nbr, nbc]  u(i,k)                        (Sec. 4.4) */
  int32_t *fb_count;     /* [1]  number of flagged blocks (may exceed capacity).
                            Points at one of the two fb_counters; fq_quantize
                            re-points it on every call                           */
  int32_t *fb_counters;  /* [4 + 2*ceil(nbr*nbc/32)], 8-byte aligned, library-managed:
                            two alternating slot counters (a call counts in one and
                            clears the other for the next call, so the quantizer is a
                            single kernel launch), a counter of completed groups of 32
                            blocks, one unused word, and one 64-bit word of decision
                            bits per group (from which fb_list is written)            */
  int32_t *fb_list;      /* [capacity] ascending list of the flagged blocks' ids bi*nbc+bk
                            (the first min(fb_count, capacity) entries are valid; when more
                            blocks are flagged than `capacity`, the lowest `capacity` ids);
                            deterministic: it does not depend on the slot assignment  */
  int32_t *fb_slot;      /* [nbr, nbc] residual slot of the block, -1 if not
                            flagged, -2 if flagged but no slot was left. Slots
                            are a bijection onto [0, fb_count) in no fixed order */
  int8_t *res_codes;     /* [capacity][16384] tile order, Q^(dQ(G))   (Sec. 4.3) */
  int8_t *res_codes_t;   /* [capacity][16384] tile order of the transposed
                            residual block, or NULL                              */
  float *res_scales;     /* [capacity]  a~ of the block in that slot  (Sec. 4.3) */
} fq_qtensor;

/* Bytes of device memory fq_qtensor_bind needs for a rows x cols matrix with
 * `capacity` residual slots (0 <= capacity <= nbr*nbc; nbr*nbc can never
 * overflow).  Returns 0 on invalid arguments.  Host-only, no HIP call. */
size_t fq_qtensor_bytes(int32_t rows, int32_t cols, int32_t block, int32_t capacity,
                        int want_transposed);

/* Carve the buffers of `out` from `base` (device, 256-byte aligned, at least
 * fq_qtensor_bytes bytes) and fill the scalar fields.  Host-only. */
fq_status fq_qtensor_bind(void *base, int32_t rows, int32_t cols, int32_t block,
                          int32_t capacity, int want_transposed, fq_qtensor *out);

/*
 * Quantize x_bf16 (device, row-major [rows, ld] bf16, ld >= cols) into `out`.
 *   per block: a = max|G|/127, codes = round-to-nearest-even(G/a) clamped to
 *   +-127 (Sec. 3.1); u from `crit`/`theta` (Sec. 4.4); for u = 1 the residual
 *   G - a*codes is quantized the same way into a residual slot (Sec. 4.3).
 *   An all-zero block has scale 0 and codes 0.  Arithmetic is IEEE binary32,
 *   division correctly rounded.  Non-finite inputs give unspecified codes.
 * Outputs: every buffer of `out` that is not NULL-optional (codes, scales,
 * mask, fb_count, fb_list, fb_slot; res_* when capacity > 0; *_t when set).
 * The first call into a freshly bound tensor also clears fb_counters.
 * fb_list is written by the workgroup that records the last decision, from all blocks' flags.
 * out->capacity may be 0 only with FQ_CRIT_NONE.  If more blocks are flagged
 * than there are slots, the surplus blocks get fb_slot = -2, fb_count still
 * reports the true count, and any fq_gemm using the tensor as A writes NaN to
 * the affected output rows; fq_qtensor_check reports FQ_ERR_CAPACITY.
 * Errors: FQ_ERR_NULL, FQ_ERR_SHAPE (rows/cols < 0, ld < cols), FQ_ERR_BLOCK,
 * FQ_ERR_ENUM, FQ_ERR_CAPACITY (capacity 0 with a fallback criterion),
 * FQ_ERR_HIP.  rows == 0 or cols == 0 is valid and only zeroes fb_count.
 * Stream capture: the call may be recorded into a HIP graph (it launches kernels only, no
 * memset); the recorded form clears the tensor's counters itself, so the graph can be
 * replayed any number of times.  Once a call into a tensor has been captured, every later call
 * into it (eager calls between replays included) takes that two-launch form as well, so eager
 * calls and replays may be mixed freely; fq_qtensor_bind resets this.
 */
fq_status fq_quantize(const void *x_bf16, int32_t rows, int32_t cols, int64_t ld,
                      int32_t block, fq_criterion crit, float theta, fq_qtensor *out,
                      void *hip_stream);

/*
 * TopK AbsMax selection (Sec. 4.4): as fq_quantize, but u = 1 for the k blocks with the
 * largest max|G| (every block if k >= nbr*nbc, none if k <= 0).  Among blocks with equal
 * max|G| the lower block id bi*nbc + bk is taken first (the paper leaves this open), so the
 * result is unique.  Three launches on `hip_stream`: max|G| of every block (kept in
 * out->scales until the last launch overwrites it with the scales), the selection (one
 * workgroup: a radix select over the nbr*nbc values), and the fused quantizer with that
 * selection as its decision; the input is read twice, (5 + f) bytes per element instead of
 * (3 + f).  out->criterion becomes FQ_CRIT_TOPK.  The number of flagged blocks is known
 * beforehand: FQ_ERR_CAPACITY if out->capacity < min(max(k, 0), nbr*nbc).  Other arguments,
 * outputs and errors as fq_quantize.
 */
fq_status fq_quantize_topk(const void *x_bf16, int32_t rows, int32_t cols, int64_t ld,
                           int32_t block, int32_t k, fq_qtensor *out, void *hip_stream);

/*
 * Block INT8 quantization with stochastic rounding (Sec. 3.1: x is rounded up with
 * probability x - floor(x), so E[Q_s(x)] = x), the form the paper uses for the output
 * gradient dY and for the stored activation context X (Sec. 5.1, 5.3).  No fallback:
 * out->criterion becomes FQ_CRIT_NONE, mask is all 0, fb_count 0, every fb_slot -1.
 * Same scale as fq_quantize (a = max|G|/127).  Element (r, c) draws its random word from
 * the counter-based generator Philox4x32-10 with key `seed` and counter (r*cols + c) >> 2
 * (output word (r*cols + c) & 3); with t = x/a in binary32 and u the word's top 24 bits,
 * code = floor(t) + [u < (t - floor(t)) * 2^24], clamped to +-127.  Results depend only on
 * (x, seed), not on launch shape, and `codes_t` holds the same draw transposed.
 * Arguments, layouts and errors as fq_quantize (capacity may be 0).
 */
fq_status fq_quantize_sr(const void *x_bf16, int32_t rows, int32_t cols, int64_t ld,
                         int32_t block, uint64_t seed, fq_qtensor *out, void *hip_stream);

/*
 * Delay Threshold (App. D, Alg. 2), host-only: the threshold a layer should use in the NEXT
 * step given the fallback count its quantizer reported in this one (fq_qtensor_check).
 * rate = n_fallback / n_blocks (binary32); returns theta / alpha if rate < r_min,
 * theta * alpha if rate > r_max, theta otherwise (also when n_blocks <= 0).  The paper
 * starts every layer at theta = 1 and uses [r_min, r_max] = [0.1, 0.3], alpha = 1.3.
 */
float fq_threshold_update(float theta, int32_t n_fallback, int32_t n_blocks, float r_min,
                          float r_max, float alpha);

/*
 * INT10 compression of an activation context with 1 x 128 groups (Sec. 5.2: what a
 * normalization or activation layer keeps for its backward pass is stored as 10-bit
 * integers per 1 x 128 group, 5/8 of the bf16 bytes; Sec. 5.3: dequantized in backward).
 * A row of `cols` values has ng = ceil(cols/128) groups; a group is the values that exist.
 *   a = max|x| / 511 (binary32, correctly rounded division),
 *   q = round-to-nearest-even(x / a) clamped to +-511 (0 when a = 0).
 * packed: device, [rows*ng] records of FQ_CTX_GROUP_BYTES = 160 bytes, group (r, j) at
 *   (r*ng + j)*160; value i of the group is the two's-complement field in bits
 *   [10 i, 10 i + 10) of the record read as a little-endian bit string; fields of values
 *   beyond `cols` are 0.  scales: device, float [rows*ng].
 * fq_ctx_packed_bytes / fq_ctx_scales_bytes give the two buffer sizes (0 on invalid or
 * overflowing shapes; host-only).  packed must be 4-byte aligned.
 * Errors: FQ_ERR_NULL, FQ_ERR_SHAPE (rows/cols < 0, ld < cols, misaligned packed), FQ_ERR_HIP.
 * rows == 0 or cols == 0 is valid and launches nothing.
 */
#define FQ_CTX_GROUP 128
#define FQ_CTX_GROUP_BYTES 160
size_t fq_ctx_packed_bytes(int32_t rows, int32_t cols);
size_t fq_ctx_scales_bytes(int32_t rows, int32_t cols);
fq_status fq_ctx_quantize(const void *x_bf16, int32_t rows, int32_t cols, int64_t ld,
                          uint8_t *packed, float *scales, void *hip_stream);

/* Inverse of fq_ctx_quantize: out_bf16[r, c] = RNE-bf16(a * q) (device, row-major
 * [rows, ldo] bf16, ldo >= cols).  Same layouts and errors. */
fq_status fq_ctx_dequantize(const uint8_t *packed, const float *scales, int32_t rows,
                            int32_t cols, void *out_bf16, int64_t ldo, void *hip_stream);

/*
 * SiLU-gated linear unit y = silu(x1) * x2, silu(x) = x / (1 + e^-x) (Sec. 4.1), as a non-linear
 * layer of Sec. 5.2: bf16 inputs and output, and in the same pass over x1 and x2 their INT10
 * contexts (exactly what fq_ctx_quantize would write) for the backward pass.  x1, x2: device,
 * row-major [rows, ld] bf16; y: [rows, ldy] bf16.  Function values are computed in binary32
 * with the hardware exponential and reciprocal (about 1 ulp each) and rounded to bf16: a
 * result is within one bf16 step of the correctly rounded value and equal to it for all but
 * about one element in a thousand; magnitudes below 2^-100 may come out as zero.
 * Errors and layouts as fq_ctx_quantize (ld, ldy >= cols).
 */
fq_status fq_glu_forward(const void *x1_bf16, const void *x2_bf16, int32_t rows, int32_t cols,
                         int64_t ld, void *y_bf16, int64_t ldy, uint8_t *ctx1_packed,
                         float *ctx1_scales, uint8_t *ctx2_packed, float *ctx2_scales,
                         void *hip_stream);

/*
 * Backward of fq_glu_forward with the contexts dequantized on the fly (Sec. 5.3): with
 * x1~ = a*q, x2~ = a*q (one binary32 multiplication each) and s = 1 / (1 + e^-x1~),
 *   dx2 = dy * x1~ * s,      dx1 = dy * x2~ * s * (1 + x1~ * (1 - s)).
 * dy: device [rows, ld_dy] bf16; dx1, dx2: device [rows, ldo] bf16.  Accuracy as in the forward
 * pass, plus an absolute error of up to 2^-20 |dy x2~| in dx1 near the zero of silu'
 * (x1~ = -1.278), where the factor in parentheses cancels.
 */
fq_status fq_glu_backward(const void *dy_bf16, int64_t ld_dy, const uint8_t *ctx1_packed,
                          const float *ctx1_scales, const uint8_t *ctx2_packed,
                          const float *ctx2_scales, int32_t rows, int32_t cols, void *dx1_bf16,
                          void *dx2_bf16, int64_t ldo, void *hip_stream);

/*
 * RMS normalization y = x * rstd * w, rstd = 1 / sqrt(mean(x^2) + eps) per row, as a non-linear
 * layer of Sec. 5.2: bf16 input x [rows, ld], gain w [cols] and output y [rows, ldy]; the same
 * pass writes what the backward pass needs: the INT10 context of x (exactly what
 * fq_ctx_quantize would write) and rstd [rows] (float).  Binary32 arithmetic (the sum of squares
 * in unspecified order, then correctly rounded division, square root and division): rstd is
 * within a few binary32 ulps of the exact value and y within one bf16 step of the correctly
 * rounded one.  cols >= 1.  Errors and layouts as fq_ctx_quantize.
 */
fq_status fq_rmsnorm_forward(const void *x_bf16, const void *w_bf16, int32_t rows, int32_t cols,
                             int64_t ld, float eps, void *y_bf16, int64_t ldy,
                             uint8_t *ctx_packed, float *ctx_scales, float *rstd,
                             void *hip_stream);

/*
 * Backward of fq_rmsnorm_forward with the context dequantized on the fly (Sec. 5.3): with
 * x~ = a*q, xh = x~ * rstd, g = dy * w,
 *   dx = rstd * (g - xh * mean(g * xh))   [rows, ldo] bf16,
 *   dw[c] = sum over rows of dy * xh      [cols] float.
 * Up to 16384 columns: one pass over dy and the context (workgroup `part` takes the rows part,
 * part + n_parts, ... : row mean, dx and its partial column sums of dy * xh from one read of
 * the row), then the sum of the parts in a fixed order, so dw is deterministic for a given
 * n_parts and dx does not depend on it.  Fastest when every pointer and pitch allows 16-byte
 * accesses, cols is a multiple of 16 and at most 12288: then two rows are in flight per
 * workgroup.  Wider rows: the row means first (one workgroup per row), then dx and the partial
 * sums from a second read.  1 <= n_parts <= 65535; one part per compute unit (256) is a good
 * choice.
 * workspace: device, float [n_parts * cols + rows], overwritten.  rows == 0 writes dw = 0.
 */
fq_status fq_rmsnorm_backward(const void *dy_bf16, int64_t ld_dy, const uint8_t *ctx_packed,
                              const float *ctx_scales, const float *rstd, const void *w_bf16,
                              int32_t rows, int32_t cols, void *dx_bf16, int64_t ldo, float *dw,
                              float *workspace, int32_t n_parts, void *hip_stream);

/*
 * fq_rmsnorm_backward for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the
 * same results, bit for bit, but the workspace is a buffer of FQ_STATIC_SCRATCH_FLOATS floats
 * (16 MiB) built into the library, one copy per GPU, held until the process ends.  The call
 * allocates and frees nothing.  FQ_ERR_SCRATCH if n_parts * cols + rows exceeds
 * FQ_STATIC_SCRATCH_FLOATS (choose a smaller n_parts); other arguments and errors as
 * fq_rmsnorm_backward.  All calls on one GPU share that GPU's buffer: calls that may overlap
 * in time on one GPU (different streams or threads) race on it and must be ordered by the
 * caller.  Nothing in the buffer needs clearing between calls (every element a call reads
 * was written by that call).
 */
#define FQ_STATIC_SCRATCH_FLOATS (4 * 1024 * 1024)
fq_status fq_rmsnorm_backward_static(const void *dy_bf16, int64_t ld_dy,
                                     const uint8_t *ctx_packed, const float *ctx_scales,
                                     const float *rstd, const void *w_bf16, int32_t rows,
                                     int32_t cols, void *dx_bf16, int64_t ldo, float *dw,
                                     int32_t n_parts, void *hip_stream);

/*
 * Fallback block GEMM (Alg. 1).  For every output tile, k-blocks ascending:
 *   C += float(P) * (a^A_ik * a^B_kj),  P the exact INT32 product of the code blocks,
 *   and, if u(i,k) = 1,  C += float(P~) * (a~^A_ik * a^B_kj)  with the residual
 *   codes of A against the same B block.  C is accumulated in FP32 by fused
 *   multiply-adds in exactly this order and stored as fp32 or as bf16
 *   (round-to-nearest-even).
 * C: device, row-major [Mout, ldc] of `cdt`, ldc >= Nout (see fq_op for shapes).
 * B must have been quantized with FQ_CRIT_NONE.
 * Errors: FQ_ERR_NULL (also a missing *_t buffer the op needs), FQ_ERR_SHAPE
 * (contraction lengths differ, ldc < Nout), FQ_ERR_BLOCK, FQ_ERR_ENUM, FQ_ERR_HIP.
 * An empty output (Mout or Nout 0) is valid and launches nothing; an empty
 * contraction writes zeros.
 */
fq_status fq_gemm(fq_op op, const fq_qtensor *A, const fq_qtensor *B, void *C,
                  fq_out_dtype cdt, int64_t ldc, void *hip_stream);

/*
 * fq_gemm within a tolerance instead of bit for bit (Sec. 4.5 / Fig. 1b: the dequantization on
 * the general-purpose ALUs is what limits the INT8 GEMM; this variant halves it).  Same operands,
 * same order of the terms, block 128 only (FQ_ERR_BLOCK otherwise).  The INT32 block products are
 * not converted: the matrix instructions accumulate onto the bit pattern of 1.25 * 2^23, the
 * finished value read as binary32 is exactly 1.25 * 2^23 + P, one fused multiply-add per element
 * adds (1.25 * 2^23 + P) * s, and 1.25 * 2^23 times the sum of the scales used is subtracted after
 * every 4 items of the k-loop.  The FP32 additions therefore round at the magnitude of the biased
 * partial sums: the result differs from fq_gemm's by up to about 2e-4 of max |C| (measured; the
 * bound does not grow with K), inside the 1e-3 this library's outputs are held to, but it is not
 * the oracle's result bit for bit.  fq_gemm stays the reference path.  Arguments and errors as
 * fq_gemm.
 */
fq_status fq_gemm_biased(fq_op op, const fq_qtensor *A, const fq_qtensor *B, void *C,
                         fq_out_dtype cdt, int64_t ldc, void *hip_stream);

/*
 * Eq. (1) (no fallback term: A and B quantized with FQ_CRIT_NONE) on the library's plain
 * kernel: one workgroup per 128 x 128 output tile, per 32 x 32 sub-tile and k-group block/32
 * matrix instructions into an INT32 tile, then one convert and one fused multiply-add per
 * element.  It is what fq_gemm runs for blocks of 64 and 32; this entry point also runs it for
 * block 128, so that the throughput curve over the group size (Sec. 4.5, Fig. 1b) can be
 * measured on one kernel.  Same results as fq_gemm, bit for bit; arguments and errors as
 * fq_gemm, plus FQ_ERR_ENUM if A carries fallback blocks.
 */
fq_status fq_gemm_plain(fq_op op, const fq_qtensor *A, const fq_qtensor *B, void *C,
                        fq_out_dtype cdt, int64_t ldc, void *hip_stream);

/*
 * How fq_gemm cuts an rows_out x cols_out output into workgroup tiles (host-only inspection;
 * App. C: the GEMM tile need not equal the quantization block).  The output is covered by
 * 256 x 256 tiles (2 x 2 quantization blocks); when their number would leave the last round of
 * the GPU's compute units mostly idle, the last block columns are covered by 128 x 384 tiles
 * (1 x 3 blocks) instead.  plan[0] = workgroups with 256 x 256 tiles, plan[1] = tile columns
 * they cover, plan[2] = columns of 128 x 384 tiles (0: none).  compute_units <= 0 means the
 * current device's count, or the value of the environment variable FQ_GEMM_CUS if that is set
 * to a positive number (fq_gemm reads the same variable; meant for tuning and tests).  The
 * plan never changes results: every output element is accumulated in Alg. 1's order.
 */
fq_status fq_gemm_tile_plan(int32_t rows_out, int32_t cols_out, int32_t compute_units,
                            int32_t plan[3]);

/* (With blocks of 64 or 32, k_block counts blocks of that size.)
 * The INT32 block product of k-block `k_block` alone (Alg. 1's INT x INT
 * product before dequantization): main term (residual_term = 0) or residual
 * term (1; zero for unflagged blocks).  p_out: device int32 [Mout, Nout]
 * row-major, dense.  Same validation as fq_gemm plus 0 <= k_block < nkb. */
fq_status fq_gemm_debug_partials(fq_op op, const fq_qtensor *A, const fq_qtensor *B,
                                 int32_t k_block, int residual_term, int32_t *p_out,
                                 void *hip_stream);

/* Convert tile-order codes (nbr*nbc blocks of a rows x cols matrix) to a dense
 * row-major int8 [rows, cols] array (device).  For inspection and tests. */
fq_status fq_codes_to_rowmajor(const int8_t *tiled, int32_t rows, int32_t cols,
                               int8_t *dense, void *hip_stream);

/* Waits for `hip_stream`, reads fb_count back and returns FQ_ERR_CAPACITY if it
 * exceeds t->capacity, FQ_OK otherwise; *count_out (host, may be NULL) gets the count. */
fq_status fq_qtensor_check(const fq_qtensor *t, int32_t *count_out, void *hip_stream);

/* Static, never-NULL description of a status code (host). */
const char *fq_status_string(fq_status s);

#ifdef __cplusplus
}
#endif
#endif /* FQ_H_ */
