// C ABI of libfq: argument validation and marshalling into kernel launches.
// Everything is checked on the host before the first HIP call.
#include "../../include/fq.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "fq_device.h"
#include "fq_kernels.h"

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Layout {
  size_t codes, codes_t, scales, mask, fb_counters, fb_list, fb_slot, res_codes, res_codes_t,
      res_scales, total;
};

inline bool valid_block(int32_t block) { return block == 128 || block == 64 || block == 32; }

bool compute_layout(int32_t rows, int32_t cols, int32_t block, int32_t capacity, int want_t,
                    Layout* L) {
  if (rows < 0 || cols < 0 || !valid_block(block) || capacity < 0) return false;
  // codes are stored in 128 x 128 blocks whatever the group size; the per-group grids are finer
  const int64_t nb128 = ceil_div(rows, FQ_BLOCK) * ceil_div(cols, FQ_BLOCK);
  const int64_t nb = ceil_div(rows, block) * ceil_div(cols, block);
  if (capacity > nb || nb > (int64_t)1 << 30) return false;
  if (block != FQ_BLOCK && capacity != 0) return false;      // fallback needs 128 x 128 blocks
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes ? bytes : 1); return o; };
  L->codes = take((size_t)nb128 * FQ_BLOCK_BYTES);
  L->codes_t = want_t ? take((size_t)nb128 * FQ_BLOCK_BYTES) : (size_t)-1;
  L->scales = take((size_t)nb * 4);
  L->mask = take((size_t)nb);
  L->fb_counters = take(16 + 8 * (size_t)((nb + 31) / 32));
  L->fb_list = take((size_t)capacity * 4);
  L->fb_slot = take((size_t)nb * 4);
  L->res_codes = take((size_t)capacity * FQ_BLOCK_BYTES);
  L->res_codes_t = want_t ? take((size_t)capacity * FQ_BLOCK_BYTES) : (size_t)-1;
  L->res_scales = take((size_t)capacity * 4);
  L->total = off;
  return true;
}

fq_status check_qtensor(const fq_qtensor* t) {
  if (!t) return FQ_ERR_NULL;
  if (!valid_block(t->block)) return FQ_ERR_BLOCK;
  if (t->block != FQ_BLOCK && t->capacity != 0) return FQ_ERR_BLOCK;
  if (t->rows < 0 || t->cols < 0 || t->capacity < 0) return FQ_ERR_SHAPE;
  if (!t->codes || !t->scales || !t->mask || !t->fb_count || !t->fb_counters || !t->fb_slot)
    return FQ_ERR_NULL;
  if (t->capacity > 0 && (!t->res_codes || !t->res_scales || !t->fb_list)) return FQ_ERR_NULL;
  if (t->capacity > 0 && t->codes_t && !t->res_codes_t) return FQ_ERR_NULL;
  return FQ_OK;
}

// Validates a GEMM call and fills the kernel parameters (without the output).
fq_status prepare_gemm(fq_op op, const fq_qtensor* A, const fq_qtensor* B, fq::GemmParams* g) {
  fq_status s = check_qtensor(A);
  if (s != FQ_OK) return s;
  s = check_qtensor(B);
  if (s != FQ_OK) return s;
  if (op != FQ_OP_NT && op != FQ_OP_NN && op != FQ_OP_TN) return FQ_ERR_ENUM;
  if (B->criterion != FQ_CRIT_NONE) return FQ_ERR_ENUM;
  if (A->criterion < FQ_CRIT_NONE || A->criterion > FQ_CRIT_TOPK) return FQ_ERR_ENUM;
  const bool a_fb = A->criterion != FQ_CRIT_NONE;
  if (a_fb && A->capacity == 0) return FQ_ERR_CAPACITY;
  if (A->block != B->block) return FQ_ERR_BLOCK;
  const int grp = A->block;
  if (grp != FQ_BLOCK && a_fb) return FQ_ERR_BLOCK;
  // code blocks are 128 x 128; the scale / slot grids have one entry per group
  const int a_r128 = (int)ceil_div(A->rows, FQ_BLOCK), a_c128 = (int)ceil_div(A->cols, FQ_BLOCK);
  const int b_r128 = (int)ceil_div(B->rows, FQ_BLOCK), b_c128 = (int)ceil_div(B->cols, FQ_BLOCK);
  const int a_nbr = (int)ceil_div(A->rows, grp), a_nbc = (int)ceil_div(A->cols, grp);
  const int b_nbr = (int)ceil_div(B->rows, grp), b_nbc = (int)ceil_div(B->cols, grp);
  *g = fq::GemmParams{};
  g->group = grp;
  g->a_scales = A->scales;
  g->a_res_scales = A->res_scales;
  g->a_slot = a_fb ? A->fb_slot : nullptr;
  g->b_scales = B->scales;
  switch (op) {
    case FQ_OP_NT:  // C[M,N] = A[M,K] B[N,K]^T
      if (A->cols != B->cols) return FQ_ERR_SHAPE;
      g->M = A->rows; g->N = B->rows;
      g->nib = a_r128; g->njb = b_r128; g->nkb = a_c128;
      g->a_codes = A->codes; g->a_res = A->res_codes; g->a_si = a_nbc; g->a_sk = 1;
      g->b_codes = B->codes; g->b_sj = b_nbc; g->b_sk = 1;
      g->a_ni = a_nbr; g->a_nk = a_nbc; g->b_nj = b_nbr;
      break;
    case FQ_OP_NN:  // C[M,K] = A[M,N] B[N,K]: B' = B^T
      if (A->cols != B->rows) return FQ_ERR_SHAPE;
      if (!B->codes_t) return FQ_ERR_NULL;
      g->M = A->rows; g->N = B->cols;
      g->nib = a_r128; g->njb = b_c128; g->nkb = a_c128;
      g->a_codes = A->codes; g->a_res = A->res_codes; g->a_si = a_nbc; g->a_sk = 1;
      g->b_codes = B->codes_t; g->b_sj = 1; g->b_sk = b_nbc;
      g->a_ni = a_nbr; g->a_nk = a_nbc; g->b_nj = b_nbc;
      break;
    case FQ_OP_TN:  // C[N,K] = A[M,N]^T B[M,K]: A' = A^T, B' = B^T
      if (A->rows != B->rows) return FQ_ERR_SHAPE;
      if (!A->codes_t || !B->codes_t) return FQ_ERR_NULL;
      if (a_fb && !A->res_codes_t) return FQ_ERR_NULL;
      g->M = A->cols; g->N = B->cols;
      g->nib = a_c128; g->njb = b_c128; g->nkb = a_r128;
      g->a_codes = A->codes_t; g->a_res = A->res_codes_t; g->a_si = 1; g->a_sk = a_nbc;
      g->b_codes = B->codes_t; g->b_sj = 1; g->b_sk = b_nbc;
      g->a_ni = a_nbc; g->a_nk = a_nbr; g->b_nj = b_nbc;
      break;
  }
  return FQ_OK;
}

}  // namespace

extern "C" {

size_t fq_qtensor_bytes(int32_t rows, int32_t cols, int32_t block, int32_t capacity,
                        int want_transposed) {
  Layout L;
  if (!compute_layout(rows, cols, block, capacity, want_transposed, &L)) return 0;
  return L.total;
}

fq_status fq_qtensor_bind(void* base, int32_t rows, int32_t cols, int32_t block,
                          int32_t capacity, int want_transposed, fq_qtensor* out) {
  if (!base || !out) return FQ_ERR_NULL;
  if (!valid_block(block)) return FQ_ERR_BLOCK;
  if (block != FQ_BLOCK && capacity != 0) return FQ_ERR_BLOCK;
  Layout L;
  if (!compute_layout(rows, cols, block, capacity, want_transposed, &L)) return FQ_ERR_SHAPE;
  if ((uintptr_t)base & 255) return FQ_ERR_SHAPE;
  char* b = static_cast<char*>(base);
  out->rows = rows; out->cols = cols; out->block = block; out->capacity = capacity;
  out->criterion = FQ_CRIT_NONE; out->epoch = 0;
  out->codes = reinterpret_cast<int8_t*>(b + L.codes);
  out->codes_t = want_transposed ? reinterpret_cast<int8_t*>(b + L.codes_t) : nullptr;
  out->scales = reinterpret_cast<float*>(b + L.scales);
  out->mask = reinterpret_cast<uint8_t*>(b + L.mask);
  out->fb_counters = reinterpret_cast<int32_t*>(b + L.fb_counters);
  out->fb_count = out->fb_counters;
  out->fb_list = reinterpret_cast<int32_t*>(b + L.fb_list);
  out->fb_slot = reinterpret_cast<int32_t*>(b + L.fb_slot);
  out->res_codes = reinterpret_cast<int8_t*>(b + L.res_codes);
  out->res_codes_t = want_transposed ? reinterpret_cast<int8_t*>(b + L.res_codes_t) : nullptr;
  out->res_scales = reinterpret_cast<float*>(b + L.res_scales);
  return FQ_OK;
}

namespace {
fq_status quantize_impl(const void* x_bf16, int32_t rows, int32_t cols, int64_t ld, int32_t block,
                        fq_criterion crit, float theta, int stochastic, uint64_t seed,
                        int32_t topk, fq_qtensor* out, void* hip_stream) {
  if (!out) return FQ_ERR_NULL;
  if (!valid_block(block)) return FQ_ERR_BLOCK;
  // groups of 64 and 32: plain round-to-nearest block INT8 only (the fallback scheme and the
  // other selectors are defined on the paper's 128 x 128 blocks)
  if (block != FQ_BLOCK && (crit != FQ_CRIT_NONE || stochastic)) return FQ_ERR_BLOCK;
  if (rows < 0 || cols < 0 || ld < cols) return FQ_ERR_SHAPE;
  if (crit < FQ_CRIT_NONE || crit > FQ_CRIT_TOPK) return FQ_ERR_ENUM;
  fq_status s = check_qtensor(out);
  if (s != FQ_OK) return s;
  if (out->rows != rows || out->cols != cols) return FQ_ERR_SHAPE;
  if (out->block != block) return FQ_ERR_BLOCK;
  const bool empty = rows == 0 || cols == 0;
  if (!empty && !x_bf16) return FQ_ERR_NULL;
  if (crit == FQ_CRIT_TOPK) {
    // the number of flagged blocks is known here, so a tensor that cannot hold them is refused
    const int64_t nb = ceil_div(rows, FQ_BLOCK) * ceil_div(cols, FQ_BLOCK);
    if (std::min<int64_t>(std::max<int64_t>(topk, 0), nb) > out->capacity) return FQ_ERR_CAPACITY;
  } else if (crit != FQ_CRIT_NONE && out->capacity == 0 && !empty) {
    return FQ_ERR_CAPACITY;
  }

  fq::QuantParams p{};
  p.x = static_cast<const uint16_t*>(x_bf16);
  p.rows = rows; p.cols = cols; p.ld = ld;
  p.nbr = (int)ceil_div(rows, block); p.nbc = (int)ceil_div(cols, block);
  p.group = block;
  p.vec_ok = (((uintptr_t)x_bf16 & 15) == 0 && (ld % 8) == 0) ? 1 : 0;
  p.crit = (int)crit; p.theta = theta; p.topk = topk; p.capacity = out->capacity;
  p.stochastic = stochastic; p.seed = seed;
  p.codes = out->codes; p.codes_t = out->codes_t;
  p.scales = out->scales; p.mask = out->mask;
  // Two alternating counters: this call counts in one and clears the other for the next call.
  // Under stream capture the launches are replayed without passing through here again, so the
  // recorded form must not depend on which counter is clean: it clears all counters first and
  // counts in counter 0.  A replay leaves counter 0 non-zero at a time the host cannot know, so
  // from then on (epoch -1) every call into the tensor, captured or not, takes that form.
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  const bool capturing =
      hipStreamIsCapturing(static_cast<hipStream_t>(hip_stream), &capture) == hipSuccess &&
      capture == hipStreamCaptureStatusActive;
  const bool sticky = capturing || out->epoch < 0;
  const bool first = out->epoch == 0 || sticky;
  const int live = sticky ? 0 : (out->epoch & 1);
  p.fb_count = out->fb_counters + live;
  p.fb_count_next = out->fb_counters + (live ^ 1);
  p.fb_groups_done = out->fb_counters + 2;
  p.fb_words = reinterpret_cast<unsigned long long*>(out->fb_counters + 4);
  p.clear_both = (first || empty) ? 1 : 0;
  out->fb_count = empty ? out->fb_counters : p.fb_count;
  if (sticky) out->epoch = -1;
  else out->epoch = empty ? 2 : (out->epoch >= (1 << 30) ? 2 + (live ^ 1) : out->epoch + 1);
  p.fb_list = out->fb_list; p.fb_slot = out->fb_slot;
  p.res_codes = out->res_codes; p.res_codes_t = out->res_codes_t; p.res_scales = out->res_scales;
  out->criterion = (int32_t)crit;
  p.fb_count_base = out->fb_counters;
  if (block != FQ_BLOCK) {
    // no fallback, nothing is counted: the counters are cleared and the tensor stays "fresh"
    out->fb_count = out->fb_counters;
    out->epoch = 0;
    if (fq::launch_quantize_group(p, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
      return FQ_ERR_HIP;
    return FQ_OK;
  }
  if (fq::launch_quantize(p, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}
}  // namespace

fq_status fq_quantize(const void* x_bf16, int32_t rows, int32_t cols, int64_t ld, int32_t block,
                      fq_criterion crit, float theta, fq_qtensor* out, void* hip_stream) {
  if (crit == FQ_CRIT_TOPK) return FQ_ERR_ENUM;   // that selection takes k: fq_quantize_topk
  return quantize_impl(x_bf16, rows, cols, ld, block, crit, theta, 0, 0, 0, out, hip_stream);
}

fq_status fq_quantize_topk(const void* x_bf16, int32_t rows, int32_t cols, int64_t ld, int32_t block,
                           int32_t k, fq_qtensor* out, void* hip_stream) {
  return quantize_impl(x_bf16, rows, cols, ld, block, FQ_CRIT_TOPK, 0.0f, 0, 0, k, out, hip_stream);
}

fq_status fq_quantize_sr(const void* x_bf16, int32_t rows, int32_t cols, int64_t ld, int32_t block,
                         uint64_t seed, fq_qtensor* out, void* hip_stream) {
  return quantize_impl(x_bf16, rows, cols, ld, block, FQ_CRIT_NONE, 0.0f, 1, seed, 0, out, hip_stream);
}

float fq_threshold_update(float theta, int32_t n_fallback, int32_t n_blocks, float r_min,
                          float r_max, float alpha) {
  if (n_blocks <= 0) return theta;
  const float rate = (float)n_fallback / (float)n_blocks;
  if (rate < r_min) return theta / alpha;
  if (rate > r_max) return theta * alpha;
  return theta;
}

namespace {
// Number of 1 x 128 groups of a rows x cols context, or -1 if the shape is invalid or too
// large for one launch.
int64_t ctx_groups(int32_t rows, int32_t cols) {
  if (rows < 0 || cols < 0) return -1;
  const int64_t n = (int64_t)rows * ceil_div(cols, FQ_CTX_GROUP);
  return n > ((int64_t)1 << 34) ? -1 : n;
}

fq_status ctx_impl(const void* x, int64_t ld, void* out, int64_t ldo, const uint8_t* packed,
                   const float* scales, int32_t rows, int32_t cols, bool dequantize,
                   void* hip_stream) {
  const int64_t n = ctx_groups(rows, cols);
  const int64_t pitch = dequantize ? ldo : ld;
  const void* dense = dequantize ? out : x;
  if (n < 0 || pitch < cols) return FQ_ERR_SHAPE;
  if (n == 0) return FQ_OK;
  if (!dense || !packed || !scales) return FQ_ERR_NULL;
  if ((uintptr_t)packed & 3) return FQ_ERR_SHAPE;
  fq::CtxParams p{};
  p.x = static_cast<const uint16_t*>(x); p.ld = ld;
  p.out = static_cast<uint16_t*>(out); p.ldo = ldo;
  p.packed = const_cast<uint8_t*>(packed); p.scales = const_cast<float*>(scales);
  p.cols = cols; p.ng = (int)ceil_div(cols, FQ_CTX_GROUP); p.n_groups = n;
  p.vec_ok = (((uintptr_t)dense & 15) == 0 && (pitch % 8) == 0) ? 1 : 0;
  if (fq::launch_ctx(p, dequantize, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}
}  // namespace

size_t fq_ctx_packed_bytes(int32_t rows, int32_t cols) {
  const int64_t n = ctx_groups(rows, cols);
  return n < 0 ? 0 : (size_t)n * FQ_CTX_GROUP_BYTES;
}

size_t fq_ctx_scales_bytes(int32_t rows, int32_t cols) {
  const int64_t n = ctx_groups(rows, cols);
  return n < 0 ? 0 : (size_t)n * sizeof(float);
}

fq_status fq_ctx_quantize(const void* x_bf16, int32_t rows, int32_t cols, int64_t ld,
                          uint8_t* packed, float* scales, void* hip_stream) {
  return ctx_impl(x_bf16, ld, nullptr, 0, packed, scales, rows, cols, false, hip_stream);
}

fq_status fq_ctx_dequantize(const uint8_t* packed, const float* scales, int32_t rows,
                            int32_t cols, void* out_bf16, int64_t ldo, void* hip_stream) {
  return ctx_impl(nullptr, 0, out_bf16, ldo, packed, scales, rows, cols, true, hip_stream);
}

namespace {
inline bool bf16_vec_ok(const void* ptr, int64_t pitch) {
  return ((uintptr_t)ptr & 15) == 0 && (pitch % 8) == 0;
}
}  // namespace

fq_status fq_glu_forward(const void* x1_bf16, const void* x2_bf16, int32_t rows, int32_t cols,
                         int64_t ld, void* y_bf16, int64_t ldy, uint8_t* ctx1_packed,
                         float* ctx1_scales, uint8_t* ctx2_packed, float* ctx2_scales,
                         void* hip_stream) {
  const int64_t n = ctx_groups(rows, cols);
  if (n < 0 || ld < cols || ldy < cols) return FQ_ERR_SHAPE;
  if (n == 0) return FQ_OK;
  if (!x1_bf16 || !x2_bf16 || !y_bf16 || !ctx1_packed || !ctx1_scales || !ctx2_packed ||
      !ctx2_scales)
    return FQ_ERR_NULL;
  if (((uintptr_t)ctx1_packed | (uintptr_t)ctx2_packed) & 3) return FQ_ERR_SHAPE;
  fq::GluParams p{};
  p.x1 = static_cast<const uint16_t*>(x1_bf16); p.x2 = static_cast<const uint16_t*>(x2_bf16);
  p.ld = ld; p.y = static_cast<uint16_t*>(y_bf16); p.ldy = ldy;
  p.packed1 = ctx1_packed; p.scales1 = ctx1_scales; p.packed2 = ctx2_packed; p.scales2 = ctx2_scales;
  p.cols = cols; p.ng = (int)ceil_div(cols, FQ_CTX_GROUP); p.n_groups = n;
  p.vec_ok = bf16_vec_ok(x1_bf16, ld) && bf16_vec_ok(x2_bf16, ld) && bf16_vec_ok(y_bf16, ldy);
  if (fq::launch_glu(p, false, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}

fq_status fq_glu_backward(const void* dy_bf16, int64_t ld_dy, const uint8_t* ctx1_packed,
                          const float* ctx1_scales, const uint8_t* ctx2_packed,
                          const float* ctx2_scales, int32_t rows, int32_t cols, void* dx1_bf16,
                          void* dx2_bf16, int64_t ldo, void* hip_stream) {
  const int64_t n = ctx_groups(rows, cols);
  if (n < 0 || ld_dy < cols || ldo < cols) return FQ_ERR_SHAPE;
  if (n == 0) return FQ_OK;
  if (!dy_bf16 || !dx1_bf16 || !dx2_bf16 || !ctx1_packed || !ctx1_scales || !ctx2_packed ||
      !ctx2_scales)
    return FQ_ERR_NULL;
  if (((uintptr_t)ctx1_packed | (uintptr_t)ctx2_packed) & 3) return FQ_ERR_SHAPE;
  fq::GluParams p{};
  p.dy = static_cast<const uint16_t*>(dy_bf16); p.ld_dy = ld_dy;
  p.dx1 = static_cast<uint16_t*>(dx1_bf16); p.dx2 = static_cast<uint16_t*>(dx2_bf16); p.ldo = ldo;
  p.packed1 = const_cast<uint8_t*>(ctx1_packed); p.scales1 = const_cast<float*>(ctx1_scales);
  p.packed2 = const_cast<uint8_t*>(ctx2_packed); p.scales2 = const_cast<float*>(ctx2_scales);
  p.cols = cols; p.ng = (int)ceil_div(cols, FQ_CTX_GROUP); p.n_groups = n;
  p.vec_ok = bf16_vec_ok(dy_bf16, ld_dy) && bf16_vec_ok(dx1_bf16, ldo) && bf16_vec_ok(dx2_bf16, ldo);
  if (fq::launch_glu(p, true, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}

fq_status fq_rmsnorm_forward(const void* x_bf16, const void* w_bf16, int32_t rows, int32_t cols,
                             int64_t ld, float eps, void* y_bf16, int64_t ldy, uint8_t* ctx_packed,
                             float* ctx_scales, float* rstd, void* hip_stream) {
  const int64_t n = ctx_groups(rows, cols);
  if (n < 0 || cols < 1 || ld < cols || ldy < cols) return FQ_ERR_SHAPE;
  if (rows == 0) return FQ_OK;
  if (!x_bf16 || !w_bf16 || !y_bf16 || !ctx_packed || !ctx_scales || !rstd) return FQ_ERR_NULL;
  if ((uintptr_t)ctx_packed & 3) return FQ_ERR_SHAPE;
  fq::RmsParams p{};
  p.x = static_cast<const uint16_t*>(x_bf16); p.ld = ld;
  p.w = static_cast<const uint16_t*>(w_bf16);
  p.y = static_cast<uint16_t*>(y_bf16); p.ldy = ldy;
  p.rstd = rstd; p.eps = eps; p.packed = ctx_packed; p.scales = ctx_scales;
  p.rows = rows; p.cols = cols; p.ng = (int)ceil_div(cols, FQ_CTX_GROUP);
  p.vec_ok = bf16_vec_ok(x_bf16, ld) && bf16_vec_ok(y_bf16, ldy);
  p.vec_w = ((uintptr_t)w_bf16 & 15) == 0;
  if (fq::launch_rmsnorm(p, false, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}

fq_status fq_rmsnorm_backward(const void* dy_bf16, int64_t ld_dy, const uint8_t* ctx_packed,
                              const float* ctx_scales, const float* rstd, const void* w_bf16,
                              int32_t rows, int32_t cols, void* dx_bf16, int64_t ldo, float* dw,
                              float* workspace, int32_t n_parts, void* hip_stream) {
  const int64_t n = ctx_groups(rows, cols);
  if (n < 0 || cols < 1 || ld_dy < cols || ldo < cols) return FQ_ERR_SHAPE;
  if (n_parts < 1 || n_parts > 65535) return FQ_ERR_SHAPE;
  if (!dw || !workspace) return FQ_ERR_NULL;
  if (rows > 0 && (!dy_bf16 || !dx_bf16 || !ctx_packed || !ctx_scales || !rstd || !w_bf16))
    return FQ_ERR_NULL;
  if ((uintptr_t)ctx_packed & 3) return FQ_ERR_SHAPE;
  fq::RmsParams p{};
  p.dy = static_cast<const uint16_t*>(dy_bf16); p.ld_dy = ld_dy;
  p.dx = static_cast<uint16_t*>(dx_bf16); p.ldo = ldo;
  p.w = static_cast<const uint16_t*>(w_bf16);
  p.rstd = const_cast<float*>(rstd); p.dw = dw; p.n_parts = n_parts;
  p.dw_parts = workspace; p.row_mean = workspace + (size_t)n_parts * cols;
  p.packed = const_cast<uint8_t*>(ctx_packed); p.scales = const_cast<float*>(ctx_scales);
  p.rows = rows; p.cols = cols; p.ng = (int)ceil_div(cols, FQ_CTX_GROUP);
  p.vec_ok = bf16_vec_ok(dy_bf16, ld_dy) && bf16_vec_ok(dx_bf16, ldo);
  p.vec_w = ((uintptr_t)w_bf16 & 15) == 0;
  // with no rows the partial sums are all zero: the kernels still run so that dw is written
  if (fq::launch_rmsnorm(p, true, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}

// Scratch memory of fq_rmsnorm_backward_static: the partial column sums and row means that
// fq_rmsnorm_backward takes through its workspace argument.  Host code never uses the array's
// name as an address: each device's copy is looked up once with hipGetSymbolAddress.
static __device__ __align__(256) float scratch[FQ_STATIC_SCRATCH_FLOATS];

namespace {
constexpr int kScratchDevices = 64;
float* g_scratch_ptr[kScratchDevices];          // per device, nullptr until looked up
std::mutex g_scratch_mutex;

// The current device's copy of `scratch`, or nullptr if the lookup fails.
float* scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kScratchDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  return g_scratch_ptr[dev];
}
}  // namespace

fq_status fq_rmsnorm_backward_static(const void* dy_bf16, int64_t ld_dy, const uint8_t* ctx_packed,
                                     const float* ctx_scales, const float* rstd, const void* w_bf16,
                                     int32_t rows, int32_t cols, void* dx_bf16, int64_t ldo,
                                     float* dw, int32_t n_parts, void* hip_stream) {
  if (rows < 0 || cols < 1 || n_parts < 1 || n_parts > 65535) return FQ_ERR_SHAPE;
  if ((int64_t)n_parts * cols + rows > (int64_t)FQ_STATIC_SCRATCH_FLOATS) return FQ_ERR_SCRATCH;
  float* ws = scratch_of_current_device();
  if (!ws) return FQ_ERR_HIP;
  return fq_rmsnorm_backward(dy_bf16, ld_dy, ctx_packed, ctx_scales, rstd, w_bf16, rows, cols,
                             dx_bf16, ldo, dw, ws, n_parts, hip_stream);
}

namespace {
enum GemmKind { kGemmExact, kGemmPlain, kGemmBiased };
fq_status gemm_impl(fq_op op, const fq_qtensor* A, const fq_qtensor* B, void* C, fq_out_dtype cdt,
                    int64_t ldc, GemmKind kind, void* hip_stream) {
  fq::GemmParams g;
  fq_status s = prepare_gemm(op, A, B, &g);
  if (s != FQ_OK) return s;
  if (cdt != FQ_OUT_F32 && cdt != FQ_OUT_BF16) return FQ_ERR_ENUM;
  if (ldc < g.N) return FQ_ERR_SHAPE;
  if (kind == kGemmBiased && g.group != FQ_BLOCK) return FQ_ERR_BLOCK;
  const bool plain = kind == kGemmPlain;
  g.biased = kind == kGemmBiased ? 1 : 0;
  if (g.M == 0 || g.N == 0) return FQ_OK;
  if (!C) return FQ_ERR_NULL;
  g.c = C; g.ldc = ldc; g.out_bf16 = cdt == FQ_OUT_BF16;
  const int64_t esz = g.out_bf16 ? 2 : 4;
  g.vec_ok = (((uintptr_t)C & 15) == 0 && (ldc * esz) % 16 == 0) ? 1 : 0;
  const hipError_t e = (plain || g.group != FQ_BLOCK)
                           ? fq::launch_gemm_group(g, false, static_cast<hipStream_t>(hip_stream))
                           : fq::launch_gemm(g, false, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FQ_OK : FQ_ERR_HIP;
}
}  // namespace

fq_status fq_gemm(fq_op op, const fq_qtensor* A, const fq_qtensor* B, void* C, fq_out_dtype cdt,
                  int64_t ldc, void* hip_stream) {
  return gemm_impl(op, A, B, C, cdt, ldc, kGemmExact, hip_stream);
}

fq_status fq_gemm_biased(fq_op op, const fq_qtensor* A, const fq_qtensor* B, void* C,
                         fq_out_dtype cdt, int64_t ldc, void* hip_stream) {
  return gemm_impl(op, A, B, C, cdt, ldc, kGemmBiased, hip_stream);
}

fq_status fq_gemm_plain(fq_op op, const fq_qtensor* A, const fq_qtensor* B, void* C,
                        fq_out_dtype cdt, int64_t ldc, void* hip_stream) {
  if (A && A->criterion != FQ_CRIT_NONE) return FQ_ERR_ENUM;    // Eq. (1) only: no fallback term
  return gemm_impl(op, A, B, C, cdt, ldc, kGemmPlain, hip_stream);
}

fq_status fq_gemm_tile_plan(int32_t rows_out, int32_t cols_out, int32_t compute_units,
                            int32_t plan[3]) {
  if (!plan) return FQ_ERR_NULL;
  if (rows_out < 0 || cols_out < 0) return FQ_ERR_SHAPE;
  int out[3];
  fq::gemm_tile_plan((int)ceil_div(rows_out, FQ_BLOCK), (int)ceil_div(cols_out, FQ_BLOCK),
                     compute_units, out);
  plan[0] = out[0]; plan[1] = out[1]; plan[2] = out[2];
  return FQ_OK;
}

fq_status fq_gemm_debug_partials(fq_op op, const fq_qtensor* A, const fq_qtensor* B,
                                 int32_t k_block, int residual_term, int32_t* p_out,
                                 void* hip_stream) {
  fq::GemmParams g;
  fq_status s = prepare_gemm(op, A, B, &g);
  if (s != FQ_OK) return s;
  if (k_block < 0 || k_block >= g.a_nk) return FQ_ERR_SHAPE;
  if (g.M == 0 || g.N == 0) return FQ_OK;
  if (!p_out) return FQ_ERR_NULL;
  g.c = p_out; g.ldc = g.N; g.out_bf16 = 0;
  g.vec_ok = (((uintptr_t)p_out & 15) == 0 && (g.N % 4) == 0) ? 1 : 0;
  g.debug_k = k_block; g.debug_residual = residual_term ? 1 : 0;
  const hipError_t e = g.group != FQ_BLOCK
                           ? fq::launch_gemm_group(g, true, static_cast<hipStream_t>(hip_stream))
                           : fq::launch_gemm(g, true, static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return FQ_ERR_HIP;
  return FQ_OK;
}

fq_status fq_codes_to_rowmajor(const int8_t* tiled, int32_t rows, int32_t cols, int8_t* dense,
                               void* hip_stream) {
  if (rows < 0 || cols < 0) return FQ_ERR_SHAPE;
  if (rows == 0 || cols == 0) return FQ_OK;
  if (!tiled || !dense) return FQ_ERR_NULL;
  if (fq::launch_untile(tiled, rows, cols, dense, static_cast<hipStream_t>(hip_stream)) !=
      hipSuccess)
    return FQ_ERR_HIP;
  return FQ_OK;
}

fq_status fq_qtensor_check(const fq_qtensor* t, int32_t* count_out, void* hip_stream) {
  fq_status s = check_qtensor(t);
  if (s != FQ_OK) return s;
  int32_t n = 0;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(&n, t->fb_count, sizeof n, hipMemcpyDeviceToHost, st) != hipSuccess)
    return FQ_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return FQ_ERR_HIP;
  if (count_out) *count_out = n;
  return n > t->capacity ? FQ_ERR_CAPACITY : FQ_OK;
}

const char* fq_status_string(fq_status s) {
  switch (s) {
    case FQ_OK: return "ok";
    case FQ_ERR_NULL: return "a required pointer is NULL";
    case FQ_ERR_SHAPE: return "invalid or inconsistent shape";
    case FQ_ERR_BLOCK: return "unsupported block size (128; 64 or 32 for plain block INT8 without fallback)";
    case FQ_ERR_ENUM: return "invalid enum value or B operand quantized with fallback";
    case FQ_ERR_CAPACITY: return "more flagged blocks than residual slots";
    case FQ_ERR_HIP: return "HIP call failed";
    case FQ_ERR_SCRATCH: return "needs more scratch memory than the library's built-in buffer holds";
  }
  return "unknown status";
}

}  // extern "C"
