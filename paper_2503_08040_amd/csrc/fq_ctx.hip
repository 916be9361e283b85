// INT10 compression of activation contexts with 1 x 128 groups.
//
// Paper: Sec. 5.2 (non-linear layers keep bf16 inputs and outputs; what they store
// for the backward pass is quantized per 1 x 128 group to 10-bit integers, 5/8 of
// the bf16 bytes), Sec. 5.3 (contexts are dequantized in the backward pass).
//
// Per group: a = max|x| / 511, q = round-to-nearest-even(x / a) clamped to +-511,
// stored as 128 ten-bit two's-complement fields, value i in bits [10 i, 10 i + 10)
// of a 160-byte little-endian record, followed in a separate array by the fp32
// scale.  Dequantization returns RNE-bf16(a * q).
//
// Eight lanes share a group: lane s owns 16 consecutive values (32 bytes of bf16
// in, 5 dwords of packed fields out), so a wavefront reads 2 KiB and writes
// 1280 contiguous bytes.  Both kernels are pure streaming and HBM-bound
// (3.28 bytes per element).
//
// The same building blocks make the fused form the paper describes for non-linear
// layers, here for the SiLU-gated linear unit y = silu(x1) * x2 (Sec. 4.1): the
// forward kernel writes y and both contexts in one pass over x1 and x2, the backward
// kernel dequantizes the contexts on the fly (Sec. 5.3).
#include "fq_device.h"
#include "fq_kernels.h"

namespace fq {

namespace {

constexpr int kCtxThreads = 256;
constexpr int kLanesPerGroup = 8;
constexpr int kValsPerLane = 16;

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  v2f f = {lo, hi};
  v2bf b = __builtin_convertvector(f, v2bf);
  return __builtin_bit_cast(uint32_t, b);
}

// This lane's position: group index (row * ng + j), lane within the group, first column.
struct LanePos {
  int64_t g, r;
  int s, c0;
  bool live;
};

__device__ inline LanePos lane_pos(int64_t n_groups, int ng) {
  LanePos q;
  const int64_t t = (int64_t)blockIdx.x * kCtxThreads + threadIdx.x;
  q.g = t / kLanesPerGroup;
  q.s = (int)(t % kLanesPerGroup);
  q.live = q.g < n_groups;   // the whole 8-lane team is live or not
  q.r = q.live ? q.g / ng : 0;
  q.c0 = (q.live ? (int)(q.g % ng) : 0) * kCtxGroup + q.s * kValsPerLane;
  return q;
}

// 16 consecutive bf16 values of a row as floats; columns >= cols (and dead lanes) read as 0.
__device__ inline void load16(const uint16_t* src, bool live, bool vec, int c0, int cols,
                              float (&x)[kValsPerLane]) {
  if (live && vec && c0 + kValsPerLane <= cols) {
    const v4u* v = reinterpret_cast<const v4u*>(src);
    const v4u lo = __builtin_nontemporal_load(v), hi = __builtin_nontemporal_load(v + 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(lo[i] << 16);
      x[2 * i + 1] = __uint_as_float(lo[i] & 0xFFFF0000u);
      x[8 + 2 * i] = __uint_as_float(hi[i] << 16);
      x[8 + 2 * i + 1] = __uint_as_float(hi[i] & 0xFFFF0000u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i)
      x[i] = (live && c0 + i < cols) ? bf16_bits_to_float(src[i]) : 0.0f;
  }
}

// 16 floats -> 16 consecutive bf16 values of a row (round-to-nearest-even).
__device__ inline void store16(uint16_t* dst, bool vec, int c0, int cols,
                               const float (&v)[kValsPerLane]) {
  if (vec && c0 + kValsPerLane <= cols) {
    v4u lo, hi;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
      hi[i] = pack_bf16x2(v[8 + 2 * i], v[8 + 2 * i + 1]);
    }
    v4u* o = reinterpret_cast<v4u*>(dst);
    o[0] = lo;
    o[1] = hi;
  } else {
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i)
      if (c0 + i < cols) dst[i] = (uint16_t)float_to_bf16_bits(v[i]);
  }
}

// Quantizes this lane's 16 values of the group (all 8 lanes of the team must call it) and
// writes its 5 dwords of the record, lane 0 of the team the scale.
__device__ inline void quantize_store(const float (&x)[kValsPerLane], const LanePos& q,
                                      uint8_t* packed, float* scales) {
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) amax = fmaxf(amax, fabsf(x[i]));
  amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
  amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
  amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
  const float a = __fdiv_rn(amax, 511.0f);
  const float a_rcp = fast_recip(a);

  uint32_t w[5] = {0, 0, 0, 0, 0};
  if (a != 0.0f) {
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) {
      float t = rint_quotient(x[i], a, a_rcp);
      t = fminf(fmaxf(t, -511.0f), 511.0f);
      const uint32_t bits = (uint32_t)(int)t & 0x3FFu;
      const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
      w[word] |= bits << sh;
      if (sh > 22) w[word + 1] |= bits >> (32 - sh);
    }
  }
  if (!q.live) return;
  uint32_t* dst = reinterpret_cast<uint32_t*>(packed + q.g * kCtxGroupBytes) + q.s * 5;
#pragma unroll
  for (int i = 0; i < 5; ++i) dst[i] = w[i];
  if (q.s == 0) scales[q.g] = a;
}

// This lane's 16 values of the group: scale * code, one binary32 multiplication each.
__device__ inline void load_dequantized(const uint8_t* packed, const float* scales,
                                        const LanePos& q, float (&v)[kValsPerLane]) {
  const uint32_t* srcw = reinterpret_cast<const uint32_t*>(packed + q.g * kCtxGroupBytes) + q.s * 5;
  uint32_t w[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) w[i] = __builtin_nontemporal_load(srcw + i);
  const float a = scales[q.g];
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) {
    const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
    uint32_t bits = w[word] >> sh;
    if (sh > 22) bits |= w[word + 1] << (32 - sh);
    const int code = (int)(bits << 22) >> 22;   // sign-extend the 10-bit field
    v[i] = a * (float)code;
  }
}

__global__ __launch_bounds__(kCtxThreads) void ctx_quantize_kernel(CtxParams p) {
  const LanePos q = lane_pos(p.n_groups, p.ng);
  float x[kValsPerLane];
  load16(p.x + q.r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, x);
  quantize_store(x, q, p.packed, p.scales);
}

__global__ __launch_bounds__(kCtxThreads) void ctx_dequantize_kernel(CtxParams p) {
  const LanePos q = lane_pos(p.n_groups, p.ng);
  if (!q.live || q.c0 >= p.cols) return;
  float v[kValsPerLane];
  load_dequantized(p.packed, p.scales, q, v);
  store16(p.out + q.r * p.ldo + q.c0, p.vec_ok, q.c0, p.cols, v);
}

// logistic function 1 / (1 + e^-x) in binary32 with the hardware exp2 and reciprocal
// approximations; e^-x = inf gives 0, e^-x = 0 gives 1.
__device__ inline float logistic(float x) {
  return __builtin_amdgcn_rcpf(1.0f + __expf(-x));
}

// y = silu(x1) * x2 (Sec. 4.1) with the INT10 contexts of both inputs written by the same
// pass (Sec. 5.2): one read of x1 and x2 instead of three.
__global__ __launch_bounds__(kCtxThreads) void glu_forward_kernel(GluParams p) {
  const LanePos q = lane_pos(p.n_groups, p.ng);
  float x1[kValsPerLane], x2[kValsPerLane], y[kValsPerLane];
  load16(p.x1 + q.r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, x1);
  load16(p.x2 + q.r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, x2);
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) y[i] = x1[i] * logistic(x1[i]) * x2[i];
  if (q.live && q.c0 < p.cols) store16(p.y + q.r * p.ldy + q.c0, p.vec_ok, q.c0, p.cols, y);
  quantize_store(x1, q, p.packed1, p.scales1);
  quantize_store(x2, q, p.packed2, p.scales2);
}

// dx2 = dy * silu(x1~), dx1 = dy * x2~ * silu'(x1~) with x1~, x2~ dequantized on the fly from
// the INT10 contexts (Sec. 5.3); silu'(x) = s (1 + x (1 - s)), s = logistic(x).
__global__ __launch_bounds__(kCtxThreads) void glu_backward_kernel(GluParams p) {
  const LanePos q = lane_pos(p.n_groups, p.ng);
  if (!q.live || q.c0 >= p.cols) return;
  float dy[kValsPerLane], x1[kValsPerLane], x2[kValsPerLane];
  load16(p.dy + q.r * p.ld_dy + q.c0, true, p.vec_ok, q.c0, p.cols, dy);
  load_dequantized(p.packed1, p.scales1, q, x1);
  load_dequantized(p.packed2, p.scales2, q, x2);
  float d1[kValsPerLane], d2[kValsPerLane];
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) {
    const float s = logistic(x1[i]);
    d2[i] = dy[i] * (x1[i] * s);
    d1[i] = dy[i] * x2[i] * (s * (1.0f + x1[i] * (1.0f - s)));
  }
  store16(p.dx1 + q.r * p.ldo + q.c0, p.vec_ok, q.c0, p.cols, d1);
  store16(p.dx2 + q.r * p.ldo + q.c0, p.vec_ok, q.c0, p.cols, d2);
}

}  // namespace

hipError_t launch_glu(const GluParams& p, bool backward, hipStream_t st) {
  if (p.n_groups == 0) return hipSuccess;
  const int64_t threads = p.n_groups * kLanesPerGroup;
  const unsigned grid = (unsigned)((threads + kCtxThreads - 1) / kCtxThreads);
  if (backward)
    hipLaunchKernelGGL(glu_backward_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
  else
    hipLaunchKernelGGL(glu_forward_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_ctx(const CtxParams& p, bool dequantize, hipStream_t st) {
  if (p.n_groups == 0) return hipSuccess;
  const int64_t threads = p.n_groups * kLanesPerGroup;
  const unsigned grid = (unsigned)((threads + kCtxThreads - 1) / kCtxThreads);
  if (dequantize)
    hipLaunchKernelGGL(ctx_dequantize_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
  else
    hipLaunchKernelGGL(ctx_quantize_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
  return hipGetLastError();
}

}  // namespace fq
