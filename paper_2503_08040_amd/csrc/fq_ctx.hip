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

__global__ __launch_bounds__(kCtxThreads) void ctx_quantize_kernel(CtxParams p) {
  const int64_t t = (int64_t)blockIdx.x * kCtxThreads + threadIdx.x;
  const int64_t g = t / kLanesPerGroup;   // group index r*ng + j
  const int s = (int)(t % kLanesPerGroup);
  const bool live = g < p.n_groups;       // the whole 8-lane team is live or not
  const int64_t r = live ? g / p.ng : 0;
  const int j = live ? (int)(g % p.ng) : 0;
  const int c0 = j * kCtxGroup + s * kValsPerLane;

  float x[kValsPerLane];
  const uint16_t* src = p.x + r * p.ld + c0;
  if (live && p.vec_ok && c0 + kValsPerLane <= p.cols) {
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
      x[i] = (live && c0 + i < p.cols) ? bf16_bits_to_float(src[i]) : 0.0f;
  }

  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) amax = fmaxf(amax, fabsf(x[i]));
  amax = fmaxf(amax, __shfl_xor(amax, 1, 64));
  amax = fmaxf(amax, __shfl_xor(amax, 2, 64));
  amax = fmaxf(amax, __shfl_xor(amax, 4, 64));
  const float a = __fdiv_rn(amax, 511.0f);

  uint32_t w[5] = {0, 0, 0, 0, 0};
  if (a != 0.0f) {
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) {
      float q = rintf(__fdiv_rn(x[i], a));
      q = fminf(fmaxf(q, -511.0f), 511.0f);
      const uint32_t bits = (uint32_t)(int)q & 0x3FFu;
      const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
      w[word] |= bits << sh;
      if (sh > 22) w[word + 1] |= bits >> (32 - sh);
    }
  }
  if (!live) return;
  uint32_t* dst = reinterpret_cast<uint32_t*>(p.packed + g * kCtxGroupBytes) + s * 5;
#pragma unroll
  for (int i = 0; i < 5; ++i) dst[i] = w[i];
  if (s == 0) p.scales[g] = a;
}

__global__ __launch_bounds__(kCtxThreads) void ctx_dequantize_kernel(CtxParams p) {
  const int64_t t = (int64_t)blockIdx.x * kCtxThreads + threadIdx.x;
  const int64_t g = t / kLanesPerGroup;
  const int s = (int)(t % kLanesPerGroup);
  if (g >= p.n_groups) return;
  const int64_t r = g / p.ng;
  const int j = (int)(g % p.ng);
  const int c0 = j * kCtxGroup + s * kValsPerLane;
  if (c0 >= p.cols) return;

  const uint32_t* srcw = reinterpret_cast<const uint32_t*>(p.packed + g * kCtxGroupBytes) + s * 5;
  uint32_t w[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) w[i] = __builtin_nontemporal_load(srcw + i);
  const float a = p.scales[g];

  float v[kValsPerLane];
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) {
    const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
    uint32_t bits = w[word] >> sh;
    if (sh > 22) bits |= w[word + 1] << (32 - sh);
    const int q = (int)(bits << 22) >> 22;   // sign-extend the 10-bit field
    v[i] = a * (float)q;
  }

  uint16_t* dst = p.out + r * p.ldo + c0;
  if (p.vec_ok && c0 + kValsPerLane <= p.cols) {
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
      if (c0 + i < p.cols) dst[i] = (uint16_t)float_to_bf16_bits(v[i]);
  }
}

}  // namespace

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
