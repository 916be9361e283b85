// Shared device-side definitions of libfq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fq {

constexpr int kBlock = 128;          // quantization block edge (Sec. 4.5 of the paper)
constexpr int kBlockBytes = 16384;   // one block of INT8 codes
constexpr int kFragBytes = 1024;     // one 32-row x 32-deep run of a block in tile order

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Byte offset of element (r, c) of a 128x128 block in tile order: fragment
// (r/32, c/32) is 1 KiB; inside it lane (r%32) + 32*((c%32)/16) owns 16
// consecutive c.
__host__ __device__ inline int tile_offset(int r, int c) {
  return (((r >> 5) * 4 + (c >> 5)) * 64 + (r & 31) + 32 * ((c & 31) >> 4)) * 16 + (c & 15);
}

__device__ inline float bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16 bit pattern, round-to-nearest-even (finite inputs).
__device__ inline uint32_t float_to_bf16_bits(float f) {
  uint32_t w = __float_as_uint(f);
  return (w + 0x7FFFu + ((w >> 16) & 1u)) >> 16;
}

// round-to-nearest-even of the correctly rounded binary32 quotient x / a, clamped to +-lim, where
// a = max|x| / lim over a set that contains x (lim = 127 or 511), without dividing in the common
// case.  With r = fast_recip(a) (an approximate reciprocal: 1 ulp by specification, 4 ulp are
// allowed for here) the product x * r differs from the true quotient by less than 2^-11 and the
// rounded quotient differs from it by less than 2^-15, so whenever x * r is farther than
// kTieGuard = 2^-10 from a half-integer, both round to the same integer.  Otherwise (about two
// elements in a thousand, or r = NaN) the quotient is formed exactly.
// The clamp is needed only when a is subnormal: a normal a is within 2^-24 (relative) of
// max|x| / lim, so |x / a| <= lim (1 + 2^-23) rounds to at most lim, while a subnormal a can be off
// by half a unit of 2^-149 and the quotient can then exceed lim by far.  fast_recip returns NaN
// for such scales, which sends every element down the exact path, where the clamp is.
// The result equals min(max(rintf(x / a), -lim), lim) in IEEE arithmetic for every finite input.
constexpr float kTieGuard = 0x1p-10f;

// Reciprocal for rint_quotient; NaN (which sends every element down the exact path) when a is
// so small or large that the approximation or the product could leave the normal range.
__device__ inline float fast_recip(float a) {
  return (a >= 0x1p-100f && a <= 0x1p100f) ? __builtin_amdgcn_rcpf(a) : __int_as_float(0x7FC00000);
}

__device__ inline float rint_quotient(float x, float a, float r, float lim) {
  const float tp = x * r;
  float k = rintf(tp);
  if (!(fabsf(tp - k) < 0.5f - kTieGuard)) k = fminf(fmaxf(rintf(__fdiv_rn(x, a)), -lim), lim);
  return k;
}

}  // namespace fq
