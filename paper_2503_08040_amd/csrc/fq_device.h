// Shared device-side definitions of libfq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fq {

constexpr int kBlock = 128;          // quantization block edge (Sec. 4.5 of the paper)
constexpr int kBlockBytes = 16384;   // one block of INT8 codes
constexpr int kFragBytes = 1024;     // one wavefront-wide 32x32 operand fragment

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

}  // namespace fq
