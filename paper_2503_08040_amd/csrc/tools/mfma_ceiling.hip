// mfma_ceiling -- what the INT8 matrix cores of this GPU sustain with no memory traffic at all.
//
// A register-only loop of one INT8 matrix instruction (2 wavefronts per SIMD on every CU, 4
// independent accumulator tiles per wavefront) is timed for about a second with (a) constant
// operands and (b) uniformly random INT8 operands, for the two instruction shapes
// v_mfma_i32_32x32x32_i8 and v_mfma_i32_16x16x64_i8 (the one the library's GEMM uses).  The part
// is power-limited: operand toggling decides the sustained clock, so (b) is the ceiling that an
// INT8 GEMM on real data competes with.  Prints one JSON line.  This is measurement support for the benchmark's roofline
// context; it is not on the product path.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kIters = 4096;
constexpr int kThreads = 512;

__global__ __launch_bounds__(kThreads) void mfma_loop(const v4i* in, float* out) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = in[(i * 2) * kThreads + threadIdx.x];
    b[i] = in[(i * 2 + 1) * kThreads + threadIdx.x];
  }
  v16i P[4] = {{0}, {0}, {0}, {0}};
  for (int it = 0; it < kIters; ++it) {
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        P[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[g], b[(g + j) & 3], P[j], 0, 0, 0);
  }
  float r = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += (float)P[j][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// The same number of multiply-accumulates with v_mfma_i32_16x16x64_i8: 32 per iteration over 8
// independent 16 x 16 accumulators.
__global__ __launch_bounds__(kThreads) void mfma16_loop(const v4i* in, float* out) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = in[(i * 2) * kThreads + threadIdx.x];
    b[i] = in[(i * 2 + 1) * kThreads + threadIdx.x];
  }
  v4i P[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) P[j] = v4i{0, 0, 0, 0};
  for (int it = 0; it < kIters; ++it) {
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        P[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[g], b[(g + j) & 3], P[j], 0, 0, 0);
  }
  float r = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) r += (float)P[j][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

#define CHECK(x)                                                        \
  do {                                                                  \
    hipError_t e_ = (x);                                                \
    if (e_ != hipSuccess) {                                             \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));    \
      return 1;                                                         \
    }                                                                   \
  } while (0)

int main() {
  hipDeviceProp_t prop;
  CHECK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  const size_t n = 8 * kThreads;
  std::vector<v4i> h(n);
  v4i* in;
  float* out;
  CHECK(hipMalloc(&in, n * sizeof(v4i)));
  CHECK(hipMalloc(&out, (size_t)cus * kThreads * 4));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  double tops[2] = {0, 0}, tops16[2] = {0, 0};
  for (int mode = 0; mode < 2; ++mode) {
    srand(1);
    for (size_t i = 0; i < n; ++i)
      for (int c = 0; c < 4; ++c) {
        uint32_t v = 0x01010101u;
        if (mode == 1) {
          v = 0;
          for (int bb = 0; bb < 4; ++bb) v |= (uint32_t)(((rand() % 255) - 127) & 0xFF) << (8 * bb);
        }
        h[i][c] = (int)v;
      }
    CHECK(hipMemcpy(in, h.data(), n * sizeof(v4i), hipMemcpyHostToDevice));
    // ~0.6 s of warm-up so the clock settles, then time 20 launches
    for (int r = 0; r < 40; ++r) hipLaunchKernelGGL(mfma_loop, dim3(cus), dim3(kThreads), 0, 0, in, out);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    const int launches = 20;
    for (int r = 0; r < launches; ++r)
      hipLaunchKernelGGL(mfma_loop, dim3(cus), dim3(kThreads), 0, 0, in, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double mfma = (double)launches * kIters * 16 * (kThreads / 64) * cus;
    tops[mode] = mfma * 2.0 * 32 * 32 * 32 / (ms * 1e-3) / 1e12;
    // the 16x16x64 shape: same warm-up, same amount of arithmetic per launch
    for (int r = 0; r < 40; ++r) hipLaunchKernelGGL(mfma16_loop, dim3(cus), dim3(kThreads), 0, 0, in, out);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < launches; ++r)
      hipLaunchKernelGGL(mfma16_loop, dim3(cus), dim3(kThreads), 0, 0, in, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    tops16[mode] = mfma * 2.0 * 32 * 32 * 32 / (ms * 1e-3) / 1e12;
  }
  printf("{\"compute_units\": %d, \"mfma_only_tops_constant_operands\": %.1f, "
         "\"mfma_only_tops_random_operands\": %.1f, "
         "\"mfma_16x16x64_only_tops_constant_operands\": %.1f, "
         "\"mfma_16x16x64_only_tops_random_operands\": %.1f}\n", cus, tops[0], tops[1], tops16[0],
         tops16[1]);
  return 0;
}
