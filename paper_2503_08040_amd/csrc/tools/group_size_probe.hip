// group_size_probe -- what the quantization group size along K costs on this GPU's matrix cores.
//
// Paper: Sec. 4.5 and Fig. 1b (INT8 block GEMM throughput falls with the group size because every
// group boundary costs a dequantization on the general-purpose ALUs; the paper therefore moves
// from 32 to 128), Sec. 4.3 (the fallback block could also be multiplied in 16-bit; the paper
// keeps INT8 and multiplies the residual instead).
//
// A register-only loop (no LDS or global traffic in the timed part, 2 wavefronts per SIMD on
// every CU, random operands) runs the inner pipeline of a block GEMM on one wavefront tile of
// four 32 x 32 sub-tiles:
//   int8, group g in {128, 64, 32}: g/32 v_mfma_i32_32x32x32_i8 into an INT32 tile, then one
//       convert + one FMA per element into the FP32 accumulators (the dequantization of
//       Eq. (1)), issued between the MFMAs of the next group;
//   int8 without dequantization: the same MFMAs alone (upper bound);
//   bf16: 8 v_mfma_f32_32x32x16_bf16 per sub-tile and 128 of K straight into the FP32
//       accumulators (what a 16-bit fallback block would cost; needs no dequantization);
//   int8 with v_mfma_i32_16x16x64_i8 (8 per step), without and with the group-128
//       dequantization: the instruction shape the library's GEMM uses.
// Prints one JSON line with the time per (32 x 32 x 128) sub-tile step and the chip-wide rate.
// Measurement support only; not on the product path.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kThreads = 512;
constexpr int kTiles = 4;      // 32 x 32 sub-tiles (FP32 accumulator tiles) per wavefront
constexpr int kSteps = 4096;   // passes over the sub-tiles per launch

__device__ __forceinline__ void pin(v16i& x) { asm volatile("" : "+v"(x)); }

// kM = MFMAs per dequantization (4: g = 128, 2: g = 64, 1: g = 32); kDequant = false drops the
// vector-ALU work.
template <int kM, bool kDequant>
__global__ __launch_bounds__(kThreads, 2) void int8_loop(const v4i* in, float* out, float s) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = in[(i * 2) * kThreads + threadIdx.x];
    b[i] = in[(i * 2 + 1) * kThreads + threadIdx.x];
  }
  float acc[kTiles][16];
#pragma unroll
  for (int u = 0; u < kTiles; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[u][i] = 0.0f;
  v16i P[2] = {{0}, {0}};
  constexpr int kPer = 16 / kM;   // elements folded per MFMA slot
  asm volatile("" : "+v"(s));     // keep the scale in a vector register

  for (int it = 0; it < kSteps; ++it) {
#pragma unroll
    for (int u = 0; u < kTiles; ++u) {
#pragma unroll
      for (int grp = 0; grp < 4 / kM; ++grp) {     // groups of this 128-deep step
        const int cur = (u * (4 / kM) + grp) & 1;
#pragma unroll
        for (int g = 0; g < kM; ++g) {
          const v16i z = {0};
          P[cur] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[(grp * kM + g) & 3], b[(u + g) & 3],
                                                         g ? P[cur] : z, 0, 0, 0);
          pin(P[cur]);
          __builtin_amdgcn_sched_barrier(0);
          if (kDequant) {
            // fold 16 / kM elements of the previous group's finished tile into the accumulators
            const int pu = (u + kTiles - 1) % kTiles;
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
              const int e = g * kPer + i;
              acc[pu][e] = __builtin_fmaf((float)P[cur ^ 1][e], s, acc[pu][e]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  }
  float r = 0;
#pragma unroll
  for (int u = 0; u < kTiles; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[u][i];
#pragma unroll
  for (int i = 0; i < 16; ++i) r += (float)(P[0][i] + P[1][i]);
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// The instruction shape the library's GEMM uses: 8 v_mfma_i32_16x16x64_i8 per sub-tile step (four
// 16 x 16 quadrants x two halves of K = 128), group 128, 2 FMAs + 2 converts after every MFMA.
template <bool kDequant>
__global__ __launch_bounds__(kThreads, 2) void int8_16x16_loop(const v4i* in, float* out, float s) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = in[(i * 2) * kThreads + threadIdx.x];
    b[i] = in[(i * 2 + 1) * kThreads + threadIdx.x];
  }
  float acc[kTiles][16];
#pragma unroll
  for (int u = 0; u < kTiles; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[u][i] = 0.0f;
  v4i P[2][4];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int q = 0; q < 4; ++q) P[c][q] = v4i{0, 0, 0, 0};
  asm volatile("" : "+v"(s));

  for (int it = 0; it < kSteps; ++it) {
#pragma unroll
    for (int u = 0; u < kTiles; ++u) {
      const int cur = u & 1;
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        const int ks = n >> 2, q = n & 3;
        const v4i z = {0, 0, 0, 0};
        P[cur][q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[(2 * ks + (q >> 1)) & 3], b[(u + n) & 3],
                                                          ks ? P[cur][q] : z, 0, 0, 0);
        asm volatile("" : "+v"(P[cur][q]));
        __builtin_amdgcn_sched_barrier(0);
        if (kDequant) {
          const int pu = (u + kTiles - 1) % kTiles;
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int e = 2 * n + i;
            acc[pu][e] = __builtin_fmaf((float)P[cur ^ 1][e >> 2][e & 3], s, acc[pu][e]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  float r = 0;
#pragma unroll
  for (int u = 0; u < kTiles; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[u][i];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) r += (float)P[c][q][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

__global__ __launch_bounds__(kThreads, 2) void bf16_loop(const v4i* in, float* out) {
  v8bf a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = __builtin_bit_cast(v8bf, in[(i * 2) * kThreads + threadIdx.x]);
    b[i] = __builtin_bit_cast(v8bf, in[(i * 2 + 1) * kThreads + threadIdx.x]);
  }
  v16f acc[kTiles];
#pragma unroll
  for (int u = 0; u < kTiles; ++u) acc[u] = v16f{0};   // |a b| <= 2^14, 16 per MFMA: the sums stay far inside FP32 range
  for (int it = 0; it < kSteps; ++it) {
#pragma unroll
    for (int u = 0; u < kTiles; ++u)
#pragma unroll
      for (int g = 0; g < 8; ++g)
        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[g & 3], b[(u + g) & 3], acc[u], 0, 0, 0);
  }
  float r = 0;
#pragma unroll
  for (int u = 0; u < kTiles; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[u][i];
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

template <typename F>
static int time_mode(F launch, double* ms_per_launch) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  // warm-up: about 0.7 s under this load so that the clock settles
  const auto t0 = std::chrono::steady_clock::now();
  do {
    for (int r = 0; r < 16; ++r) launch();
    CHECK(hipDeviceSynchronize());
  } while (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < 0.7);
  const int launches = 64;
  CHECK(hipEventRecord(e0));
  for (int r = 0; r < launches; ++r) launch();
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  *ms_per_launch = ms / launches;
  CHECK(hipGetLastError());
  return 0;
}

int main() {
  hipDeviceProp_t prop;
  CHECK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  const size_t n = 8 * kThreads;
  std::vector<v4i> h8(n), h16(n);
  srand(1);
  for (size_t i = 0; i < n; ++i)
    for (int c = 0; c < 4; ++c) {
      uint32_t v = 0, w = 0;
      for (int bb = 0; bb < 4; ++bb) v |= (uint32_t)(((rand() % 255) - 127) & 0xFF) << (8 * bb);
      // two bf16 values with small random integer magnitudes (sign, exponent 127..133, 7-bit mantissa)
      for (int hh = 0; hh < 2; ++hh) {
        const uint32_t bits = ((uint32_t)(rand() & 1) << 15) | ((uint32_t)(127 + rand() % 7) << 7) |
                              (uint32_t)(rand() & 0x7F);
        w |= bits << (16 * hh);
      }
      h8[i][c] = (int)v;
      h16[i][c] = (int)w;
    }
  v4i *in8, *in16;
  float* out;
  CHECK(hipMalloc(&in8, n * sizeof(v4i)));
  CHECK(hipMalloc(&in16, n * sizeof(v4i)));
  CHECK(hipMalloc(&out, (size_t)cus * kThreads * 4));
  CHECK(hipMemcpy(in8, h8.data(), n * sizeof(v4i), hipMemcpyHostToDevice));
  CHECK(hipMemcpy(in16, h16.data(), n * sizeof(v4i), hipMemcpyHostToDevice));

  const dim3 grid(cus), block(kThreads);
  const float s = 1e-12f;
  double ms[7];
  if (time_mode([&] { hipLaunchKernelGGL((int8_loop<4, false>), grid, block, 0, 0, in8, out, s); }, &ms[0])) return 1;
  if (time_mode([&] { hipLaunchKernelGGL((int8_loop<4, true>), grid, block, 0, 0, in8, out, s); }, &ms[1])) return 1;
  if (time_mode([&] { hipLaunchKernelGGL((int8_loop<2, true>), grid, block, 0, 0, in8, out, s); }, &ms[2])) return 1;
  if (time_mode([&] { hipLaunchKernelGGL((int8_loop<1, true>), grid, block, 0, 0, in8, out, s); }, &ms[3])) return 1;
  if (time_mode([&] { hipLaunchKernelGGL(bf16_loop, grid, block, 0, 0, in16, out); }, &ms[4])) return 1;
  if (time_mode([&] { hipLaunchKernelGGL((int8_16x16_loop<false>), grid, block, 0, 0, in8, out, s); }, &ms[5])) return 1;
  if (time_mode([&] { hipLaunchKernelGGL((int8_16x16_loop<true>), grid, block, 0, 0, in8, out, s); }, &ms[6])) return 1;

  // one sub-tile step = 32 x 32 x 128 multiply-accumulates; per launch and wavefront: kTiles * kSteps
  const double steps = (double)kTiles * kSteps, waves = (double)cus * (kThreads / 64);
  const char* names[7] = {"int8_no_dequant", "int8_group128", "int8_group64", "int8_group32",
                          "bf16_direct", "int8_16x16x64_no_dequant", "int8_16x16x64_group128"};
  printf("{\"compute_units\": %d", cus);
  for (int m = 0; m < 7; ++m) {
    const double ns_step = ms[m] * 1e6 / steps;                 // per wavefront, 2 wavefronts share a SIMD
    const double tops = steps * waves * 2.0 * 32 * 32 * 128 / (ms[m] * 1e-3) / 1e12;
    printf(", \"%s\": {\"ns_per_subtile_step\": %.2f, \"tops\": %.1f}", names[m], ns_step, tops);
  }
  printf("}\n");
  return 0;
}
