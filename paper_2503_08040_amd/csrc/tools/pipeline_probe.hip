// pipeline_probe -- the inner pipeline of the block GEMM in the cycle domain (measurement support).
//
// Paper: Sec. 4.2 Eq. (1) (INT8 block product dequantized per block on the general-purpose ALUs),
// Sec. 4.5 / Fig. 1b (that dequantization is what limits small groups).
//
// Register-resident loops, 2 wavefronts per SIMD on every compute unit (or 1), random INT8
// operands, every instruction of the loop body written in inline assembly so that the stream is
// exactly what is listed: per MFMA "slot" one v_mfma_i32_16x16x64_i8 (or v_mfma_i32_32x32x32_i8),
// NF v_fmac_f32 and NC v_cvt_f32_i32, optionally R ds_read_b128 per 32 x 32 x 128 unit, operands
// in architectural or accumulation registers.  Each wavefront reads the shader clock counter
// (s_memtime) and the constant 100 MHz counter (s_memrealtime) around its loop, so every mode is
// reported as cycles per unit AND as the clock the GPU ran at: the part is power-managed, and a
// time-domain figure alone cannot tell "more cycles" from "lower clock".
// Prints one JSON object per mode, one per line.
#include <hip/hip_runtime.h>
#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(1);} } while (0)

__device__ __forceinline__ uint64_t memtime_now() {
  uint64_t t; asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t)); return t; }
__device__ __forceinline__ uint64_t realtime_now() {
  uint64_t t; asm volatile("s_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t)); return t; }

constexpr int kUnits = 4;
constexpr int kWindowBytes = 2 << 20;   // L2-resident source of the direct-to-LDS loads, shared by all workgroups
constexpr size_t kFarBytes = 128u << 20;  // second source behind the window: too large for an L2, private
                                          // addresses per workgroup, so its loads miss the L2

// AB: 0 A/B fragments in VGPRs, 1 in AGPRs.  NF/NC: FMAs / converts per MFMA.  R: ds_read_b128 per unit.
// SS: 1 = scale from an SGPR.  CV: 1 = the first MFMA of a pair also reads C from registers.
// D: direct-to-LDS loads (global_load_lds_dwordx4, 1 KiB per wavefront each) from an L2-resident
// window into a part of the LDS that nothing reads: 1 = one per unit, 2 = eight in a burst every
// 8 units (right behind the barrier when BAR is set), 3 = the eight over the first six of every 8
// units, so that the last has two units to land before the wait that precedes the barrier, 4 = half
// the wavefronts (one per SIMD) one per unit and the other half two per unit in the first 4 of 8.  BAR: 1 = s_barrier every 8 units.
// D = 6: the two wavefronts of a SIMD half an item apart (wavefronts 0-3 and 4-7 as two teams): a
// barrier every 4 units, which is the item boundary (wait for the loads, burst of 8 loads) of one
// team and the middle of the item of the other, alternately.
// SW: 1 = at its item boundary a wavefront reads its first operands again behind the barrier and waits
// for them, as a k-loop must whose next ring slot only becomes valid at the barrier.
template <int AB, int NF, int NC, int R, int SS, int CV, int kThreads, int D = 0, int BAR = 0, int SW = 0>
__global__ __launch_bounds__(kThreads, 1) void probe(const v4i* in, float* out, uint64_t* stamps, float s, int trips,
                                                     const int8_t* window, int far_every) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned dma_voff = (unsigned)lane * 16u;
  auto dma = [&](int cnt) {   // cnt: running number of this wavefront's loads
    const int8_t* from = window + (size_t)(((cnt * 8 + w) * 1024) & (kWindowBytes - 1));
    if (far_every > 0 && (cnt & (far_every - 1)) == 0)    // every far_every-th load (a power of two) misses the L2
      from = window + kWindowBytes + (((size_t)(cnt * 8 + w) * 1024 + (size_t)blockIdx.x * 299 * 1024) & (kFarBytes - 1));
    const unsigned to = 65536u + (unsigned)w * 8192u + (unsigned)(cnt & 7) * 1024u;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(to), "v"(dma_voff), "s"(from) : "memory");
  };
  for (int i = 0; i < 16; ++i)
    *reinterpret_cast<v4i*>(lds + w * 16384 + i * 1024 + lane * 16) = in[(i & 7) * 512 + (threadIdx.x & 511)];
  __syncthreads();
  v4i fr[2][8];   // [buffer][a0..a3, b0..b3]
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    v4i v = in[i * 512 + (threadIdx.x & 511)];
    if (AB) { asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(fr[0][i][0]) : "v"(v[0]));
              asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(fr[0][i][1]) : "v"(v[1]));
              asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(fr[0][i][2]) : "v"(v[2]));
              asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(fr[0][i][3]) : "v"(v[3])); fr[1][i] = fr[0][i]; }
    else { fr[0][i] = v; fr[1][i] = v; }
  }
  float acc[kUnits][16];
#pragma unroll
  for (int u = 0; u < kUnits; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[u][i] = 0.0f;
  v4i P[2][4];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int q = 0; q < 4; ++q) P[c][q] = v4i{0, 0, 0, 0};
  float T[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  float sv = s;
  asm volatile("" : "+v"(sv));
  const unsigned lds_addr = (unsigned)(w * 16384 + lane * 16);
  if (D == 5 && threadIdx.x < 4) reinterpret_cast<volatile int*>(lds + 140 * 1024)[threadIdx.x] = 0;
  __syncthreads();
  const uint64_t t0 = memtime_now(), r0 = realtime_now();
  if (D == 5 && w < 4) {
    // this wavefront only requests: the 16 loads per 8 units that it and its partner on the SIMD
    // would have issued, until the partner (which only computes) reports that it is through
    volatile int* done = reinterpret_cast<volatile int*>(lds + 140 * 1024);
    uint64_t issue = 0;
    int cnt = 0;
    for (; done[w] == 0 && cnt < (1 << 24); cnt += 8) {
      const uint64_t i0 = memtime_now();
      for (int i = 0; i < 8; ++i) dma(cnt + i);
      issue += memtime_now() - i0;      // until the 8th load has left the wavefront
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    if (threadIdx.x == 0) { stamps[4 * blockIdx.x + 2] = issue; stamps[4 * blockIdx.x + 3] = (uint64_t)cnt; }
    out[blockIdx.x * blockDim.x + threadIdx.x] = 0.0f;
    return;
  }
  for (int it = 0; it < trips; ++it) {
#pragma unroll
    for (int u = 0; u < kUnits; ++u) {
      const int cur = u & 1, nxt = cur ^ 1;
      if (R > 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      auto switch_slot = [&]() {
        if (SW && !AB) {
#pragma unroll
          for (int n = 0; n < R; ++n)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(fr[0][n]) : "v"(lds_addr), "n"(n * 1024));
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
      };
      if (D == 6) {
        if (u == 0) {
          const bool boundary = ((it + (w >> 2)) & 1) == 0;      // of this wavefront's team
          if (boundary) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          asm volatile("s_barrier" ::: "memory");
          if (boundary) {
            for (int i = 0; i < 8; ++i) dma(it * 4 + i);
            switch_slot();
          }
        }
      } else if (u == 0 && (it & 1) == 0) {
        // every 8 units: what the k-loop of the GEMM does once per item
        if (D) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (BAR) asm volatile("s_barrier" ::: "memory");
        if (D == 2) for (int i = 0; i < 8; ++i) dma(it * 4 + i);
        switch_slot();
      }
      if (D == 1) dma(it * kUnits + u);
      if (D == 3) {   // the 8 loads over the first 6 of the 8 units: 2 2 1 1 1 1 0 0
        const int u8 = (it & 1) * 4 + u;
        if (u8 < 6) dma(it * 4 + u);
        if (u8 < 2) dma(it * 4 + u + 1);
      }
      if (D == 4) {   // one wavefront of every SIMD one load per unit, the other two per unit in 4 of 8 units
        if (w < 4) dma(it * kUnits + u);
        else if ((it & 1) == 0) { dma(it * 4 + 2 * u); dma(it * 4 + 2 * u + 1); }
      }
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        const int ks = n >> 2, q = n & 3;
        const int ai = (2 * ks + (q >> 1)) & 3, bi = 4 + ((2 * ks + (q & 1)) & 3);
        if (AB) {
          if (ks || CV) asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(P[cur][q]) : "a"(fr[cur][ai]), "a"(fr[cur][bi]));
          else asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, 0" : "=v"(P[cur][q]) : "a"(fr[cur][ai]), "a"(fr[cur][bi]));
        } else {
          if (ks || CV) asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(P[cur][q]) : "v"(fr[cur][ai]), "v"(fr[cur][bi]));
          else asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, 0" : "=v"(P[cur][q]) : "v"(fr[cur][ai]), "v"(fr[cur][bi]));
        }
        if (n < R) {
          if (AB) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=a"(fr[nxt][n]) : "v"(lds_addr), "n"(n * 1024));
          else asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(fr[nxt][n]) : "v"(lds_addr), "n"(n * 1024));
        }
        const int pu = (u + kUnits - 1) % kUnits;
#pragma unroll
        for (int i = 0; i < NF; ++i) {
          const int e = (NF * n + i) & 15;
          if (SS) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[pu][e]) : "s"(s), "v"(T[i]));
          else asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[pu][e]) : "v"(T[i]), "v"(sv));
        }
#pragma unroll
        for (int i = 0; i < NC; ++i) {
          const int e = (NC * n + i) & 15;
          asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(T[i]) : "v"(P[nxt][e >> 2][e & 3]));
        }
      }
    }
  }
  const uint64_t t1 = memtime_now(), r1 = realtime_now();
  float r = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) r += T[i];
#pragma unroll
  for (int u = 0; u < kUnits; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[u][i];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) r += (float)(P[c][q][i]);
  if (!AB) {
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int q = 0; q < 8; ++q) r += (float)fr[c][q][0];
  } else {
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int q = 0; q < 8; ++q) { int x; asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(fr[c][q][0])); r += (float)x; }
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
  if (D == 5) {
    if (lane == 0) reinterpret_cast<volatile int*>(lds + 140 * 1024)[w - 4] = 1;
    if (threadIdx.x == 256) { stamps[4 * blockIdx.x] = t1 - t0; stamps[4 * blockIdx.x + 1] = r1 - r0; }
  } else if (threadIdx.x == 0) { stamps[4 * blockIdx.x] = t1 - t0; stamps[4 * blockIdx.x + 1] = r1 - r0; }
}


// One trip = 2 pairs of units (4 units): chains X and Y interleaved, 4 MFMAs each (K = 128), and the
// dequantization of the previous pair's tiles spread over the 8 MFMA slots: NV instructions per slot
// (half FMAs, half converts).  CH: 1 = the two chains interleave, 0 = each chain's MFMAs back to back.
// R: ds_read_b128 per unit (operands of the next pair), D and BAR as in probe<>.
template <int NV, int CH, int kThreads, int R = 0, int D = 0, int BAR = 0>
__global__ __launch_bounds__(kThreads, 1) void probe32(const v4i* in, float* out, uint64_t* stamps, float s, int trips,
                                                       const int8_t* window, int /*far_every*/) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (int i = 0; i < 16; ++i)
    *reinterpret_cast<v4i*>(lds + w * 16384 + i * 1024 + lane * 16) = in[(i & 7) * 512 + (threadIdx.x & 511)];
  __syncthreads();
  const unsigned dma_voff = (unsigned)lane * 16u;
  auto dma = [&](int cnt) {
    const int8_t* from = window + (size_t)(((cnt * 8 + w) * 1024) & (kWindowBytes - 1));
    const unsigned to = 65536u + (unsigned)w * 8192u + (unsigned)(cnt & 7) * 1024u;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(to), "v"(dma_voff), "s"(from) : "memory");
  };
  v4i f[2][8];    // [buffer][a0..a3, b0..b3]
#pragma unroll
  for (int i = 0; i < 8; ++i) { f[0][i] = in[i * 512 + (threadIdx.x & 511)]; f[1][i] = f[0][i]; }
  float acc[4][16];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[u][i] = 0.0f;
  v16i P[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) P[c] = v16i{0};
  float T[4] = {0, 0, 0, 0};
  float sv = s;
  asm volatile("" : "+v"(sv));
  const unsigned lds_addr = (unsigned)(w * 16384 + lane * 16);
  __syncthreads();
  const uint64_t t0 = memtime_now(), r0 = realtime_now();
  for (int it = 0; it < trips; ++it) {
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {          // pair of units: tiles P[2pr], P[2pr+1]; dequantizes the other pair
      const int x = 2 * pr, y = 2 * pr + 1, ox = 2 * (pr ^ 1), oy = ox + 1;
      const int cur = pr, nxt = pr ^ 1;
      if (R > 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (pr == 0 && (it & 1) == 0) {
        if (D) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (BAR) asm volatile("s_barrier" ::: "memory");
        if (D == 2) for (int i = 0; i < 8; ++i) dma(it * 4 + i);
      }
      if (D == 1) { dma(it * 4 + 2 * pr); dma(it * 4 + 2 * pr + 1); }
      if (D == 3) {   // the 8 loads over the first 3 of the 4 pairs: 3 3 2 0
        const int p4 = (it & 1) * 2 + pr;
        if (p4 < 3) { dma(it * 4 + 2 * pr); dma(it * 4 + 2 * pr + 1); }
        if (p4 < 2) dma(it * 4 + 2 * pr + 2);
      }
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        const int chain = CH ? (n & 1) : (n >> 2), step = CH ? (n >> 1) : (n & 3);
        const int t = chain ? y : x;
        if (step) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(P[t]) : "v"(f[cur][step]), "v"(f[cur][4 + ((step + chain) & 3)]));
        else asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0" : "=v"(P[t]) : "v"(f[cur][step]), "v"(f[cur][4 + ((step + chain) & 3)]));
        if (n < 2 * R && n < 8) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[nxt][n]) : "v"(lds_addr), "n"(n * 1024));
        constexpr int nf = NV / 2, nc = NV - NV / 2;
        const int ot = (n < 4) ? ox : oy;     // tile being folded in this slot
#pragma unroll
        for (int i = 0; i < nf; ++i) {
          const int e = (nf * n + i) & 15;
          asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[ot][e]) : "v"(T[i]), "v"(sv));
        }
#pragma unroll
        for (int i = 0; i < nc; ++i) {
          const int e = (nc * n + i) & 15;
          asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(T[i]) : "v"(P[ot][e]));
        }
      }
    }
  }
  const uint64_t t1 = memtime_now(), r1 = realtime_now();
  float r = T[0] + T[1] + T[2] + T[3];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[u][i] + (float)P[u][i];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int q = 0; q < 8; ++q) r += (float)f[c][q][0];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
  if (threadIdx.x == 0) { stamps[4 * blockIdx.x] = t1 - t0; stamps[4 * blockIdx.x + 1] = r1 - r0; }
}


// The 16-bit alternative of Sec. 4.3 for a flagged block: its 32 x 32 x 128 step in bf16 on the
// matrix cores, 8 v_mfma_f32_32x32x16_bf16 straight into FP32 accumulators.  CONV: 1 = the B
// operand is made from INT8 codes on the way (per MFMA and lane 8 codes: sign-extend, convert,
// scale, pack: 28 vector instructions), which is what keeping the weights in INT8 would need;
// 0 = both operands are bf16 on chip already (twice the operand bytes of the INT8 residual).
typedef float v16f __attribute__((ext_vector_type(16)));
template <int CONV, int kThreads>
__global__ __launch_bounds__(kThreads, 1) void probe_bf16(const v4i* in, float* out, uint64_t* stamps, float s, int trips,
                                                          const int8_t* /*window*/, int /*far_every*/) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // bf16 bit patterns with small magnitudes: sign, exponent 120..127, mantissa from the input
    const v4i r0 = in[i * 512 + (threadIdx.x & 511)], r1 = in[(4 + i) * 512 + (threadIdx.x & 511)];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      a[i][c] = (r0[c] & 0x807F807F) | 0x3C003C00 | ((r0[c] >> 4) & 0x03800380);
      b[i][c] = (r1[c] & 0x807F807F) | 0x3C003C00 | ((r1[c] >> 4) & 0x03800380);
    }
  }
  v16f acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) acc[u] = v16f{0};
  float sv = s;
  asm volatile("" : "+v"(sv));
  const uint64_t t0 = memtime_now(), r0 = realtime_now();
  for (int it = 0; it < trips; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        v4i bb = b[(u + g) & 3];
        if (CONV) {
          // 8 INT8 codes (two dwords of the fragment) -> 8 scaled bf16 values (four dwords)
          const v4i src = b[(u + g) & 3];
          float f[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            int c8;
            asm volatile("v_bfe_i32 %0, %1, %2, 8" : "=v"(c8) : "v"(src[e >> 2]), "n"(8 * (e & 3)));
            asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(f[e]) : "v"(c8));
            asm volatile("v_mul_f32 %0, %0, %1" : "+v"(f[e]) : "v"(sv));
          }
#pragma unroll
          for (int e = 0; e < 4; ++e)
            asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(bb[e]) : "v"(f[2 * e]), "v"(f[2 * e + 1]));
        }
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[u]) : "v"(a[g & 3]), "v"(bb));
      }
  }
  const uint64_t t1 = memtime_now(), r1 = realtime_now();
  float r = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[u][i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = r;
  if (threadIdx.x == 0) { stamps[4 * blockIdx.x] = t1 - t0; stamps[4 * blockIdx.x + 1] = r1 - r0; }
}


static int g_cus;
static v4i* g_in; static float* g_out; static uint64_t* g_stamps; static int8_t* g_window;

template <typename K>
static void time_kernel(K k, int threads, int units_per_trip, const char* name, const char* desc, int far_every = 0) {
  const int trips = 2048;
  const int ldsb = 144 * 1024;      // one workgroup per compute unit
  CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, ldsb));
  auto launch = [&] { hipLaunchKernelGGL(k, dim3(g_cus), dim3(threads), ldsb, 0, g_in, g_out, g_stamps, 1e-12f, trips,
                                         (const int8_t*)g_window, far_every); };
  const auto t0 = std::chrono::steady_clock::now();
  do { for (int r = 0; r < 8; ++r) launch(); CHECK(hipDeviceSynchronize()); }
  while (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < 0.4);
  hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  const int launches = 20;
  CHECK(hipEventRecord(e0));
  for (int r = 0; r < launches; ++r) launch();
  CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
  float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
  std::vector<uint64_t> st(4 * g_cus);
  CHECK(hipMemcpy(st.data(), g_stamps, st.size() * 8, hipMemcpyDeviceToHost));
  double mt = 0, rt = 0;
  double issue = 0, loads = 0;
  for (int i = 0; i < g_cus; ++i) { mt += st[4 * i]; rt += st[4 * i + 1]; issue += st[4 * i + 2]; loads += st[4 * i + 3]; }
  CHECK(hipMemset(g_stamps, 0, st.size() * 8));
  const double units = (double)trips * units_per_trip;
  const double wps = threads / 256;                           // wavefronts per SIMD
  const double ns_simd_unit = ms / launches * 1e6 / units / wps;
  const double mhz = mt / rt * 100.0;
  const double tops = units * (double)g_cus * (threads / 64) * 2.0 * 32 * 32 * 128 / (ms / launches * 1e-3) / 1e12;
  printf("{\"mode\": \"%s\", \"what\": \"%s\", \"waves_per_simd\": %d, \"ns_per_simd_unit\": %.1f, "
         "\"cycles_per_simd_unit\": %.1f, \"wave_cycles_per_unit\": %.1f, \"clock_mhz\": %.0f, \"chip_tops\": %.0f}\n",
         name, desc, threads / 256, ns_simd_unit, ns_simd_unit * mhz * 1e-3, mt / g_cus / units, mhz, tops);
  if (loads > 0)
    printf("{\"mode\": \"%s\", \"requesting_wave\": {\"loads_per_wave\": %.0f, \"issue_cycles_per_load\": %.1f, "
           "\"cycles_per_load_with_wait\": %.1f}}\n", name, loads / g_cus, issue / loads, mt / loads);
  fflush(stdout);
}

int main() {
  hipDeviceProp_t prop; CHECK(hipGetDeviceProperties(&prop, 0));
  g_cus = prop.multiProcessorCount;
  const size_t n = 8 * 512;
  std::vector<v4i> h(n);
  srand(1);
  for (size_t i = 0; i < n; ++i) for (int c = 0; c < 4; ++c) {
    uint32_t v = 0; for (int bb = 0; bb < 4; ++bb) v |= (uint32_t)(((rand() % 255) - 127) & 0xFF) << (8 * bb);
    h[i][c] = (int)v; }
  CHECK(hipMalloc(&g_in, n * sizeof(v4i))); CHECK(hipMalloc(&g_out, (size_t)g_cus * 512 * 4)); CHECK(hipMalloc(&g_stamps, g_cus * 32)); CHECK(hipMemset(g_stamps, 0, g_cus * 32));
  CHECK(hipMemcpy(g_in, h.data(), n * sizeof(v4i), hipMemcpyHostToDevice));
  CHECK(hipMalloc(&g_window, kWindowBytes + kFarBytes)); CHECK(hipMemset(g_window, 1, kWindowBytes + kFarBytes));
  // a "unit" is a 32 x 32 x 128 multiply-accumulate of one wavefront: 8 MFMA 16x16x64 or 4 MFMA 32x32x32
  //                 AB NF NC R SS CV threads
  time_kernel(probe<0, 0, 0, 0, 0, 0, 512>, 512, kUnits, "mfma16_only", "8 MFMA 16x16x64 per unit, nothing else");
  time_kernel(probe<0, 1, 1, 0, 0, 0, 512>, 512, kUnits, "mfma16_1fma_1cvt", "per MFMA: 1 FMA + 1 convert (half the exact dequantization)");
  time_kernel(probe<0, 2, 2, 0, 0, 0, 512>, 512, kUnits, "mfma16_2fma_2cvt", "per MFMA: 2 FMA + 2 converts = the exact dequantization of Eq. (1) at group 128");
  time_kernel(probe<0, 3, 3, 0, 0, 0, 512>, 512, kUnits, "mfma16_3fma_3cvt", "per MFMA: 3 FMA + 3 converts");
  time_kernel(probe<0, 4, 0, 0, 0, 0, 512>, 512, kUnits, "mfma16_4fma", "per MFMA: 4 FMA");
  time_kernel(probe<0, 0, 4, 0, 0, 0, 512>, 512, kUnits, "mfma16_4cvt", "per MFMA: 4 converts");
  time_kernel(probe<0, 8, 0, 0, 0, 0, 512>, 512, kUnits, "mfma16_8fma", "per MFMA: 8 FMA (the mix of group 64)");
  time_kernel(probe<1, 2, 2, 0, 0, 0, 512>, 512, kUnits, "mfma16_2fma_2cvt_ab_in_agpr", "exact dequantization, A/B operands in accumulation registers");
  time_kernel(probe<0, 2, 2, 0, 1, 0, 512>, 512, kUnits, "mfma16_2fma_2cvt_sgpr_scale", "exact dequantization, scale from a scalar register");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512>, 512, kUnits, "mfma16_2fma_2cvt_3reads", "exact dequantization + 3 ds_read_b128 per unit (what the GEMM's wavefront tile needs)");
  time_kernel(probe<0, 0, 0, 3, 0, 0, 512>, 512, kUnits, "mfma16_3reads", "MFMA + 3 ds_read_b128 per unit, no dequantization");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 0, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_barrier", "the same + a workgroup barrier every 8 units");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 1, 0>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_spread", "the same (no barrier) + one 1 KiB direct-to-LDS load per unit and wavefront (the GEMM's staging volume)");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_spread_barrier", "barrier every 8 units + one direct-to-LDS load per unit");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 2, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_burst_barrier", "barrier every 8 units + the 8 direct-to-LDS loads right behind it (the GEMM's k-loop)");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_spread_barrier_far8", "the same, every 8th load misses the L2", 8);
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 2, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_burst_barrier_far8", "burst behind the barrier, every 8th load misses the L2", 8);
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_spread_barrier_far2", "one load per unit, every 2nd load misses the L2", 2);
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 2, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_burst_barrier_far2", "burst behind the barrier, every 2nd load misses the L2", 2);
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 3, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_early_barrier", "barrier every 8 units + the 8 loads over the first 6 units");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 4, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_mixed_barrier", "barrier every 8 units + per SIMD one wavefront 1 load per unit, the other 2 per unit in the first 4 units");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 5, 0>, 512, kUnits, "mfma16_2fma_2cvt_3reads_partner_requests", "one wavefront per SIMD computes (cycles are its own, 1 wavefront), its partner only issues direct-to-LDS loads back to back");
  time_kernel(probe<0, 0, 0, 3, 0, 0, 512, 2, 1>, 512, kUnits, "mfma16_3reads_dma_burst_barrier", "MFMA + reads + barrier + burst loads, no dequantization");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 2, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_burst_barrier_switch", "the GEMM's k-loop + the first operand reads of an item behind its barrier");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 6, 1, 0>, 512, kUnits, "mfma16_2fma_2cvt_3reads_teams_half_item_apart", "the two wavefronts of a SIMD half an item apart: barrier every 4 units, burst of 8 loads at a wavefront's own item boundary");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 6, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_teams_half_item_apart_switch", "the same + the first operand reads of an item behind its barrier");
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 2, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_dma_burst_barrier_switch_far8", "the GEMM's k-loop + first reads behind the barrier, every 8th load misses the L2", 8);
  time_kernel(probe<0, 2, 2, 3, 0, 0, 512, 6, 1, 1>, 512, kUnits, "mfma16_2fma_2cvt_3reads_teams_half_item_apart_switch_far8", "teams half an item apart + first reads behind the barrier, every 8th load misses the L2", 8);
  time_kernel(probe<0, 2, 2, 0, 0, 0, 256>, 256, kUnits, "mfma16_2fma_2cvt_1wave", "exact dequantization, one wavefront per SIMD");
  time_kernel(probe32<0, 1, 512>, 512, 4, "mfma32_only", "4 MFMA 32x32x32 per unit, nothing else");
  time_kernel(probe32<6, 1, 512>, 512, 4, "mfma32_6valu", "per MFMA 32x32x32: 3 FMA + 3 converts");
  time_kernel(probe32<8, 1, 512>, 512, 4, "mfma32_4fma_4cvt", "per MFMA 32x32x32: 4 FMA + 4 converts = the exact dequantization");
  time_kernel(probe32<10, 1, 512>, 512, 4, "mfma32_10valu", "per MFMA 32x32x32: 5 FMA + 5 converts");
  time_kernel(probe32<8, 0, 512>, 512, 4, "mfma32_4fma_4cvt_chained", "exact dequantization, the 4 MFMAs of a tile back to back");
  time_kernel(probe32<8, 1, 512, 3>, 512, 4, "mfma32_4fma_4cvt_3reads", "exact dequantization + 3 ds_read_b128 per unit");
  time_kernel(probe32<8, 0, 512, 3>, 512, 4, "mfma32_4fma_4cvt_3reads_chained", "the same, MFMAs of a tile back to back");
  time_kernel(probe32<8, 1, 512, 3, 0, 1>, 512, 4, "mfma32_4fma_4cvt_3reads_barrier", "the same (interleaved) + a workgroup barrier every 8 units");
  time_kernel(probe32<8, 1, 512, 3, 1, 1>, 512, 4, "mfma32_4fma_4cvt_3reads_dma_spread_barrier", "barrier every 8 units + one direct-to-LDS load per unit");
  time_kernel(probe32<8, 1, 512, 3, 3, 1>, 512, 4, "mfma32_4fma_4cvt_3reads_dma_early_barrier", "barrier every 8 units + the 8 loads over the first 6 units");
  time_kernel(probe32<8, 1, 512, 3, 1, 0>, 512, 4, "mfma32_4fma_4cvt_3reads_dma_spread", "one direct-to-LDS load per unit, no barrier");
  time_kernel(probe32<8, 1, 512, 3, 2, 1>, 512, 4, "mfma32_4fma_4cvt_3reads_dma_burst_barrier", "barrier every 8 units + the 8 direct-to-LDS loads right behind it");
  time_kernel(probe_bf16<0, 512>, 512, 4, "bf16_fallback_step", "the 16-bit alternative for a flagged block: 8 MFMA 32x32x16 bf16 per unit, both operands bf16 on chip");
  time_kernel(probe_bf16<1, 512>, 512, 4, "bf16_fallback_step_b_from_int8", "the same with the B operand converted from INT8 codes on the way (28 vector instructions per MFMA)");
  return 0;
}
