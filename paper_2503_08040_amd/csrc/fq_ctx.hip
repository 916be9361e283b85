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
// kStream: load with the non-temporal hint.  Which form is faster was measured per kernel on
// a 4096 x 11008 activation: ordinary loads everywhere except in the SiLU-GLU kernels' large
// streams (two activations forward, two contexts backward); anything read more than once (the
// gain of a normalization, the operands of its two backward passes) must be ordinary.
template <bool kStream = false>
__device__ inline void load16(const uint16_t* src, bool live, bool vec, int c0, int cols,
                              float (&x)[kValsPerLane]) {
  if (live && vec && c0 + kValsPerLane <= cols) {
    const v4u* v = reinterpret_cast<const v4u*>(src);
    const v4u lo = kStream ? __builtin_nontemporal_load(v) : v[0];
    const v4u hi = kStream ? __builtin_nontemporal_load(v + 1) : v[1];
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

// The same 16 values left in their packed form (two per dword, low half first), and the unpacking.
__device__ inline void load16_raw(const uint16_t* src, bool live, bool vec, int c0, int cols,
                                  v4u (&raw)[2]) {
  if (live && vec && c0 + kValsPerLane <= cols) {
    const v4u* v = reinterpret_cast<const v4u*>(src);
    raw[0] = v[0];
    raw[1] = v[1];
  } else {
#pragma unroll
    for (int d = 0; d < 8; ++d) {
      uint32_t wd = 0;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
        if (live && c0 + 2 * d + hh < cols) wd |= (uint32_t)src[2 * d + hh] << (16 * hh);
      raw[d >> 2][d & 3] = wd;
    }
  }
}

__device__ inline void unpack16(const v4u (&raw)[2], float (&x)[kValsPerLane]) {
#pragma unroll
  for (int d = 0; d < 8; ++d) {
    x[2 * d] = __uint_as_float(raw[d >> 2][d & 3] << 16);
    x[2 * d + 1] = __uint_as_float(raw[d >> 2][d & 3] & 0xFFFF0000u);
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

  // The rounded quotient k lies in [-511, 511] (rint_quotient clamps where a clamp can matter).
  // k + 512 is a positive 10-bit number that differs from k's
  // two's-complement field in bit 9 only: the fields are assembled from it without masking and
  // one XOR per dword flips the sixteen sign bits at the end (0x200 repeated every 10 bits).
  uint32_t w[5] = {0, 0, 0, 0, 0};
  if (a != 0.0f) {
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) {
      const uint32_t bits = (uint32_t)(rint_quotient(x[i], a, a_rcp, 511.0f) + 512.0f);
      const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
      w[word] |= bits << sh;
      if (sh > 22) w[word + 1] |= bits >> (32 - sh);
    }
    // bit 9 of field i is bit 10 i + 9 of the 160-bit record
    w[0] ^= 0x20080200u;
    w[1] ^= 0x08020080u;
    w[2] ^= 0x02008020u;
    w[3] ^= 0x00802008u;
    w[4] ^= 0x80200802u;
  }
  if (!q.live) return;
  uint32_t* dst = reinterpret_cast<uint32_t*>(packed + q.g * kCtxGroupBytes) + q.s * 5;
#pragma unroll
  for (int i = 0; i < 5; ++i) dst[i] = w[i];
  if (q.s == 0) scales[q.g] = a;
}

// This lane's 16 values of the group: scale * code, one binary32 multiplication each.
template <bool kStream = false>
__device__ inline void load_dequantized(const uint8_t* packed, const float* scales,
                                        const LanePos& q, float (&v)[kValsPerLane]) {
  const uint32_t* srcw = reinterpret_cast<const uint32_t*>(packed + q.g * kCtxGroupBytes) + q.s * 5;
  uint32_t w[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) w[i] = kStream ? __builtin_nontemporal_load(srcw + i) : srcw[i];
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
  load16<true>(p.x1 + q.r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, x1);
  load16<true>(p.x2 + q.r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, x2);
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
  load_dequantized<true>(p.packed1, p.scales1, q, x1);
  load_dequantized<true>(p.packed2, p.scales2, q, x2);
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

// The two kernels above for matrices that allow 16-byte accesses with cols a multiple of 16 (a
// live lane then owns 16 whole values).  Every load of a thread is issued before the first value
// is used: in the general form each operand's loads sit in a branch of their own together with
// their unpacking, so one operand had arrived before the next was requested.  A lane without
// values reads the first values of its row and drops them.
__global__ __launch_bounds__(kCtxThreads) void glu_forward_vec_kernel(GluParams p) {
  const LanePos q = lane_pos(p.n_groups, p.ng);
  const bool on = q.live && q.c0 < p.cols;
  const int c = on ? q.c0 : 0;
  const v4u* a1 = reinterpret_cast<const v4u*>(p.x1 + q.r * p.ld + c);
  const v4u* a2 = reinterpret_cast<const v4u*>(p.x2 + q.r * p.ld + c);
  v4u r1[2], r2[2];
  r1[0] = __builtin_nontemporal_load(a1);
  r1[1] = __builtin_nontemporal_load(a1 + 1);
  r2[0] = __builtin_nontemporal_load(a2);
  r2[1] = __builtin_nontemporal_load(a2 + 1);
  const v4u zero4 = {0u, 0u, 0u, 0u};
  if (!on) r1[0] = r1[1] = r2[0] = r2[1] = zero4;
  float x1[kValsPerLane], x2[kValsPerLane], y[kValsPerLane];
  unpack16(r1, x1);
  unpack16(r2, x2);
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) y[i] = x1[i] * logistic(x1[i]) * x2[i];
  if (on) store16(p.y + q.r * p.ldy + q.c0, true, q.c0, p.cols, y);
  quantize_store(x1, q, p.packed1, p.scales1);
  quantize_store(x2, q, p.packed2, p.scales2);
}

// the 5 dwords of this lane's 16 ten-bit fields -> scale * code
__device__ inline void dequantize16(const uint32_t (&w)[5], float a, float (&v)[kValsPerLane]) {
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) {
    const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
    uint32_t bits = w[word] >> sh;
    if (sh > 22) bits |= w[word + 1] << (32 - sh);
    const int code = (int)(bits << 22) >> 22;   // sign-extend the 10-bit field
    v[i] = a * (float)code;
  }
}

__global__ __launch_bounds__(kCtxThreads) void glu_backward_vec_kernel(GluParams p) {
  const LanePos q = lane_pos(p.n_groups, p.ng);
  if (!q.live || q.c0 >= p.cols) return;
  const v4u* ad = reinterpret_cast<const v4u*>(p.dy + q.r * p.ld_dy + q.c0);
  const uint32_t* s1 = reinterpret_cast<const uint32_t*>(p.packed1 + q.g * kCtxGroupBytes) + q.s * 5;
  const uint32_t* s2 = reinterpret_cast<const uint32_t*>(p.packed2 + q.g * kCtxGroupBytes) + q.s * 5;
  v4u rd[2];
  uint32_t w1[5], w2[5];
  rd[0] = ad[0];
  rd[1] = ad[1];
#pragma unroll
  for (int i = 0; i < 5; ++i) w1[i] = __builtin_nontemporal_load(s1 + i);
#pragma unroll
  for (int i = 0; i < 5; ++i) w2[i] = __builtin_nontemporal_load(s2 + i);
  const float sa1 = p.scales1[q.g], sa2 = p.scales2[q.g];
  float dy[kValsPerLane], x1[kValsPerLane], x2[kValsPerLane];
  unpack16(rd, dy);
  dequantize16(w1, sa1, x1);
  dequantize16(w2, sa2, x2);
  float d1[kValsPerLane], d2[kValsPerLane];
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) {
    const float s = logistic(x1[i]);
    d2[i] = dy[i] * (x1[i] * s);
    d1[i] = dy[i] * x2[i] * (s * (1.0f + x1[i] * (1.0f - s)));
  }
  store16(p.dx1 + q.r * p.ldo + q.c0, true, q.c0, p.cols, d1);
  store16(p.dx2 + q.r * p.ldo + q.c0, true, q.c0, p.cols, d2);
}

// ---- RMS normalization with a fused INT10 context --------------------------------------------
// One 256-thread workgroup walks a row in chunks of 32 groups (4096 columns): thread t is lane
// t % 8 of group t / 8 of the chunk, the same team layout as above.
constexpr int kRowChunkGroups = kCtxThreads / kLanesPerGroup;   // 32 groups = 4096 columns
constexpr int kRmsMaxChunks = 4;                                // forward keeps rows of up to 4 chunks in registers

__device__ inline LanePos row_pos(int64_t r, int chunk, int ng) {
  LanePos q;
  const int j = chunk * kRowChunkGroups + (int)(threadIdx.x / kLanesPerGroup);
  q.s = (int)(threadIdx.x % kLanesPerGroup);
  q.live = j < ng;
  q.r = r;
  q.g = r * ng + (q.live ? j : 0);
  q.c0 = (q.live ? j : 0) * kCtxGroup + q.s * kValsPerLane;
  return q;
}

// sum over the workgroup; every thread gets the result.  red: 4 floats of LDS.
__device__ inline float block_sum(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();  // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// y = x * rstd * w, rstd = 1 / sqrt(mean(x^2) + eps); also writes rstd and the INT10 context of x.
// kCache: the row (at most kRmsMaxChunks chunks) stays in registers between the two passes;
// otherwise it is read a second time (cache-hot).
template <bool kCache>
__global__ __launch_bounds__(kCtxThreads) void rmsnorm_forward_kernel(RmsParams p) {
  __shared__ float red[4];
  const int64_t r = blockIdx.x;
  const int chunks = (p.ng + kRowChunkGroups - 1) / kRowChunkGroups;
  // the cached row stays in the packed form it was loaded in (half the registers of floats)
  v4u xraw[kCache ? kRmsMaxChunks : 1][2];
  float xc[kValsPerLane];
  float ss = 0.0f;
  if (kCache) {
#pragma unroll
    for (int ch = 0; ch < kRmsMaxChunks; ++ch) {
      const LanePos q = row_pos(r, ch, p.ng);
      load16_raw(p.x + r * p.ld + q.c0, q.live && ch < chunks, p.vec_ok, q.c0, p.cols, xraw[ch]);
    }
#pragma unroll
    for (int ch = 0; ch < kRmsMaxChunks; ++ch) {
      unpack16(xraw[ch], xc);
#pragma unroll
      for (int i = 0; i < kValsPerLane; ++i) ss = __builtin_fmaf(xc[i], xc[i], ss);
    }
  } else {
    for (int ch = 0; ch < chunks; ++ch) {
      const LanePos q = row_pos(r, ch, p.ng);
      load16(p.x + r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, xc);
#pragma unroll
      for (int i = 0; i < kValsPerLane; ++i) ss = __builtin_fmaf(xc[i], xc[i], ss);
    }
  }
  ss = block_sum(ss, red);
  if (kCache) {
    // keep only the packed row across the reduction: the floats are cheap to unpack again
#pragma unroll
    for (int ch = 0; ch < kRmsMaxChunks; ++ch)
      asm volatile("" : "+v"(xraw[ch][0]), "+v"(xraw[ch][1]));
  }
  const float rstd = __fdiv_rn(1.0f, __fsqrt_rn(__fdiv_rn(ss, (float)p.cols) + p.eps));
  if (threadIdx.x == 0) p.rstd[r] = rstd;
  auto finish = [&](int ch, const float (&x)[kValsPerLane]) {
    const LanePos q = row_pos(r, ch, p.ng);
    float w[kValsPerLane], y[kValsPerLane];
    load16(p.w + q.c0, q.live, p.vec_w, q.c0, p.cols, w);
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) y[i] = x[i] * rstd * w[i];
    if (q.live && q.c0 < p.cols) store16(p.y + r * p.ldy + q.c0, p.vec_ok, q.c0, p.cols, y);
    quantize_store(x, q, p.packed, p.scales);
  };
  if (kCache) {
#pragma unroll
    for (int ch = 0; ch < kRmsMaxChunks; ++ch)
      if (ch < chunks) {                        // uniform over the workgroup
        unpack16(xraw[ch], xc);
        finish(ch, xc);
      }
  } else {
    for (int ch = 0; ch < chunks; ++ch) {
      const LanePos q = row_pos(r, ch, p.ng);
      load16(p.x + r * p.ld + q.c0, q.live, p.vec_ok, q.c0, p.cols, xc);
      finish(ch, xc);
    }
  }
}

// The forward kernel for rows of kCh chunks whose matrices and gain allow 16-byte accesses, cols a
// multiple of 16: the loads of the whole row are issued before the first value is used (in the
// general form every chunk's loads sit in a branch of their own), and the gain of the whole row
// is requested before the reduction instead of chunk by chunk behind it.
template <int kCh>
__global__ __launch_bounds__(kCtxThreads) void rmsnorm_forward_vec_kernel(RmsParams p) {
  __shared__ float red[4];
  const int64_t r = blockIdx.x;
  const v4u zero4 = {0u, 0u, 0u, 0u};
  v4u xraw[kCh][2], wraw[kCh][2];
  LanePos q[kCh];
  bool on[kCh];
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    q[ch] = row_pos(r, ch, p.ng);
    on[ch] = q[ch].live && q[ch].c0 < p.cols;
    const v4u* a = reinterpret_cast<const v4u*>(p.x + r * p.ld + (on[ch] ? q[ch].c0 : 0));
    xraw[ch][0] = a[0];
    xraw[ch][1] = a[1];
  }
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    const v4u* a = reinterpret_cast<const v4u*>(p.w + (on[ch] ? q[ch].c0 : 0));
    wraw[ch][0] = a[0];
    wraw[ch][1] = a[1];
  }
  float xc[kValsPerLane];
  float ss = 0.0f;
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    if (!on[ch]) xraw[ch][0] = xraw[ch][1] = zero4;
    unpack16(xraw[ch], xc);
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) ss = __builtin_fmaf(xc[i], xc[i], ss);
  }
  ss = block_sum(ss, red);
  // keep only the packed row across the reduction: the floats are cheap to unpack again
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) asm volatile("" : "+v"(xraw[ch][0]), "+v"(xraw[ch][1]));
  const float rstd = __fdiv_rn(1.0f, __fsqrt_rn(__fdiv_rn(ss, (float)p.cols) + p.eps));
  if (threadIdx.x == 0) p.rstd[r] = rstd;
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    float w[kValsPerLane], y[kValsPerLane];
    unpack16(xraw[ch], xc);
    unpack16(wraw[ch], w);
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) y[i] = xc[i] * rstd * w[i];
    if (on[ch]) store16(p.y + r * p.ldy + q[ch].c0, true, q[ch].c0, p.cols, y);
    quantize_store(xc, q[ch], p.packed, p.scales);
  }
}

// First backward kernel, one workgroup per row: m[r] = mean over the row of g * xh, with
// xh = x~ * rstd (x~ dequantized from the context) and g = dy * w.
__global__ __launch_bounds__(kCtxThreads) void rmsnorm_rowdot_kernel(RmsParams p) {
  __shared__ float red[4];
  const int64_t r = blockIdx.x;
  const int chunks = (p.ng + kRowChunkGroups - 1) / kRowChunkGroups;
  const float rstd = p.rstd[r];
  float m = 0.0f;
  for (int ch = 0; ch < chunks; ++ch) {
    const LanePos q = row_pos(r, ch, p.ng);
    if (!q.live || q.c0 >= p.cols) continue;
    float dy[kValsPerLane], w[kValsPerLane], xq[kValsPerLane];
    load16(p.dy + r * p.ld_dy + q.c0, true, p.vec_ok, q.c0, p.cols, dy);
    load16(p.w + q.c0, true, p.vec_w, q.c0, p.cols, w);
    load_dequantized(p.packed, p.scales, q, xq);
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) m = __builtin_fmaf(dy[i] * w[i], xq[i] * rstd, m);
  }
  m = block_sum(m, red);
  if (threadIdx.x == 0) p.row_mean[r] = __fdiv_rn(m, (float)p.cols);
}

// Second backward kernel, workgroup (chunk, part): for the rows part, part + n_parts, ... and
// the 4096 columns of the chunk, dx = rstd * (g - xh * m[r]) and the partial column sums of
// dy * xh over those rows.
__global__ __launch_bounds__(kCtxThreads) void rmsnorm_dx_dw_kernel(RmsParams p) {
  const int ch = blockIdx.x, part = blockIdx.y;
  const LanePos q0 = row_pos(0, ch, p.ng);
  if (!q0.live || q0.c0 >= p.cols) return;      // no reductions in this kernel: lanes may leave
  float w[kValsPerLane], dwacc[kValsPerLane];
  load16(p.w + q0.c0, true, p.vec_w, q0.c0, p.cols, w);
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i) dwacc[i] = 0.0f;
  for (int64_t r = part; r < p.rows; r += p.n_parts) {
    const LanePos q = row_pos(r, ch, p.ng);
    const float rstd = p.rstd[r], m = p.row_mean[r];
    float dy[kValsPerLane], xq[kValsPerLane], dx[kValsPerLane];
    load16(p.dy + r * p.ld_dy + q.c0, true, p.vec_ok, q.c0, p.cols, dy);
    load_dequantized(p.packed, p.scales, q, xq);
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) {
      const float xh = xq[i] * rstd;
      dx[i] = rstd * (dy[i] * w[i] - xh * m);
      dwacc[i] = __builtin_fmaf(dy[i], xh, dwacc[i]);
    }
    store16(p.dx + r * p.ldo + q.c0, p.vec_ok, q.c0, p.cols, dx);
  }
  float* dst = p.dw_parts + (int64_t)part * p.cols + q0.c0;
#pragma unroll
  for (int i = 0; i < kValsPerLane; ++i)
    if (q0.c0 + i < p.cols) dst[i] = dwacc[i];
}

// Backward in one pass for rows of up to 16384 columns (rows that the two-team kernel further
// down does not take: unaligned ones, and 16-byte rows wider than 12288 columns): a 512-thread
// workgroup `part` takes the
// rows part, part + n_parts, ... one at a time, thread t the 16 values of lane t % 8 of group
// t / 8 in each half of the row (8192 columns).  The row's dy and context are read once (one row
// ahead of their use); dy and xh = x~ * rstd stay in registers while the workgroup reduces the row's
// mean m of g * xh (g = dy * w), then dx = rstd * (g - xh * m) is written and dy * xh is added to
// the workgroup's column sums, which leave through the same [n_parts, cols] partial sums as in
// the two-pass form.  Per element: 2 (dy) + 1.28 (context) read, 2 (dx) written instead of twice
// the reads.
constexpr int kBwdThreads = 512;
constexpr int kBwdChunkGroups = kBwdThreads / kLanesPerGroup;      // 64 groups = 8192 columns
constexpr int kBwdMaxChunks = 2;

// kVec: every matrix of the call allows 16-byte accesses and cols is a multiple of 16, so a live
// lane always owns 16 whole values: its loads and stores are unconditional vector accesses (dead
// lanes read a valid address and discard what they get), which keeps the row loop free of the
// per-access branches of the general form.
template <int kCh, bool kVec>
__global__ __launch_bounds__(kBwdThreads, 2) void rmsnorm_backward_row_kernel(RmsParams p) {
  __shared__ float red[kBwdThreads / 64];
  const int part = blockIdx.x;
  const int s = (int)(threadIdx.x % kLanesPerGroup);
  float wv[kCh][kValsPerLane];      // the gain, unpacked once
  float dwacc[kCh][kValsPerLane];
  bool live[kCh];
  int grp[kCh], c0[kCh];
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    const int j = ch * kBwdChunkGroups + (int)(threadIdx.x / kLanesPerGroup);
    const int c = j * kCtxGroup + s * kValsPerLane;
    live[ch] = j < p.ng && c < p.cols;
    grp[ch] = live[ch] ? j : 0;     // a dead lane reads the row's first values and drops them
    c0[ch] = live[ch] ? c : 0;
    load16(p.w + c0[ch], live[ch], p.vec_w, c0[ch], p.cols, wv[ch]);
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) dwacc[ch][i] = 0.0f;
  }
  const v4u zero4 = {0u, 0u, 0u, 0u};
  // the packed dy and context of a row, requested one row ahead of their use
  v4u dyn[kCh][2];
  uint32_t cwn[kCh][5];
  float csn[kCh], rstdn = 0.0f;
  auto request = [&](int64_t r) {
    rstdn = p.rstd[r];      // first: the loads return in order, and this one is needed first
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      const int64_t g = r * p.ng + grp[ch];
      const uint32_t* srcw = reinterpret_cast<const uint32_t*>(p.packed + g * kCtxGroupBytes) + s * 5;
      if (kVec) {
        const v4u* v = reinterpret_cast<const v4u*>(p.dy + r * p.ld_dy + c0[ch]);
        dyn[ch][0] = v[0];
        dyn[ch][1] = v[1];
#pragma unroll
        for (int i = 0; i < 5; ++i) cwn[ch][i] = srcw[i];
        csn[ch] = p.scales[g];
      } else {
        load16_raw(p.dy + r * p.ld_dy + c0[ch], live[ch], p.vec_ok, c0[ch], p.cols, dyn[ch]);
#pragma unroll
        for (int i = 0; i < 5; ++i) cwn[ch][i] = live[ch] ? srcw[i] : 0u;
        csn[ch] = live[ch] ? p.scales[g] : 0.0f;
      }
    }
  };
  if (part < p.rows) request(part);
  for (int64_t r = part; r < p.rows; r += p.n_parts) {
    v4u dyr[kCh][2];
    uint32_t cw[kCh][5];
    float cs[kCh];
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      // (kVec: what a dead lane has read is dropped here)
      dyr[ch][0] = (kVec && !live[ch]) ? zero4 : dyn[ch][0];
      dyr[ch][1] = (kVec && !live[ch]) ? zero4 : dyn[ch][1];
#pragma unroll
      for (int i = 0; i < 5; ++i) cw[ch][i] = cwn[ch][i];
      cs[ch] = (kVec && !live[ch]) ? 0.0f : csn[ch];
    }
    const float rstd = rstdn;
    if (r + p.n_parts < p.rows) request(r + p.n_parts);
    float xh[kCh][kValsPerLane], dyf[kCh][kValsPerLane];
    float m = 0.0f;
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      unpack16(dyr[ch], dyf[ch]);
#pragma unroll
      for (int i = 0; i < kValsPerLane; ++i) {
        const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
        uint32_t bits = cw[ch][word] >> sh;
        if (sh > 22) bits |= cw[ch][word + 1] << (32 - sh);
        const int code = (int)(bits << 22) >> 22;   // sign-extend the 10-bit field
        xh[ch][i] = (cs[ch] * (float)code) * rstd;
        m = __builtin_fmaf(dyf[ch][i] * wv[ch][i], xh[ch][i], m);
      }
    }
    // sum over the workgroup, every thread gets the result
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m += __shfl_xor(m, off, 64);
    __syncthreads();  // red may still be read from the previous row
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = ((red[0] + red[1]) + (red[2] + red[3])) + ((red[4] + red[5]) + (red[6] + red[7]));
    m = __fdiv_rn(m, (float)p.cols);
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      float dx[kValsPerLane];
#pragma unroll
      for (int i = 0; i < kValsPerLane; ++i) {
        dx[i] = rstd * (dyf[ch][i] * wv[ch][i] - xh[ch][i] * m);
        dwacc[ch][i] = __builtin_fmaf(dyf[ch][i], xh[ch][i], dwacc[ch][i]);
      }
      if (kVec) {
        if (live[ch]) {
          v4u lo, hi;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            lo[i] = pack_bf16x2(dx[2 * i], dx[2 * i + 1]);
            hi[i] = pack_bf16x2(dx[8 + 2 * i], dx[8 + 2 * i + 1]);
          }
          v4u* o = reinterpret_cast<v4u*>(p.dx + r * p.ldo + c0[ch]);
          o[0] = lo;
          o[1] = hi;
        }
      } else if (live[ch]) {
        store16(p.dx + r * p.ldo + c0[ch], p.vec_ok, c0[ch], p.cols, dx);
      }
    }
  }
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    if (!live[ch]) continue;
    float* dst = p.dw_parts + (int64_t)part * p.cols + c0[ch];
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i)
      if (c0[ch] + i < p.cols) dst[i] = dwacc[ch][i];
  }
}

// Backward in one pass for 16-byte rows of up to 12288 columns, the form the tall activations
// of Sec. 5 take.  A team of 256 threads takes one row at a time, thread t the 16 values of lane
// t % 8 of group t / 8 in each 4096-column chunk.  It keeps the row's dy and context as loaded
// (packed bf16 pairs, 10-bit fields) and decodes them twice, before and after the row's
// reduction, instead of holding decoded floats across it: half the registers per value, so a
// second row's loads fit beside the first.
constexpr int kTeamThreads = 256;
constexpr int kTeamGroups = kTeamThreads / kLanesPerGroup;           // 32 groups = 4096 columns
constexpr int kTeamMaxChunks = 3;

// sum over the wavefront's 64 lanes, every lane gets it: four steps inside a row of 16 lanes by
// data-parallel-primitive moves, two across rows through the LDS crossbar
__device__ inline float wave_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));   // lane ^ 1
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));   // lane ^ 2
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));  // 7 - lane (of 8)
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));  // 15 - lane
  v += __shfl_xor(v, 16, 64);
  v += __shfl_xor(v, 32, 64);
  return v;
}

// Two such teams form a workgroup, half a row apart: in every step one team decodes a
// row and reduces it while the other finishes the row it reduced in the step before, with one
// barrier per step; at the end the second team's column sums are added to the first team's through
// LDS, so a compute unit writes one set of partial sums and not two.  A team's rows alternate
// between two register buffers: a row's dy and context are requested into the free buffer while the
// row before it is reduced, two steps ahead of their use.
template <int kCh>
struct PairState {
  float dwacc[kCh][kValsPerLane];
  bool live[kCh];
  int grp[kCh], c0[kCh];
  v4u dy[2][kCh][2];
  uint32_t cw[2][kCh][5];
  float cs[2][kCh], rstd[2];
};

template <int kCh, int kTeam>
__device__ __forceinline__ void pair_team_rows(const RmsParams& p, PairState<kCh>& st, float* red,
                                               const v4u* wl, int part, int t, int s) {
  auto request = [&](int b, int64_t r) {
    st.rstd[b] = p.rstd[r];      // first: the loads return in order, and this one is needed first
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      const int64_t g = r * p.ng + st.grp[ch];
      const uint32_t* srcw = reinterpret_cast<const uint32_t*>(p.packed + g * kCtxGroupBytes) + s * 5;
      const v4u* v = reinterpret_cast<const v4u*>(p.dy + r * p.ld_dy + st.c0[ch]);
      st.dy[b][ch][0] = v[0];
      st.dy[b][ch][1] = v[1];
#pragma unroll
      for (int i = 0; i < 5; ++i) st.cw[b][ch][i] = srcw[i];
      st.cs[b][ch] = p.scales[g];
    }
  };
  // element i of chunk ch in buffer b: dy, w and xh = (scale * code) * rstd
  auto decode = [&](int b, int ch, int i, const v4u (&wv)[2], float& dyf, float& wf, float& xh) {
    const uint32_t dw = st.dy[b][ch][i >> 3][(i >> 1) & 3], ww = wv[i >> 3][(i >> 1) & 3];
    dyf = __uint_as_float((i & 1) ? (dw & 0xFFFF0000u) : (dw << 16));
    wf = __uint_as_float((i & 1) ? (ww & 0xFFFF0000u) : (ww << 16));
    const int pos = 10 * i, word = pos >> 5, sh = pos & 31;
    uint32_t bits = st.cw[b][ch][word] >> sh;
    if (sh > 22) bits |= st.cw[b][ch][word + 1] << (32 - sh);
    const int code = (int)(bits << 22) >> 22;
    xh = (st.cs[b][ch] * (float)code) * st.rstd[b];
  };
  // one row of this team in buffer b: first half, barrier, second half, barrier
  auto row = [&](int b, int64_t r, int64_t r_next) {
    // Wait here, on every path, for all of buffer b: otherwise the compiler, which places its
    // waits per path, waits again further down, behind the request for the next row, and the
    // memory counter being in order that wait would also cover the request.
    asm volatile("" ::"v"(st.rstd[b]));
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      asm volatile("" ::"v"(st.dy[b][ch][0]), "v"(st.dy[b][ch][1]), "v"(st.cw[b][ch][0]),
                   "v"(st.cw[b][ch][1]), "v"(st.cw[b][ch][2]), "v"(st.cw[b][ch][3]),
                   "v"(st.cw[b][ch][4]), "v"(st.cs[b][ch]));
    }
    if (r_next < p.rows) request(b ^ 1, r_next);
    float m = 0.0f;
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      if (st.live[ch]) {
        const v4u wv[2] = {wl[(2 * ch) * kTeamThreads + t], wl[(2 * ch + 1) * kTeamThreads + t]};
#pragma unroll
        for (int i = 0; i < kValsPerLane; ++i) {
          float dyf, wf, xh;
          decode(b, ch, i, wv, dyf, wf, xh);
          m = __builtin_fmaf(dyf * wf, xh, m);
        }
      }
    }
    m = wave_sum(m);
    if ((t & 63) == 0) red[t >> 6] = m;
    __syncthreads();
    m = (red[0] + red[1]) + (red[2] + red[3]);
    m = __fdiv_rn(m, (float)p.cols);
    const float rstd = st.rstd[b];
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      if (st.live[ch]) {
        const v4u wv[2] = {wl[(2 * ch) * kTeamThreads + t], wl[(2 * ch + 1) * kTeamThreads + t]};
        float dx[kValsPerLane];
#pragma unroll
        for (int i = 0; i < kValsPerLane; ++i) {
          float dyf, wf, xh;
          decode(b, ch, i, wv, dyf, wf, xh);
          dx[i] = rstd * (dyf * wf - xh * m);
          st.dwacc[ch][i] = __builtin_fmaf(dyf, xh, st.dwacc[ch][i]);
        }
        v4u lo, hi;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          lo[i] = pack_bf16x2(dx[2 * i], dx[2 * i + 1]);
          hi[i] = pack_bf16x2(dx[8 + 2 * i], dx[8 + 2 * i + 1]);
        }
        v4u* o = reinterpret_cast<v4u*>(p.dx + r * p.ldo + st.c0[ch]);
        o[0] = lo;
        o[1] = hi;
      }
    }
    __syncthreads();
  };
  // The workgroup's rows part, part + n_parts, ... alternate between the teams; team 0 has the
  // first and therefore at least as many as team 1, which starts one step later.  Both teams
  // pass the same number of barriers: 2 n0 + 1, n0 = team 0's rows.
  const int64_t stride = 2 * (int64_t)p.n_parts, first_row = part + (int64_t)kTeam * p.n_parts;
  const int64_t n0 = part < p.rows ? (p.rows - 1 - part) / stride + 1 : 0;
  const int64_t mine = first_row < p.rows ? (p.rows - 1 - first_row) / stride + 1 : 0;
  if (n0 == 0) return;
  if (mine > 0) request(0, first_row);
  if (kTeam == 1) __syncthreads();
  int64_t r = first_row;
  for (int64_t k = 0; k + 1 < mine; k += 2, r += 2 * stride) {
    row(0, r, r + stride);
    row(1, r + stride, r + 2 * stride);
  }
  if (mine & 1) row(0, r, p.rows);
  for (int64_t left = 2 * n0 + 1 - kTeam - 2 * mine; left > 0; --left) __syncthreads();
}

template <int kCh>
__global__ __launch_bounds__(2 * kTeamThreads, 2) void rmsnorm_backward_pair_kernel(RmsParams p) {
  __shared__ float red[2][kTeamThreads / 64];
  // the gain as loaded (bf16 pairs, 32 bytes per thread and chunk) while the rows are processed,
  // then team 1's column sums
  __shared__ __align__(16) float shared[kCh * kValsPerLane * kTeamThreads];
  v4u* wl = reinterpret_cast<v4u*>(shared);
  float (*dwx)[kTeamThreads] = reinterpret_cast<float (*)[kTeamThreads]>(shared);
  const int part = blockIdx.x;
  const int team = (int)(threadIdx.x / kTeamThreads);      // the same for a whole wavefront
  const int t = (int)(threadIdx.x % kTeamThreads);
  const int s = t % kLanesPerGroup;
  PairState<kCh> st;
#pragma unroll
  for (int ch = 0; ch < kCh; ++ch) {
    const int j = ch * kTeamGroups + t / kLanesPerGroup;
    const int c = j * kCtxGroup + s * kValsPerLane;
    st.live[ch] = j < p.ng && c < p.cols;
    st.grp[ch] = st.live[ch] ? j : 0;     // a dead lane reads the row's first values and drops them
    st.c0[ch] = st.live[ch] ? c : 0;
    if (team == 0) {
      const v4u* v = reinterpret_cast<const v4u*>(p.w + st.c0[ch]);
      wl[(2 * ch) * kTeamThreads + t] = v[0];
      wl[(2 * ch + 1) * kTeamThreads + t] = v[1];
    }
#pragma unroll
    for (int i = 0; i < kValsPerLane; ++i) st.dwacc[ch][i] = 0.0f;
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      st.dy[b][ch][0] = st.dy[b][ch][1] = v4u{0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < 5; ++i) st.cw[b][ch][i] = 0u;
      st.cs[b][ch] = 0.0f;
    }
    st.rstd[b] = 0.0f;
  }
  __syncthreads();
  if (team == 0) pair_team_rows<kCh, 0>(p, st, red[0], wl, part, t, s);
  else pair_team_rows<kCh, 1>(p, st, red[1], wl, part, t, s);
  if (team == 1) {
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch)
#pragma unroll
      for (int i = 0; i < kValsPerLane; ++i) dwx[ch * kValsPerLane + i][t] = st.dwacc[ch][i];
  }
  __syncthreads();
  if (team == 0) {
#pragma unroll
    for (int ch = 0; ch < kCh; ++ch) {
      if (!st.live[ch]) continue;
      float* dst = p.dw_parts + (int64_t)part * p.cols + st.c0[ch];
#pragma unroll
      for (int i = 0; i < kValsPerLane; ++i) dst[i] = st.dwacc[ch][i] + dwx[ch * kValsPerLane + i][t];
    }
  }
}

// dw[c] = sum of the partial sums, in a fixed order: thread (slice k of 16, column c) adds the
// parts k, k + 16, k + 32, ... into eight interleaved running sums (eight loads in flight), folds
// them pairwise, and the sixteen slice sums of a column are folded pairwise in slice order.
constexpr int kDwCols = 32, kDwSlices = 16;
__global__ __launch_bounds__(kDwCols * kDwSlices) void rmsnorm_dw_kernel(const float* parts, int n_parts,
                                                                      int cols, float* dw) {
  __shared__ float red[kDwSlices][kDwCols];
  const int lc = threadIdx.x % kDwCols, k = threadIdx.x / kDwCols;
  const int c = blockIdx.x * kDwCols + lc;
  float s[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  if (c < cols) {
    int i = k;
    for (; i + 7 * kDwSlices < n_parts; i += 8 * kDwSlices) {
#pragma unroll
      for (int j = 0; j < 8; ++j) s[j] += parts[(int64_t)(i + j * kDwSlices) * cols + c];
    }
#pragma unroll
    for (int j = 0; j < 7; ++j)     // at most seven parts are left for this slice
      if (i + j * kDwSlices < n_parts) s[j] += parts[(int64_t)(i + j * kDwSlices) * cols + c];
  }
  red[k][lc] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  __syncthreads();
  for (int half = kDwSlices / 2; half > 0; half >>= 1) {
    if (k < half) red[k][lc] += red[k + half][lc];
    __syncthreads();
  }
  if (k == 0 && c < cols) dw[c] = red[0][lc];
}

}  // namespace

hipError_t launch_rmsnorm(const RmsParams& p, bool backward, hipStream_t st) {
  const int chunks = (p.ng + kRowChunkGroups - 1) / kRowChunkGroups;
  if (!backward) {
    if (p.rows == 0) return hipSuccess;
    const dim3 grid((unsigned)p.rows), block(kCtxThreads);
    const bool vec = p.vec_ok && p.vec_w && p.cols % kValsPerLane == 0;
    if (vec && chunks == 1) hipLaunchKernelGGL(rmsnorm_forward_vec_kernel<1>, grid, block, 0, st, p);
    else if (vec && chunks == 2) hipLaunchKernelGGL(rmsnorm_forward_vec_kernel<2>, grid, block, 0, st, p);
    else if (vec && chunks == 3) hipLaunchKernelGGL(rmsnorm_forward_vec_kernel<3>, grid, block, 0, st, p);
    else if (vec && chunks == 4) hipLaunchKernelGGL(rmsnorm_forward_vec_kernel<4>, grid, block, 0, st, p);
    else if (chunks <= kRmsMaxChunks)
      hipLaunchKernelGGL(rmsnorm_forward_kernel<true>, dim3((unsigned)p.rows), dim3(kCtxThreads), 0, st, p);
    else
      hipLaunchKernelGGL(rmsnorm_forward_kernel<false>, dim3((unsigned)p.rows), dim3(kCtxThreads), 0, st, p);
    return hipGetLastError();
  }
  // no rows: nothing is read (the other pointers may be NULL); summing zero parts writes dw = 0
  const int n_parts = p.rows > 0 ? p.n_parts : 0;
  const int bwd_chunks = (p.ng + kBwdChunkGroups - 1) / kBwdChunkGroups;
  if (p.rows > 0 && bwd_chunks <= kBwdMaxChunks) {
    const dim3 grid((unsigned)p.n_parts), block(kBwdThreads);
    const bool vec = p.vec_ok && p.vec_w && p.cols % kValsPerLane == 0;
    const dim3 pair(2 * kTeamThreads);
    if (vec && p.ng <= kTeamGroups) {
      hipLaunchKernelGGL((rmsnorm_backward_pair_kernel<1>), grid, pair, 0, st, p);
    } else if (vec && p.ng <= 2 * kTeamGroups) {
      hipLaunchKernelGGL((rmsnorm_backward_pair_kernel<2>), grid, pair, 0, st, p);
    } else if (vec && p.ng <= kTeamMaxChunks * kTeamGroups) {
      hipLaunchKernelGGL((rmsnorm_backward_pair_kernel<3>), grid, pair, 0, st, p);
    } else if (bwd_chunks == 1) {
      hipLaunchKernelGGL((rmsnorm_backward_row_kernel<1, false>), grid, block, 0, st, p);
    } else {
      if (vec) hipLaunchKernelGGL((rmsnorm_backward_row_kernel<2, true>), grid, block, 0, st, p);
      else hipLaunchKernelGGL((rmsnorm_backward_row_kernel<2, false>), grid, block, 0, st, p);
    }
  } else if (p.rows > 0) {
    hipLaunchKernelGGL(rmsnorm_rowdot_kernel, dim3((unsigned)p.rows), dim3(kCtxThreads), 0, st, p);
    hipLaunchKernelGGL(rmsnorm_dx_dw_kernel, dim3((unsigned)chunks, (unsigned)p.n_parts),
                       dim3(kCtxThreads), 0, st, p);
  }
  hipLaunchKernelGGL(rmsnorm_dw_kernel, dim3((unsigned)((p.cols + kDwCols - 1) / kDwCols)),
                     dim3(kDwCols * kDwSlices), 0, st, p.dw_parts,
                     n_parts, p.cols, p.dw);
  return hipGetLastError();
}

hipError_t launch_glu(const GluParams& p, bool backward, hipStream_t st) {
  if (p.n_groups == 0) return hipSuccess;
  const int64_t threads = p.n_groups * kLanesPerGroup;
  const unsigned grid = (unsigned)((threads + kCtxThreads - 1) / kCtxThreads);
  const bool vec = p.vec_ok && p.cols % kValsPerLane == 0;
  if (backward) {
    if (vec) hipLaunchKernelGGL(glu_backward_vec_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
    else hipLaunchKernelGGL(glu_backward_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
  } else {
    if (vec) hipLaunchKernelGGL(glu_forward_vec_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
    else hipLaunchKernelGGL(glu_forward_kernel, dim3(grid), dim3(kCtxThreads), 0, st, p);
  }
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
