// Fallback block GEMM on the gfx950 INT8 matrix cores.
//
// Paper: Sec. 4.2 Eq. (1) (INT8 x INT8 -> INT32 block product, dequantized by
// a^A a^B, FP32 accumulator), Sec. 4.3 Alg. 1 (k-loop on chip; for a flagged
// A block a second INT8 product with the residual codes against the same B
// block), Sec. 4.5 / App. C (the GEMM tile need not equal the quantization
// block).
//
// Shape of the kernel (differs from the paper's 128^3 CUDA tile on purpose):
//   - workgroup = 8 wavefronts (2 per SIMD), output tile 256 x 256 = 2 x 2
//     quantization blocks.  Wavefront (h, jq) owns rows [64h, 64h+64) of BOTH
//     i-blocks and the 64-column quarter jq of the tile: 4 x 2 sub-tiles of
//     32 x 32, 128 FP32 accumulators per lane in architectural VGPRs (the
//     vector ALU cannot read accumulation registers, so the accumulators it
//     updates must not live there);
//   - the k-loop runs over "items": the main product of k-block k and, when
//     one of the tile's two A blocks is flagged at k, a residual item right
//     after it.  A and B operands sit in two independent double-buffered LDS
//     rings (2 x 32 KiB each): an item always brings a new A pair (codes or
//     residual codes), a new B pair only when k advances, so the residual
//     product re-uses the B blocks already on chip exactly as Alg. 1 says.
//     Because every wavefront spans both i-blocks, a residual item costs each
//     wavefront work in proportion to the number of flagged blocks: the
//     overhead is proportional to the fallback rate;
//   - operands reach LDS by direct global->LDS 16-byte loads (blocks are stored
//     in operand order, see fq.h), one barrier per item;
//   - per 32 x 32 sub-tile: 4 v_mfma_i32_32x32x32_i8 (K = 128) into an INT32
//     tile, then one convert + one FMA per element folds it into the FP32
//     accumulators with the scalar scale of that block pair.
// The accumulation order per output element is exactly Alg. 1's (k ascending,
// main term then residual term), so results match a sequential evaluation
// bit for bit.
#include "fq_device.h"
#include "fq_kernels.h"

namespace fq {

namespace {

constexpr int kThreads = 512;
constexpr int kRingBytes = 2 * kBlockBytes;     // one A pair or one B pair
constexpr int kLdsBytes = 4 * kRingBytes;       // A ring x2, B ring x2 = 128 KiB

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

// One wavefront copies 8 KiB (8 fragments) global -> LDS with direct loads.
__device__ inline void stage_half_block(const int8_t* src, int8_t* lds_dst, int lane) {
#pragma unroll
  for (int f = 0; f < 8; ++f) {
    __builtin_amdgcn_global_load_lds((gbl_void*)(src + f * kFragBytes + lane * 16),
                                     (lds_void*)(lds_dst + f * kFragBytes), 16, 0, 0);
  }
}

__device__ inline v4i lds_frag(const int8_t* blk, int rg, int ks, int lane) {
  return *reinterpret_cast<const v4i*>(blk + ((rg * 4 + ks) * 64 + lane) * 16);
}

}  // namespace

template <bool kDebug>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const a_ring = lds;                   // [2][2 blocks]
  int8_t* const b_ring = lds + 2 * kRingBytes;  // [2][2 blocks]

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = w >> 2, jq = w & 3;

  // ---- tile of this workgroup; out-of-range blocks repeat the last valid one (never stored)
  const int tiles_j = (p.njb + 1) >> 1;
  const int ti = blockIdx.x / tiles_j, tj = blockIdx.x - ti * tiles_j;
  const int ib0 = ti * 2, ib1 = min(ti * 2 + 1, p.nib - 1);
  const int jb0 = tj * 2, jb1 = min(tj * 2 + 1, p.njb - 1);
  const int jb = (jq >> 1) ? jb1 : jb0;   // the j-block this wave multiplies with

  // ---- what this wave stages: waves 0-3 the A pair, waves 4-7 the B pair, 8 KiB each
  const bool stage_a = w < 4;
  const int sblk = (w & 2) ? (stage_a ? ib1 : jb1) : (stage_a ? ib0 : jb0);
  const int shalf = (w >> 1) & 1;            // which block of the pair
  const int soff = shalf * kBlockBytes + (w & 1) * (kBlockBytes / 2);
  const int8_t* const smain = (stage_a ? p.a_codes : p.b_codes) +
                              (int64_t)sblk * p.nkb * kBlockBytes + (w & 1) * (kBlockBytes / 2);

  // Scales and slots are read-only for the whole kernel: reading them through the constant
  // address space makes them scalar loads, which do not share a counter with the LDS loads.
  typedef const __attribute__((address_space(4))) float cfloat;
  typedef const __attribute__((address_space(4))) int32_t cint;
  cfloat* const a_sc = (cfloat*)p.a_scales;
  cfloat* const b_sc = (cfloat*)p.b_scales;
  cfloat* const r_sc = (cfloat*)p.a_res_scales;
  cint* const a_sl = (cint*)p.a_slot;
  const bool has_fb = p.a_slot != nullptr;
  const int ia0 = ib0 * p.a_si, ia1 = ib1 * p.a_si, ibj = jb * p.b_sj;

  float acc[4][2][16];
#pragma unroll
  for (int si = 0; si < 4; ++si)
#pragma unroll
    for (int sj = 0; sj < 2; ++sj)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[si][sj][r] = 0.0f;
  bool poison0 = false, poison1 = false;

  const int k_begin = kDebug ? p.debug_k : 0;
  const int k_end = kDebug ? p.debug_k + 1 : p.nkb;
  if (k_begin >= k_end) goto store;   // empty contraction: all zeros

  {
  // prologue: main item of the first k-block into ring slot 0
  stage_half_block(smain + (int64_t)k_begin * kBlockBytes,
                   (stage_a ? a_ring : b_ring) + soff, lane);

  // scalars of the current k-block, fetched one item ahead
  int slot0 = has_fb ? a_sl[ia0 + k_begin * p.a_sk] : -1;
  int slot1 = has_fb ? a_sl[ia1 + k_begin * p.a_sk] : -1;
  float sa0 = a_sc[ia0 + k_begin * p.a_sk], sa1 = a_sc[ia1 + k_begin * p.a_sk];
  float sb = b_sc[ibj + k_begin * p.b_sk];
  float rs0 = 0.0f, rs1 = 0.0f;

  int k = k_begin;
  int res = 0;     // 0: main item, 1: residual item of k
  int t = 0;       // item counter: A ring slot = t & 1
  while (k < k_end) {
    // this wave's direct-to-LDS loads must have landed before the barrier publishes them
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    const int bsel = (k - k_begin) & 1;
    const int asel = t & 1;

    // ---- prefetch the next item
    const bool next_res = !res && (slot0 >= 0 || slot1 >= 0);
    const int next_k = next_res ? k : k + 1;
    if (next_res) {
      if (stage_a) {
        const int s = shalf ? slot1 : slot0;
        if (s >= 0)
          stage_half_block(p.a_res + (int64_t)s * kBlockBytes + (w & 1) * (kBlockBytes / 2),
                           a_ring + (asel ^ 1) * kRingBytes + soff, lane);
      }
      if (slot0 >= 0) rs0 = r_sc[slot0];
      if (slot1 >= 0) rs1 = r_sc[slot1];
    } else if (next_k < k_end) {
      stage_half_block(smain + (int64_t)next_k * kBlockBytes,
                       (stage_a ? a_ring + (asel ^ 1) * kRingBytes
                                : b_ring + (bsel ^ 1) * kRingBytes) + soff, lane);
    }
    // scalars of k-block k+1 (used from the next main item on)
    int nslot0 = -1, nslot1 = -1;
    float nsa0 = 0.0f, nsa1 = 0.0f, nsb = 0.0f;
    if (!next_res && next_k < k_end) {
      if (has_fb) {
        nslot0 = a_sl[ia0 + next_k * p.a_sk];
        nslot1 = a_sl[ia1 + next_k * p.a_sk];
      }
      nsa0 = a_sc[ia0 + next_k * p.a_sk];
      nsa1 = a_sc[ia1 + next_k * p.a_sk];
      nsb = b_sc[ibj + next_k * p.b_sk];
    }

    // ---- scales of this item (wave-uniform scalars)
    float s0, s1;
    bool do0 = true, do1 = true;
    if (!res) {
      s0 = sa0 * sb;
      s1 = sa1 * sb;
      poison0 |= slot0 == -2;
      poison1 |= slot1 == -2;
    } else {
      do0 = slot0 >= 0;
      do1 = slot1 >= 0;
      s0 = rs0 * sb;
      s1 = rs1 * sb;
    }
    const bool record = !kDebug || (res == p.debug_residual);

    const int8_t* la = a_ring + asel * kRingBytes;
    const int8_t* lb = b_ring + bsel * kRingBytes + (jq >> 1) * kBlockBytes;

    v4i bq[2][4];
#pragma unroll
    for (int sj = 0; sj < 2; ++sj)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) bq[sj][ks] = lds_frag(lb, 2 * (jq & 1) + sj, ks, lane);

#pragma unroll
    for (int si = 0; si < 4; ++si) {
      const bool active = (si < 2) ? do0 : do1;
      if (!active) continue;   // wave-uniform
      const float s = (si < 2) ? s0 : s1;
      const int8_t* lablk = la + (si >> 1) * kBlockBytes;
      v4i aq[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) aq[ks] = lds_frag(lablk, 2 * h + (si & 1), ks, lane);
#pragma unroll
      for (int sj = 0; sj < 2; ++sj) {
        v16i P = {0};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          P = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq[ks], bq[sj][ks], P, 0, 0, 0);
        if (record) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            if (kDebug) acc[si][sj][r] = __int_as_float(P[r]);
            else acc[si][sj][r] = __builtin_fmaf((float)P[r], s, acc[si][sj][r]);
          }
        }
      }
    }

    // ---- advance
    if (next_res) {
      res = 1;
    } else {
      res = 0;
      k = k + 1;
      slot0 = nslot0; slot1 = nslot1; sa0 = nsa0; sa1 = nsa1; sb = nsb;
    }
    ++t;
  }
  }

store:
  // ---- store: sub-tile (si, sj), register r -> row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
  if (tj * 2 + (jq >> 1) >= p.njb) return;
  const int col_base = jb * kBlock + (jq & 1) * 64 + (lane & 31);
#pragma unroll
  for (int si = 0; si < 4; ++si) {
    if ((si >> 1) && ti * 2 + 1 >= p.nib) continue;
    const int ib = (si >> 1) ? ib1 : ib0;
    const bool poison = !kDebug && ((si >> 1) ? poison1 : poison0);
    const int row_base = ib * kBlock + h * 64 + (si & 1) * 32 + 4 * (lane >> 5);
#pragma unroll
    for (int sj = 0; sj < 2; ++sj) {
      const int col = col_base + sj * 32;
      if (col >= p.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row_base + 8 * (r >> 2) + (r & 3);
        if (row >= p.M) continue;
        // a flagged block whose residual found no slot cannot be computed: poison its rows
        const float v = poison ? __int_as_float(0x7FC00000) : acc[si][sj][r];
        const int64_t off = (int64_t)row * p.ldc + col;
        if (!kDebug && p.out_bf16)
          reinterpret_cast<uint16_t*>(p.c)[off] = (uint16_t)float_to_bf16_bits(v);
        else
          reinterpret_cast<float*>(p.c)[off] = v;
      }
    }
  }
}

hipError_t launch_gemm(const GemmParams& p, bool debug, hipStream_t st) {
  const int tiles = ((p.nib + 1) / 2) * ((p.njb + 1) / 2);
  if (tiles == 0) return hipSuccess;
  static bool attr_set[2] = {false, false};
  auto kern = debug ? gemm_kernel<true> : gemm_kernel<false>;
  if (!attr_set[debug]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set[debug] = true;
  }
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(kThreads), kLdsBytes, st, p);
  return hipGetLastError();
}

}  // namespace fq
