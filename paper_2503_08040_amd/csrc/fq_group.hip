// Block INT8 quantization and GEMM with quantization groups smaller than 128 x 128.
//
// Paper: Sec. 4.5 and Fig. 1b (the throughput of an INT8 block GEMM falls with the group size,
// because every group boundary along K costs a dequantization on the general-purpose ALUs; the
// paper therefore moves from 32 x 32 to 128 x 128), Sec. 4.2 Eq. (1) (the block GEMM itself),
// Sec. 3.1 (per-group scale a = max|G| / 127 and round-to-nearest codes).
//
// These kernels make the group size g in {32, 64} a real, tested path (plain block INT8, no
// fallback: the paper's fallback scheme is defined on its 128 x 128 blocks), so that the curve
// of Fig. 1b can be measured on this GPU.  Codes keep the storage of the 128 path (16 KiB
// blocks in operand order, see fq.h); only the scale / mask / slot grids become finer
// (ceil(rows/g) x ceil(cols/g)).  The GEMM is a plain 128 x 128-tile kernel: four wavefronts,
// each 32 rows x 128 columns; B blocks staged through LDS (double-buffered direct loads), A
// fragments straight from global memory; per 32 x 32 sub-tile and k-group g/32
// v_mfma_i32_32x32x32_i8 into an INT32 tile, then one convert + one FMA per element with the
// scale pair of that group.  The accumulation order per output element is Eq. (1)'s (k-groups
// ascending), so results match the sequential evaluation bit for bit.  The same kernel also
// runs g = 128 (for the sweep: one kernel, three group sizes); the tuned g = 128 path of
// fq_gemm.hip is what fq_gemm uses for block 128.
#include "fq_device.h"
#include "fq_kernels.h"

namespace fq {

namespace {

constexpr int kQThreads = 256;
constexpr int kGThreads = 256;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

// packed bf16 pair / code helpers (same register layout as the 128 quantizer: a thread holds
// rows rp + 32 pz, pz = 0..3, and 16 consecutive columns 16 cc .. 16 cc + 15)
__device__ inline float x_at(const v4i (&raw)[4][2], int pz, int e) {
  const uint32_t w = (uint32_t)raw[pz][e >> 3][(e & 7) >> 1];
  return __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
}

__device__ inline void load_rows(const QuantParams& p, int bi, int bk, int rp, int cc, v4i (&raw)[4][2]) {
  const int row0 = bi * kBlock, col0 = bk * kBlock + cc * 16;
  const bool inner = (row0 + kBlock <= p.rows) && (bk * kBlock + kBlock <= p.cols) && p.vec_ok;
  if (inner) {
#pragma unroll
    for (int pz = 0; pz < 4; ++pz) {
      const uint16_t* src = p.x + (int64_t)(row0 + pz * 32 + rp) * p.ld + col0;
      raw[pz][0] = *reinterpret_cast<const v4i*>(src);
      raw[pz][1] = *reinterpret_cast<const v4i*>(src + 8);
    }
  } else {
#pragma unroll
    for (int pz = 0; pz < 4; ++pz) {
      const int r = row0 + pz * 32 + rp;
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        uint32_t w = 0;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int c = col0 + 2 * d + hh;
          if (r < p.rows && c < p.cols) w |= (uint32_t)p.x[(int64_t)r * p.ld + c] << (16 * hh);
        }
        raw[pz][d >> 2][d & 3] = (int)w;
      }
    }
  }
}

}  // namespace

// One workgroup per 128 x 128 region = (128/kG)^2 quantization groups.  Sec. 3.1 per group.
template <int kG, bool kWantT>
__global__ __launch_bounds__(kQThreads, 2) void quantize_group_kernel(QuantParams p) {
  constexpr int kS = kBlock / kG;                  // groups per region edge: 2 or 4
  __shared__ unsigned amax_bits[kS * kS];          // max |G| per group (bit patterns of floats >= 0)
  __shared__ __attribute__((aligned(16))) int8_t img[kWantT ? kBlockBytes : 16];
  const int blk = blockIdx.x;
  const int nbc128 = (p.cols + kBlock - 1) / kBlock;
  const int bi = blk / nbc128, bk = blk - bi * nbc128;
  const int t = threadIdx.x, cc = t & 7, rp = t >> 3;
  if (t < kS * kS) amax_bits[t] = 0u;
  v4i raw[4][2];
  load_rows(p, bi, bk, rp, cc, raw);
  __syncthreads();
  // group of (row rp + 32 pz, columns 16 cc ..): row group (rp + 32 pz) / kG, column group 16 cc / kG
  const int gc = (16 * cc) / kG;
#pragma unroll
  for (int pz = 0; pz < 4; ++pz) {
    float m = 0.0f;
#pragma unroll
    for (int e = 0; e < 16; ++e) m = fmaxf(m, fabsf(x_at(raw, pz, e)));
    const int gr = (rp + 32 * pz) / kG;
    atomicMax(&amax_bits[gr * kS + gc], __float_as_uint(m));
  }
  __syncthreads();
  v4i q[4];
#pragma unroll
  for (int pz = 0; pz < 4; ++pz) {
    const int gr = (rp + 32 * pz) / kG;
    const float amax = __uint_as_float(amax_bits[gr * kS + gc]);
    const float a = __fdiv_rn(amax, 127.0f);
    const float a_rcp = fast_recip(a);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float k = (a == 0.0f) ? 0.0f : rint_quotient(x_at(raw, pz, e), a, a_rcp, 127.0f);
      const int code = (int)k & 0xFF;
      if ((e & 3) == 0) q[pz][e >> 2] = code;
      else q[pz][e >> 2] |= code << (8 * (e & 3));
    }
  }
  int8_t* cdst = p.codes + (int64_t)blk * kBlockBytes;
#pragma unroll
  for (int pz = 0; pz < 4; ++pz)
    *reinterpret_cast<v4i*>(cdst + tile_offset(pz * 32 + rp, cc * 16)) = q[pz];
  if (kWantT) {
    const int nbr128 = (p.rows + kBlock - 1) / kBlock;
#pragma unroll
    for (int pz = 0; pz < 4; ++pz) {
      const int r = pz * 32 + rp;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        img[tile_offset(cc * 16 + e, r)] = (int8_t)((uint32_t)q[pz][e >> 2] >> (8 * (e & 3)));
    }
    __syncthreads();
    const v4i* src = reinterpret_cast<const v4i*>(img);
    v4i* out = reinterpret_cast<v4i*>(p.codes_t + ((int64_t)bk * nbr128 + bi) * kBlockBytes);
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i * kQThreads + t] = src[i * kQThreads + t];
  }
  // per-group outputs (groups of this region that exist in the matrix)
  if (t < kS * kS) {
    const int gr = bi * kS + t / kS, gcol = bk * kS + t % kS;
    if (gr < p.nbr && gcol < p.nbc) {
      const int at = gr * p.nbc + gcol;
      p.scales[at] = __fdiv_rn(__uint_as_float(amax_bits[t]), 127.0f);
      p.mask[at] = 0;
      p.fb_slot[at] = -1;
    }
  }
}

// Block GEMM of Eq. (1) for group size kG: one workgroup per 128 x 128 output tile.
template <int kG>
__global__ __launch_bounds__(kGThreads, 2) void gemm_group_kernel(GemmParams p) {
  constexpr int kS = kBlock / kG;        // k-groups per 128-deep block
  constexpr int kM = kG / 32;            // MFMAs (K = 32) per group
  __shared__ __attribute__((aligned(1024))) int8_t bbuf[2][kBlockBytes];
  const int ib = blockIdx.x / p.njb, jb = blockIdx.x - ib * p.njb;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  typedef const __attribute__((address_space(4))) float cfloat;
  cfloat* const a_sc = (cfloat*)p.a_scales;
  cfloat* const b_sc = (cfloat*)p.b_scales;
  // group rows / columns of this wave's rows and of each 32-column sub-tile, clamped to the
  // grids (groups beyond the matrix hold zero codes, any scale will do)
  const int gi = min((ib * kBlock + 32 * w) / kG, p.a_ni - 1);
  int gj[4];
#pragma unroll
  for (int sj = 0; sj < 4; ++sj) gj[sj] = min((jb * kBlock + 32 * sj) / kG, p.b_nj - 1);

  float acc[4][16];
#pragma unroll
  for (int sj = 0; sj < 4; ++sj)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[sj][r] = 0.0f;

  const int8_t* const arow = p.a_codes + (int64_t)ib * p.nkb * kBlockBytes;
  const int8_t* const brow = p.b_codes + (int64_t)jb * p.nkb * kBlockBytes;
  // this wave's quarter of a B block: 4 KiB = 4 direct 16-byte-per-lane loads
  auto stage_b = [&](int kb, int buf) {
    const int8_t* src = brow + (int64_t)kb * kBlockBytes + w * 4096;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((gbl_void*)(src + i * 1024 + lane * 16),
                                       (lds_void*)(&bbuf[buf][w * 4096 + i * 1024]), 16, 0, 0);
  };
  auto load_a = [&](int kb, v4i (&a)[4]) {
    const int8_t* src = arow + (int64_t)kb * kBlockBytes;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      a[ks] = *reinterpret_cast<const v4i*>(src + ((w * 4 + ks) * 64 + lane) * 16);
  };

  v4i a_cur[4], a_nxt[4];
  if (p.nkb > 0) {
    stage_b(0, 0);
    load_a(0, a_cur);
  }
  for (int kb = 0; kb < p.nkb; ++kb) {
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0): this wave's share of B block kb landed
    __syncthreads();                       // ... and everyone's; buffer (kb + 1) & 1 is free
    if (kb + 1 < p.nkb) {
      stage_b(kb + 1, (kb + 1) & 1);
      load_a(kb + 1, a_nxt);
    }
    const int8_t* const bb = bbuf[kb & 1];
#pragma unroll
    for (int g = 0; g < kS; ++g) {
      const int kg = min(kb * kS + g, p.a_nk - 1);
      const float sa = a_sc[gi * p.a_si + kg * p.a_sk];
#pragma unroll
      for (int sj = 0; sj < 4; ++sj) {
        v16i P = {0};
#pragma unroll
        for (int m = 0; m < kM; ++m) {
          const int ks = g * kM + m;
          const v4i b = *reinterpret_cast<const v4i*>(bb + ((sj * 4 + ks) * 64 + lane) * 16);
          P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_cur[ks], b, P, 0, 0, 0);
        }
        const float s = sa * b_sc[gj[sj] * p.b_sj + kg * p.b_sk];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[sj][r] = __builtin_fmaf((float)P[r], s, acc[sj][r]);
      }
    }
    if (kb + 1 < p.nkb) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) a_cur[ks] = a_nxt[ks];
    }
  }
  // store: lane l holds column l % 32 and rows 8 (r / 4) + 4 (l / 32) + r % 4 of each sub-tile
#pragma unroll
  for (int sj = 0; sj < 4; ++sj) {
    const int col = jb * kBlock + sj * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = ib * kBlock + w * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row < p.M && col < p.N) {
        if (p.out_bf16)
          reinterpret_cast<uint16_t*>(p.c)[(int64_t)row * p.ldc + col] = (uint16_t)float_to_bf16_bits(acc[sj][r]);
        else
          reinterpret_cast<float*>(p.c)[(int64_t)row * p.ldc + col] = acc[sj][r];
      }
    }
  }
}

// INT32 product of one k-group (inspection / tests): group debug_k of size p.group.
__global__ __launch_bounds__(256) void partials_group_kernel(GemmParams p) {
  const int ib = blockIdx.x / p.njb, jb = blockIdx.x - ib * p.njb;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int k0 = p.debug_k * p.group;                   // first contraction index of the group
  const int kb = k0 / kBlock, ks0 = (k0 % kBlock) / 32, nks = p.group / 32;
  const int8_t* ablk = p.a_codes + ((int64_t)ib * p.nkb + kb) * kBlockBytes;
  const int8_t* bblk = p.b_codes + ((int64_t)jb * p.nkb + kb) * kBlockBytes;
  int32_t* const out = reinterpret_cast<int32_t*>(p.c);
  for (int sj = 0; sj < 4; ++sj) {
    v16i P = {0};
    if (!p.debug_residual) {
      for (int ks = ks0; ks < ks0 + nks; ++ks) {
        const v4i a = *reinterpret_cast<const v4i*>(ablk + ((w * 4 + ks) * 64 + lane) * 16);
        const v4i b = *reinterpret_cast<const v4i*>(bblk + ((sj * 4 + ks) * 64 + lane) * 16);
        P = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, P, 0, 0, 0);
      }
    }
    const int col = jb * kBlock + sj * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = ib * kBlock + w * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row < p.M && col < p.N) out[(int64_t)row * p.ldc + col] = P[r];
    }
  }
}

// Clears the slot counters of a tensor quantized without fallback.
__global__ void clear_fb_counters_kernel(int32_t* counters, int n) {
  if ((int)threadIdx.x < n) counters[threadIdx.x] = 0;
}

hipError_t launch_quantize_group(const QuantParams& p, hipStream_t st) {
  hipLaunchKernelGGL(clear_fb_counters_kernel, dim3(1), dim3(64), 0, st, p.fb_count_base, 4);
  const int nb128 = ((p.rows + kBlock - 1) / kBlock) * ((p.cols + kBlock - 1) / kBlock);
  if (nb128 == 0) return hipGetLastError();
  const dim3 grid(nb128), block(kQThreads);
  if (p.group == 32) {
    if (p.codes_t) hipLaunchKernelGGL((quantize_group_kernel<32, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((quantize_group_kernel<32, false>), grid, block, 0, st, p);
  } else {
    if (p.codes_t) hipLaunchKernelGGL((quantize_group_kernel<64, true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((quantize_group_kernel<64, false>), grid, block, 0, st, p);
  }
  return hipGetLastError();
}

hipError_t launch_gemm_group(const GemmParams& p, bool debug, hipStream_t st) {
  if (p.nib == 0 || p.njb == 0) return hipSuccess;
  const dim3 grid(p.nib * p.njb);
  if (debug) {
    hipLaunchKernelGGL(partials_group_kernel, grid, dim3(256), 0, st, p);
  } else if (p.group == 32) {
    hipLaunchKernelGGL(gemm_group_kernel<32>, grid, dim3(kGThreads), 0, st, p);
  } else if (p.group == 64) {
    hipLaunchKernelGGL(gemm_group_kernel<64>, grid, dim3(kGThreads), 0, st, p);
  } else {
    hipLaunchKernelGGL(gemm_group_kernel<128>, grid, dim3(kGThreads), 0, st, p);
  }
  return hipGetLastError();
}

}  // namespace fq
