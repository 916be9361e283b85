// Host-visible launch interface between the C ABI layer and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fq {

struct QuantParams {
  const uint16_t* x;   // bf16 bits, row-major [rows, ld]
  int rows, cols;
  int64_t ld;
  int nbr, nbc;        // scale / mask / slot grid: ceil(rows / group) x ceil(cols / group)
  int group;           // quantization group edge: 128, or 64 / 32 (plain block INT8 only)
  int vec_ok;          // base 16-byte aligned and ld % 8 == 0: full blocks use 16-byte loads
  int crit;
  int stochastic;      // 1: stochastic rounding with `seed` (crit must be 0)
  uint64_t seed;
  float theta;
  int topk;            // crit 5: number of blocks that fall back (largest abs-max first)
  int capacity;
  int8_t* codes;
  int8_t* codes_t;     // nullptr: no transposed copies
  float* scales;
  uint8_t* mask;
  int32_t* fb_count_base;  // the tensor's counter buffer (groups < 128: cleared, nothing counted)
  int32_t* fb_count;       // live slot counter of this call (zero on entry)
  int32_t* fb_count_next;  // counter of the next call: cleared by this call
  int32_t* fb_groups_done;       // groups of 32 blocks whose decisions are all recorded (zero between calls)
  unsigned long long* fb_words;  // per group: decided bits | flagged bits << 32 (zero between calls)
  int clear_both;          // first use of the tensor (or empty input): clear all counters first
  int32_t* fb_list;
  int32_t* fb_slot;
  int8_t* res_codes;
  int8_t* res_codes_t;
  float* res_scales;
};

// The GEMM always runs in "NT on tile-order operands" form: operand A' has
// nib x nkb blocks, B' has njb x nkb blocks, block (i,k) at (i*nkb + k)*16384.
// Scales / slots of the stored matrices are reached through strides so that a
// transposed use (block (i,k) of A' = stored block (k,i)) needs no copy.
struct GemmParams {
  const int8_t* a_codes;
  const int8_t* a_res;        // residual slots (layout matching a_codes' orientation) or nullptr
  const float* a_scales;
  const float* a_res_scales;
  const int32_t* a_slot;      // nullptr: A has no fallback
  int a_si, a_sk;             // strides of block (i,k) in a_scales / a_slot
  const int8_t* b_codes;
  const float* b_scales;
  int b_sj, b_sk;
  void* c;                    // [M, ldc] fp32 / bf16, or int32 in debug mode
  int64_t ldc;
  int M, N;                   // valid output extent
  int nib, njb, nkb;
  int out_bf16;
  int vec_ok;                 // C base and row pitch allow 16-byte stores
  int n_main, main_tj, tail_tj;   // tile plan, filled in by launch_gemm
  int group;                  // quantization group edge (128, 64, 32)
  int a_ni, a_nk, b_nj;       // extents of the scale grids along i, k (A) and j (B), in groups
  int biased;                 // tolerance variant: biased INT32 accumulation (gemm_biased_kernel)
  int debug_k;                // debug mode: the single k-block (k-group) to evaluate
  int debug_residual;         // debug mode: 0 main term, 1 residual term
};

// 1 x 128 group INT10 context compression (quantize: x -> packed, scales;
// dequantize: packed, scales -> out).
constexpr int kCtxGroup = 128;
constexpr int kCtxGroupBytes = 160;
struct CtxParams {
  const uint16_t* x;   // bf16 bits, row-major [rows, ld]        (quantize)
  int64_t ld;
  uint16_t* out;       // bf16 bits, row-major [rows, ldo]       (dequantize)
  int64_t ldo;
  uint8_t* packed;     // [rows*ng][160]
  float* scales;       // [rows*ng]
  int cols, ng;
  int64_t n_groups;    // rows * ng
  int vec_ok;          // the bf16 side allows 16-byte accesses
};

// SiLU-gated linear unit with fused INT10 contexts (forward: x1, x2 -> y, contexts; backward:
// dy, contexts -> dx1, dx2).  All bf16 matrices are row-major [rows, pitch].
struct GluParams {
  const uint16_t* x1;
  const uint16_t* x2;
  int64_t ld;          // pitch of x1 and x2
  uint16_t* y;
  int64_t ldy;
  const uint16_t* dy;
  int64_t ld_dy;
  uint16_t* dx1;
  uint16_t* dx2;
  int64_t ldo;         // pitch of dx1 and dx2
  uint8_t* packed1;
  float* scales1;
  uint8_t* packed2;
  float* scales2;
  int cols, ng;
  int64_t n_groups;
  int vec_ok;          // every bf16 matrix of the call allows 16-byte accesses
};

// RMS normalization with a fused INT10 context (forward: x, w -> y, rstd, context; backward:
// dy, context, rstd, w -> dx, dw through dw_parts [n_parts, cols]).
struct RmsParams {
  const uint16_t* x;   // forward input [rows, ld]
  int64_t ld;
  const uint16_t* w;   // gain [cols] bf16
  uint16_t* y;
  int64_t ldy;
  float* rstd;         // [rows]: written by forward, read by backward
  float eps;
  const uint16_t* dy;
  int64_t ld_dy;
  uint16_t* dx;
  int64_t ldo;
  float* dw;           // [cols]
  float* dw_parts;     // [n_parts, cols] workspace
  float* row_mean;     // [rows] workspace: mean over the row of g * xh
  int n_parts;
  uint8_t* packed;
  float* scales;
  int64_t rows;
  int cols, ng;
  int vec_ok;          // the [rows, pitch] bf16 matrices of the call allow 16-byte accesses
  int vec_w;           // so does w
};

hipError_t launch_quantize(const QuantParams& p, hipStream_t st);
hipError_t launch_untile(const int8_t* tiled, int rows, int cols, int8_t* dense, hipStream_t st);
hipError_t launch_gemm(const GemmParams& p, bool debug, hipStream_t st);
// groups of 32 / 64 (and the plain 128 kernel): fq_group.hip
hipError_t launch_quantize_group(const QuantParams& p, hipStream_t st);
hipError_t launch_gemm_group(const GemmParams& p, bool debug, hipStream_t st);
// out = {workgroups with 2x2-block tiles, tile columns they cover, 1x3-block tile columns};
// cus <= 0: the current device's compute units (or FQ_GEMM_CUS).
void gemm_tile_plan(int nib, int njb, int cus, int out[3]);
hipError_t launch_rmsnorm(const RmsParams& p, bool backward, hipStream_t st);
hipError_t launch_glu(const GluParams& p, bool backward, hipStream_t st);
hipError_t launch_ctx(const CtxParams& p, bool dequantize, hipStream_t st);

}  // namespace fq
