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
constexpr int kXcds = 8;      // accelerator complex dies, each with a private L2
constexpr int kGroupN = 4;    // tile columns per rasterization group
constexpr int kRingBytes = 2 * kBlockBytes;     // one A pair or one B pair
constexpr int kStagePitch = 72;                 // floats per row of the epilogue staging patch
constexpr int kStageBytesPerWave = 64 * kStagePitch * 4;
constexpr int kLdsBytes = 8 * kStageBytesPerWave;   // 144 KiB: covers the rings (A x2, B x2 = 128 KiB)
static_assert(kLdsBytes >= 4 * kRingBytes, "LDS must hold both operand rings");

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

// One wavefront copies 8 KiB (8 fragments) global -> LDS with direct loads.  `src` and
// `lds_dst` are wave-uniform; the per-lane part of the address is the 32-bit offset lane*16,
// so the loads use the scalar-base addressing form and need no 64-bit address registers.
__device__ inline void stage_half_block(const int8_t* src, int8_t* lds_dst, int lane) {
  const unsigned voff = (unsigned)lane * 16u;
  // make the uniformity of the base explicit (folds away when it is already scalar)
  const uint64_t a = reinterpret_cast<uint64_t>(src);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  src = reinterpret_cast<const int8_t*>(((uint64_t)hi << 32) | lo);
  // 4 loads share one base (global and LDS) and differ only in the instruction offset
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    gbl_void* g = (gbl_void*)(src + b * 4 * kFragBytes + voff);
    lds_void* l = (lds_void*)(lds_dst + b * 4 * kFragBytes);
    __builtin_amdgcn_global_load_lds(g, l, 16, 0 * kFragBytes, 0);
    __builtin_amdgcn_global_load_lds(g, l, 16, 1 * kFragBytes, 0);
    __builtin_amdgcn_global_load_lds(g, l, 16, 2 * kFragBytes, 0);
    __builtin_amdgcn_global_load_lds(g, l, 16, 3 * kFragBytes, 0);
  }
}

// two floats -> two bf16 (round-to-nearest-even) in one dword, low half first
__device__ inline int pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  f32x2 v = {a, b};
  return __builtin_bit_cast(int, __builtin_convertvector(v, bf16x2));
}

__device__ inline v4i lds_frag(const int8_t* blk, int rg, int ks, int lane) {
  return *reinterpret_cast<const v4i*>(blk + ((rg * 4 + ks) * 64 + lane) * 16);
}


// Empty volatile asm statements that take values as read-write register operands.  The
// compiler may not reorder volatile asm, so the instructions producing the operands stay
// before the statement and their consumers after it: this pins the source order of otherwise
// freely movable pure instructions (MFMA, convert, FMA) without emitting any code.
__device__ __forceinline__ void pin(v16i& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(float& a, float& b, float& c, float& d) {
  asm volatile("" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// Per-wavefront register state of the k-loop.
struct WaveState {
  float acc[4][2][16];   // FP32 accumulators: sub-tile (si, sj), 16 elements per lane
  v4i aq[2][4];          // A fragments (ks = 0..3) of two consecutive si: si uses aq[si & 1]
  v4i bq[2][4];          // B fragments of this wave's two column groups
  v16i P[2];             // INT32 tiles: sub-tile u accumulates into P[u & 1]
  float T[4];            // elements converted in the previous slot, waiting for their FMA
};

// The k-loop is one continuous software pipeline over sub-tiles ("units": u = 2*si + sj, 8 per
// item).  Unit u is 4 slots; slot g issues MFMA g (K = 32 of the 128) of unit u and, in the 32
// cycles the matrix core needs for it, 8 vector-ALU instructions that fold the finished INT32
// tile of unit u-1 into the FP32 accumulators: the 4 FMAs of the elements converted one slot
// earlier, then the 4 converts of elements 4g..4g+3.  An FMA never waits for its convert, and a
// convert reads an MFMA result that is at least 11 issue slots old, as the hardware requires.
// Fragment registers are refilled from LDS well before their next use: the A fragments of si+1
// are fetched into a second register buffer while si is being multiplied (LDS latency under
// load is several hundred cycles), and units 6 and 7 fetch the B fragments and the first A
// fragments of the NEXT item, so that no item starts with a burst of LDS reads.  Scheduling
// fences pin this order.
//   a_cur: A pair of the current item in LDS; a_nxt / b_nxt: A pair / B block of the next item.
//   s0, s1: scales of the current item's two i-blocks; sp: scale of the previous item's si = 3.
template <int u>
__device__ __forceinline__ void run_unit(WaveState& st, const int8_t* a_cur, const int8_t* a_nxt,
                                         const int8_t* b_nxt, int h, int jq, int lane, float s0,
                                         float s1, float sp) {
  constexpr int si = u >> 1, sj = u & 1;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    {
      const v16i z = {0};
      st.P[u & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(st.aq[si & 1][g], st.bq[sj][g],
                                                          g ? st.P[u & 1] : z, 0, 0, 0);
      // A fragments of the next si (of the next item for si = 3) go into the other aq buffer
      // a whole unit before their first use
      if (u < 6 && sj == 0)
        st.aq[(si + 1) & 1][g] =
            lds_frag(a_cur + ((si + 1) >> 1) * kBlockBytes, 2 * h + ((si + 1) & 1), g, lane);
      if (u == 6) {
        st.aq[0][g] = lds_frag(a_nxt, 2 * h, g, lane);
        st.bq[0][g] = lds_frag(b_nxt, 2 * (jq & 1), g, lane);
      }
      if (u == 7) st.bq[1][g] = lds_frag(b_nxt, 2 * (jq & 1) + 1, g, lane);
      pin(st.P[u & 1]);
    }
    __builtin_amdgcn_sched_barrier(0);   // MFMA first: its destination must not alias live tiles
    {
      // FMAs of the 4 elements converted in the previous slot (unit u-1, or u-2 for g = 0);
      // negative units are units 6, 7 of the previous item (si = 3)
      const int fu = g ? u - 1 : u - 2, fc = g ? g - 1 : 3;
      const int fsi = fu < 0 ? 3 : (fu >> 1), fsj = fu & 1;
      const float s = fu < 0 ? sp : (fsi < 2 ? s0 : s1);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        st.acc[fsi][fsj][4 * fc + i] = __builtin_fmaf(st.T[i], s, st.acc[fsi][fsj][4 * fc + i]);
      pin(st.acc[fsi][fsj][4 * fc], st.acc[fsi][fsj][4 * fc + 1], st.acc[fsi][fsj][4 * fc + 2],
          st.acc[fsi][fsj][4 * fc + 3]);
    }
    __builtin_amdgcn_sched_barrier(0);   // FMAs before converts
#pragma unroll
    for (int i = 0; i < 4; ++i) st.T[i] = (float)st.P[(u - 1) & 1][4 * g + i];
    pin(st.T[0], st.T[1], st.T[2], st.T[3]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Folds the last unit (si = 3, sj = 1) of the last item into the accumulators.
__device__ __forceinline__ void drain(WaveState& st, float s1) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int fsj = g ? 1 : 0, fc = g ? g - 1 : 3;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      st.acc[3][fsj][4 * fc + i] = __builtin_fmaf(st.T[i], s1, st.acc[3][fsj][4 * fc + i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) st.T[i] = (float)st.P[1][4 * g + i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) st.acc[3][1][12 + i] = __builtin_fmaf(st.T[i], s1, st.acc[3][1][12 + i]);
}

// Scalars of one k-block: residual slots and scales of the tile's two A blocks, scale of this
// wave's B block.
struct KRec {
  int slot0, slot1;
  float sa0, sa1, sb;
  float rs0, rs1;   // residual scales of the two A blocks (valid where the slot is >= 0)
};

}  // namespace

__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const a_ring = lds;                   // [2][2 blocks]
  int8_t* const b_ring = lds + 2 * kRingBytes;  // [2][2 blocks]
  constexpr bool kDebug = false;

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = w >> 2, jq = w & 3;

  // ---- tile of this workgroup; out-of-range blocks repeat the last valid one (never stored).
  // Workgroups are dealt to the 8 XCDs round-robin by id, and each XCD has its own L2.  Remap
  // ids so that one XCD works through a contiguous run of tiles, and order the tiles in groups
  // of kGroupN tile-columns walked row by row: the ~32 tiles resident on an XCD then form an
  // 8 x 4 patch that shares its A and B blocks through that L2.  Grouping by columns (not rows)
  // gives every XCD tiles from all tile-rows, so fallback blocks clustered in a few block-rows
  // (the worst case of Sec. 6.3) load the XCDs evenly.
  const int tiles_i = (p.nib + 1) >> 1, tiles_j = (p.njb + 1) >> 1;
  int ti, tj;
  {
    const int total = tiles_i * tiles_j;
    const int b = blockIdx.x, xcd = b % kXcds, l = b / kXcds;
    const int q = total / kXcds, rem = total % kXcds;
    const int L = xcd * q + min(xcd, rem) + l;
    const int group = kGroupN * tiles_i;
    const int g0 = (L / group) * kGroupN;
    const int gn = min(kGroupN, tiles_j - g0);
    const int within = L - (L / group) * group;
    tj = g0 + within % gn;
    ti = within / gn;
  }
  const int ib0 = ti * 2, ib1 = min(ti * 2 + 1, p.nib - 1);
  const int jb0 = tj * 2, jb1 = min(tj * 2 + 1, p.njb - 1);
  const int jb = (jq >> 1) ? jb1 : jb0;   // the j-block this wave multiplies with

  // ---- what this wave stages: waves 0-3 the A pair, waves 4-7 the B pair, 8 KiB each
  const bool stage_a = w < 4;
  const int shalf = (w >> 1) & 1;            // which block of the pair
  const int sblk = shalf ? (stage_a ? ib1 : jb1) : (stage_a ? ib0 : jb0);
  const int soff = shalf * kBlockBytes + (w & 1) * (kBlockBytes / 2);
  const int8_t* const smain = (stage_a ? p.a_codes : p.b_codes) +
                              (int64_t)sblk * p.nkb * kBlockBytes + (w & 1) * (kBlockBytes / 2);

  // Scales and slots are read-only for the whole kernel: reading them through the constant
  // address space makes them scalar loads, which do not share a counter with the vector loads.
  typedef const __attribute__((address_space(4))) float cfloat;
  typedef const __attribute__((address_space(4))) int32_t cint;
  cfloat* const a_sc = (cfloat*)p.a_scales;
  cfloat* const b_sc = (cfloat*)p.b_scales;
  cfloat* const r_sc = (cfloat*)p.a_res_scales;
  cint* const a_sl = (cint*)p.a_slot;
  const bool has_fb = p.a_slot != nullptr;
  const int ia0 = ib0 * p.a_si, ia1 = ib1 * p.a_si, ibj = jb * p.b_sj;
  const int nkb = p.nkb;

  auto load_rec = [&](int k) -> KRec {
    KRec r{-1, -1, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    if (k < nkb) {
      if (has_fb) {
        r.slot0 = a_sl[ia0 + k * p.a_sk];
        r.slot1 = a_sl[ia1 + k * p.a_sk];
      }
      r.sa0 = a_sc[ia0 + k * p.a_sk];
      r.sa1 = a_sc[ia1 + k * p.a_sk];
      r.sb = b_sc[ibj + k * p.b_sk];
    }
    return r;
  };
  // Residual scales depend on the slots, so they are fetched one step after the record itself:
  // by then the slots have arrived and the dependent load does not stall the wavefront.
  auto load_res_scales = [&](KRec& r) {
    if (r.slot0 >= 0) r.rs0 = r_sc[r.slot0];
    if (r.slot1 >= 0) r.rs1 = r_sc[r.slot1];
  };
  // Stages this wave's 8 KiB share of item (k, res) into ring slot `asel` (A) / k & 1 (B).
  auto stage_item = [&](int k, int res, const KRec& r, int asel, bool new_b) {
    if (stage_a) {
      const int8_t* src;
      if (res) {
        const int s = shalf ? r.slot1 : r.slot0;
        if (s < 0) return;   // unflagged half: nothing to bring (its scale will be zero)
        src = p.a_res + (int64_t)s * kBlockBytes + (w & 1) * (kBlockBytes / 2);
      } else {
        src = smain + (int64_t)k * kBlockBytes;
      }
      stage_half_block(src, a_ring + asel * kRingBytes + soff, lane);
    } else if (new_b) {
      stage_half_block(smain + (int64_t)k * kBlockBytes, b_ring + (k & 1) * kRingBytes + soff, lane);
    }
  };

  WaveState st;
  float (&acc)[4][2][16] = st.acc;
#pragma unroll
  for (int si = 0; si < 4; ++si)
#pragma unroll
    for (int sj = 0; sj < 2; ++sj)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.acc[si][sj][r] = 0.0f;
  bool poison0 = false, poison1 = false;
  if (nkb <= 0) goto store;   // empty contraction: all zeros

  {
    // ---- prologue: items 0 and 1 into the two ring slots
    // records are fetched two k-blocks ahead so that no scalar load is waited for in the loop
    KRec r0 = load_rec(0), r1 = load_rec(1), r2 = load_rec(2);
    int k = 0, res = 0, t = 0;
    stage_item(0, 0, r0, 0, true);
    {
      const bool n1res = r0.slot0 >= 0 || r0.slot1 >= 0;
      if (n1res) stage_item(0, 1, r0, 1, false);
      else if (1 < nkb) stage_item(1, 0, r1, 1, true);
    }
    load_res_scales(r0);
    load_res_scales(r1);
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0): this wave's direct-to-LDS loads landed
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      st.aq[0][g] = lds_frag(a_ring, 2 * h, g, lane);
      st.bq[0][g] = lds_frag(b_ring + (jq >> 1) * kBlockBytes, 2 * (jq & 1), g, lane);
      st.bq[1][g] = lds_frag(b_ring + (jq >> 1) * kBlockBytes, 2 * (jq & 1) + 1, g, lane);
    }
    st.P[1] = v16i{0};
#pragma unroll
    for (int i = 0; i < 4; ++i) st.T[i] = 0.0f;
    float sp = 0.0f;                       // scale of the previous item's second i-block

    for (;;) {
      // ---- the items after this one (all wave-uniform scalar logic)
      const bool n1res = !res && (r0.slot0 >= 0 || r0.slot1 >= 0);
      const int n1k = n1res ? k : k + 1;
      const bool has1 = n1k < nkb;
      const bool n2res = !n1res && (r1.slot0 >= 0 || r1.slot1 >= 0);
      const int n2k = (n1res || n2res) ? k + 1 : k + 2;
      const bool has2 = n2k < nkb;

      // ---- scales of this item
      float s0, s1;
      if (!res) {
        s0 = r0.sa0 * r0.sb;
        s1 = r0.sa1 * r0.sb;
        poison0 |= r0.slot0 == -2;
        poison1 |= r0.slot1 == -2;
      } else {   // an unflagged half multiplies stale LDS contents by zero: adds +0
        s0 = r0.slot0 >= 0 ? r0.rs0 * r0.sb : 0.0f;
        s1 = r0.slot1 >= 0 ? r0.rs1 * r0.sb : 0.0f;
      }

      const int8_t* const a_cur = a_ring + (t & 1) * kRingBytes;
      const int8_t* const a_nxt = a_ring + ((t + 1) & 1) * kRingBytes;
      const int8_t* const b_nxt = b_ring + (n1k & 1) * kRingBytes + (jq >> 1) * kBlockBytes;

      run_unit<0>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);
      run_unit<1>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);
      run_unit<2>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);
      run_unit<3>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);
      run_unit<4>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);
      run_unit<5>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);

      // All LDS reads of this item are issued (units 6, 7 run from registers).  Wait for them
      // and for the next item's direct-to-LDS loads, then the barrier publishes the next item
      // and frees this item's ring slots for the item after it.
      __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
      __syncthreads();
      if (has2) {
        if (n2res) stage_item(k + 1, 1, r1, t & 1, false);
        else stage_item(n2k, 0, r1, t & 1, n2k != n1k);
      }

      run_unit<6>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);
      run_unit<7>(st, a_cur, a_nxt, b_nxt, h, jq, lane, s0, s1, sp);

      sp = s1;
      if (!has1) break;
      // ---- advance to the next item
      ++t;
      if (n1res) {
        res = 1;
      } else {
        res = 0;
        ++k;
        r0 = r1;
        r1 = r2;
        load_res_scales(r1);      // its slots were fetched an item ago
        r2 = load_rec(k + 2);
      }
    }
    drain(st, sp);
  }
store:
  // ---- epilogue.  The MFMA result layout (lane = column, registers = rows) would give 64-byte
  // global stores; instead each wavefront transposes its tile through a private LDS patch
  // (64 rows x 64 columns of FP32 at a time, row pitch 72 floats: conflict-free both ways) and
  // writes whole 128/256-byte row segments with 16-byte stores.
  __syncthreads();   // every wavefront is done reading the operand rings
  if (tj * 2 + (jq >> 1) >= p.njb) return;
  float* const stg = reinterpret_cast<float*>(lds + w * kStageBytesPerWave);
  const int col0 = jb * kBlock + (jq & 1) * 64;        // first column of this wave's tile
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    if (half && ti * 2 + 1 >= p.nib) break;
    const bool poison = !kDebug && (half ? poison1 : poison0);
    // a flagged block whose residual found no slot cannot be computed: poison its rows
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int sj = 0; sj < 2; ++sj)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rl = s2 * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const int cl = sj * 32 + (lane & 31);
          stg[rl * kStagePitch + cl] = poison ? __int_as_float(0x7FC00000) : acc[half * 2 + s2][sj][r];
        }
    const int row0 = (half ? ib1 : ib0) * kBlock + h * 64;
    if (!kDebug && p.out_bf16) {
      uint16_t* const C = reinterpret_cast<uint16_t*>(p.c);
      const int c8 = (lane & 7) * 8;
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int rl = it * 8 + (lane >> 3);
        const int row = row0 + rl, col = col0 + c8;
        const float4 lo = *reinterpret_cast<const float4*>(stg + rl * kStagePitch + c8);
        const float4 hi = *reinterpret_cast<const float4*>(stg + rl * kStagePitch + c8 + 4);
        if (row >= p.M || col >= p.N) continue;
        uint16_t* dst = C + (int64_t)row * p.ldc + col;
        if (p.vec_ok && col + 8 <= p.N) {
          v4i o;
          o[0] = pack_bf16x2(lo.x, lo.y); o[1] = pack_bf16x2(lo.z, lo.w);
          o[2] = pack_bf16x2(hi.x, hi.y); o[3] = pack_bf16x2(hi.z, hi.w);
          *reinterpret_cast<v4i*>(dst) = o;
        } else {
          const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (col + e < p.N) dst[e] = (uint16_t)float_to_bf16_bits(v[e]);
        }
      }
    } else {
      float* const C = reinterpret_cast<float*>(p.c);
      const int c4 = (lane & 15) * 4;
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int rl = it * 4 + (lane >> 4);
        const int row = row0 + rl, col = col0 + c4;
        const float4 v = *reinterpret_cast<const float4*>(stg + rl * kStagePitch + c4);
        if (row >= p.M || col >= p.N) continue;
        float* dst = C + (int64_t)row * p.ldc + col;
        if (p.vec_ok && col + 4 <= p.N) {
          *reinterpret_cast<float4*>(dst) = v;
        } else {
          const float e4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + e < p.N) dst[e] = e4[e];
        }
      }
    }
  }
}

// The INT32 block product of one k-block, main or residual term (inspection / tests): one
// workgroup per 128 x 128 output block, wavefront w computes rows [32w, 32w+32) straight from
// global memory.
__global__ __launch_bounds__(256) void partials_kernel(GemmParams p) {
  const int ib = blockIdx.x / p.njb, jb = blockIdx.x - ib * p.njb;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int k = p.debug_k;
  const int8_t* ablk = p.a_codes + ((int64_t)ib * p.nkb + k) * kBlockBytes;
  bool zero = false;
  if (p.debug_residual) {
    const int slot = p.a_slot ? p.a_slot[ib * p.a_si + k * p.a_sk] : -1;
    zero = slot < 0;
    ablk = p.a_res + (int64_t)(zero ? 0 : slot) * kBlockBytes;
  }
  const int8_t* bblk = p.b_codes + ((int64_t)jb * p.nkb + k) * kBlockBytes;
  int32_t* const out = reinterpret_cast<int32_t*>(p.c);
#pragma unroll
  for (int sj = 0; sj < 4; ++sj) {
    v16i P = {0};
    if (!zero) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
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

hipError_t launch_gemm(const GemmParams& p, bool debug, hipStream_t st) {
  if (debug) {
    if (p.nib * p.njb == 0) return hipSuccess;
    hipLaunchKernelGGL(partials_kernel, dim3(p.nib * p.njb), dim3(256), 0, st, p);
    return hipGetLastError();
  }
  const int tiles = ((p.nib + 1) / 2) * ((p.njb + 1) / 2);
  if (tiles == 0) return hipSuccess;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(gemm_kernel, dim3(tiles), dim3(kThreads), kLdsBytes, st, p);
  return hipGetLastError();
}

}  // namespace fq
