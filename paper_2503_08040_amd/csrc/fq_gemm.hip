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
//     quantization blocks.  Wavefront (h, c) owns all 128 rows of i-block h and
//     the 64-column quarter c of the tile: 4 x 2 sub-tiles of 32 x 32, 128 FP32
//     accumulators per lane in architectural VGPRs (the vector ALU cannot read
//     accumulation registers, so the accumulators it updates must not live
//     there).  A second geometry, 1 x 3 blocks (128 x 384, 2 x 3 sub-tiles per
//     wavefront), covers the last block columns when the 2 x 2 tiles would
//     leave the final round of the chip mostly idle;
//   - the k-loop runs over "items": the main product of k-block k and, when
//     one of the tile's A blocks is flagged at k, a residual item right
//     after it.  A and B operands sit in two independent double-buffered LDS
//     rings (64 KiB each for 2 x 2): an item always brings a new A set (codes or
//     residual codes), a new B set only when k advances, so the residual
//     product re-uses the B blocks already on chip exactly as Alg. 1 says.
//     A residual item is work only for the wavefronts whose i-block is flagged
//     at that k: the others skip its multiplications (they still take part in
//     staging and in the barrier), so with one of the two blocks flagged the
//     item runs on one wavefront per SIMD and costs about 60 % of a full item;
//   - operands reach LDS by direct global->LDS 16-byte loads (blocks are stored
//     in operand order, see fq.h), one barrier per item;
//   - per 32 x 32 sub-tile: 8 v_mfma_i32_16x16x64_i8 (four 16 x 16 quadrants x
//     two halves of K = 128) into an INT32 tile, then one convert + one FMA per
//     element folds it into the FP32 accumulators with the scalar scale of that
//     block pair.  (The 16x16x64 form sustains a third more than 32x32x32 on this
//     part and leaves the dequantizing pipeline about 10 % faster.)
// The accumulation order per output element is exactly Alg. 1's (k ascending,
// main term then residual term) in both geometries, so results match a
// sequential evaluation bit for bit and do not depend on the tile plan.
#include <algorithm>
#include <atomic>
#include <cstdlib>

#include "fq_device.h"
#include "fq_kernels.h"

// Ablation switches (measurement support; the library itself is built with none of them, and a
// build with one computes wrong products on purpose).  Each removes or adds one component of the
// k-loop so that its cost can be read off a timing of the whole kernel:
//   FQ_ABLATE_NO_DMA        no global -> LDS loads (the rings keep whatever they hold)
//   FQ_ABLATE_NO_MULTIPLY   no wavefront multiplies: loads, waits, barriers and epilogue only
//   FQ_ABLATE_NO_DEQUANT    the MFMAs and their LDS reads, without the converts and FMAs
//   FQ_ABLATE_EXTRA_SALU=n  n dependent scalar additions behind every barrier of the k-loop
//   FQ_ABLATE_DMA_HOT       every global -> LDS load reads from the first MiB of the A codes (which
//                           must be that large), so that all of them hit the L2
//   FQ_ABLATE_ONE_STAGER    wavefronts 0-3 (one per SIMD) issue all loads, 16 each, 4-7 none
//   FQ_ABLATE_TEAM_SKEW     (computes the right products) the two wavefronts of a SIMD half an item
//                           apart in the 2 x 2 geometry: the wavefronts of i-block 0 and of i-block
//                           1 form two teams with two barriers per item, each the item boundary of
//                           one team and the middle of the item of the other; a team loads its own
//                           A block, team 0 the B blocks as well.  The B operands of an item sit in
//                           registers after its first two units, which is why two ring slots still
//                           suffice.
namespace fq {

namespace {

constexpr int kThreads = 512;
constexpr int kMaxDevices = 64;   // per-device host-side caches
constexpr int kXcds = 8;      // accelerator complex dies, each with a private L2
constexpr int kGroupN = 4;    // tile columns per rasterization group
constexpr int kRingBytes = 2 * kBlockBytes;     // one A pair or one B pair
constexpr int kLdsBytes = 4 * kRingBytes;       // 128 KiB: two A sets + two B sets; the epilogue
                                                // staging patches re-use the same memory

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
#ifdef FQ_ABLATE_NO_DMA
  if (voff != 0xFFFFFFFFu) return;
#endif
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

// One wavefront copies 4 KiB (4 fragments) global -> LDS: one group of stage_half_block.
__device__ inline void stage_quarter_block(const int8_t* src, int8_t* lds_dst, int lane) {
  const unsigned voff = (unsigned)lane * 16u;
  const uint64_t a = reinterpret_cast<uint64_t>(src);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  src = reinterpret_cast<const int8_t*>(((uint64_t)hi << 32) | lo);
#ifdef FQ_ABLATE_NO_DMA
  if (voff != 0xFFFFFFFFu) return;
#endif
  gbl_void* g = (gbl_void*)(src + voff);
  lds_void* l = (lds_void*)lds_dst;
  __builtin_amdgcn_global_load_lds(g, l, 16, 0 * kFragBytes, 0);
  __builtin_amdgcn_global_load_lds(g, l, 16, 1 * kFragBytes, 0);
  __builtin_amdgcn_global_load_lds(g, l, 16, 2 * kFragBytes, 0);
  __builtin_amdgcn_global_load_lds(g, l, 16, 3 * kFragBytes, 0);
}

// two floats -> two bf16 (round-to-nearest-even) in one dword, low half first
__device__ inline int pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  f32x2 v = {a, b};
  return __builtin_bit_cast(int, __builtin_convertvector(v, bf16x2));
}

// One operand of v_mfma_i32_16x16x64_i8 out of a block stored in tile order: rows (or
// columns) [32 rg + 16 rh, +16), contraction [64 ks, +64).  Lane l supplies row l % 16 and the
// 16 contraction-contiguous bytes of group l / 16, i.e. the bytes at tile_offset(row, 64 ks +
// 16 (l / 16)): whole 256-byte runs per 16 lanes, conflict-free.  The order of the contraction
// inside the instruction does not matter as long as both operands use the same one.
__device__ inline v4i lds_frag(const int8_t* blk, int rg, int rh, int ks, int lane) {
  return *reinterpret_cast<const v4i*>(blk + ((rg * 4 + ks * 2) * 64 + rh * 16) * 16 +
                                       (lane + 16 * (lane >> 4)) * 16);
}


// Empty volatile asm statements that take values as read-write register operands.  The
// compiler may not reorder volatile asm, so the instructions producing the operands stay
// before the statement and their consumers after it: this pins the source order of otherwise
// freely movable pure instructions (MFMA, convert, FMA) without emitting any code.
__device__ __forceinline__ void pin(v4i& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ void pin(float& a, float& b) { asm volatile("" : "+v"(a), "+v"(b)); }

// Geometry of a workgroup tile: kBI x kBJ quantization blocks, computed by 8 wavefronts laid
// out 2 (row halves h) x 4 (column groups c).  Wavefront (h, c) owns rows [64h, 64h+64) of every
// i-block of the tile and the 32*kBJ columns starting at 32*kBJ*c: kSI x kSJ sub-tiles of
// 32 x 32.  Two geometries are used: 2 x 2 blocks (256 x 256, 8 sub-tiles per wavefront) for
// the bulk of the output and 1 x 3 blocks (128 x 384, 6 sub-tiles) for the columns left over
// when the 2 x 2 tiles do not fill a whole number of rounds of the chip (see launch_gemm).
template <int kBI_, int kBJ_>
struct Geo {
  static constexpr int kBI = kBI_, kBJ = kBJ_;
  static constexpr int kSI = 2 * kBI;        // 32-row groups per wavefront
  static constexpr int kSJ = kBJ;            // 32-column groups per wavefront
  static constexpr int kUnits = kSI * kSJ;   // sub-tiles per wavefront and item
  static constexpr int kASet = kBI * kBlockBytes;   // the A blocks of one item in LDS
  static constexpr int kBSet = kBJ * kBlockBytes;   // the B blocks of one k-block in LDS
  // A wavefront's columns lie in one j-block when kBJ = 2 and in up to two when kBJ = 3, so the
  // scale of a sub-tile depends on sj only in the second case.
  static constexpr int kSC = (kBJ == 2) ? 1 : kSJ;  // distinct scale columns per i-block
  static constexpr int kSP = (kBJ == 2) ? 1 : 2;    // distinct scales of an item's last two units
  static constexpr int kStageCols = 32 * kSJ;
  static constexpr int kStagePitch = kStageCols + 4;   // floats per staged row: 4 rows apart = 16 banks apart
  static constexpr int kStageBytesPerWave = 32 * kStagePitch * 4;
  // Rows of a wavefront.  With two i-blocks per tile, wavefront half h owns all 128 rows of
  // i-block h (so that a residual item of one flagged block is work for that half of the
  // wavefronts only); with one i-block it owns rows [64h, 64h+64) of it.  si counts the
  // wavefront's 32-row groups: its i-block and its row group inside that block.
  __device__ static constexpr int a_block(int h, int /*si*/) { return kBI == 2 ? h : 0; }
  __device__ static constexpr int a_group(int h, int si) { return kBI == 2 ? si : 2 * h + si; }
  static_assert(2 * (kASet + kBSet) <= kLdsBytes, "operand rings must fit");
  static_assert(8 * kStageBytesPerWave <= kLdsBytes, "epilogue staging must fit");
  static_assert(kBI + kBJ == 4, "8 wavefronts stage 8 half-blocks per item");
};

// Per-wavefront register state of the k-loop.
template <class G>
struct WaveState {
  // FP32 accumulators: sub-tile (si, sj), 16 elements per lane; element 4 q + r belongs to
  // quadrant q = 2 rh + ch of the sub-tile: row 16 rh + 4 (lane / 16) + r, column 16 ch + lane % 16
  float acc[G::kSI][G::kSJ][16];
  v4i aq[2][2][2];                 // A operands [rh][ks] of two consecutive si: si uses aq[si & 1]
  v4i bq[G::kSJ][2][2];            // B operands [ch][ks] of this wave's column groups
  v4i P[2][4];                     // INT32 quadrants: sub-tile u accumulates into P[u & 1]
  float T[2];                      // elements converted in the previous slot, waiting for their FMA
};

// Scales of one item as this wavefront's units see them: s[sc] = a^A (or a~^A) of the
// wavefront's i-block times a^B of the j-block that scale column sc lies in.
template <class G>
struct ItemScales {
  float s[G::kSC];
};

// The k-loop is one continuous software pipeline over sub-tiles ("units": u = kSJ*si + sj).
// A unit is 8 slots.  Slot n issues one v_mfma_i32_16x16x64_i8 of unit u: contraction half
// ks = n / 4 of quadrant q = n % 4 (q = 2 rh + ch: row half rh, column half ch of the 32 x 32
// sub-tile), so the two MFMAs that accumulate into the same quadrant are four slots apart.  In
// the 16 cycles the matrix core needs for it the slot also issues 4 vector-ALU instructions that
// fold the finished INT32 tile of unit u-1 into the FP32 accumulators: the 2 FMAs of the
// elements converted one slot earlier, then the 2 converts of elements 2n, 2n+1.  An FMA never
// waits for its convert, and a convert reads a quadrant whose last MFMA is at least four slots
// old.  Operand registers are refilled from LDS well before their next use: the A operands of
// si+1 are fetched into a second register buffer while si is being multiplied (LDS latency
// under load is several hundred cycles), and the last two units fetch the B operands and the
// first A operands of the NEXT item (a B operand right after its last use), so that no item
// starts with a burst of LDS reads.  Scheduling fences pin this order.
//   a_cur: A set of the current item in LDS; a_nxt / b_nxt: A set / B set of the next item.
//   sc: scales of the current item; sp: scales of the previous item's last two units.
//   h, c: this wavefront's row half and column group.
//   kBiased: the tolerance variant (see gemm_biased_kernel): the first MFMA of a quadrant starts
//   from `magic` (the bit pattern of 1.25 * 2^23 in every element) instead of zero, so that the
//   finished INT32 value, read as binary32, IS 1.25 * 2^23 + P, exactly; the slot then issues only
//   the 2 FMAs of elements 2n, 2n+1 of unit u-1 straight from that tile and no converts.
template <class G, int u, bool kBiased>
__device__ __forceinline__ void run_unit(WaveState<G>& st, const int8_t* a_cur, const int8_t* a_nxt,
                                         const int8_t* b_nxt, int h, int c, int lane,
                                         const ItemScales<G>& sc, const float (&sp)[G::kSP],
                                         const v4i& magic) {
  constexpr int kSJ = G::kSJ, kUnits = G::kUnits;
  constexpr int si = u / kSJ, sj = u % kSJ;
  // B operand (ch, ks) of column group cg = kSJ*c + j of the tile: block cg / 4, group cg % 4
  auto b_frag = [&](int j, int ch, int ks) {
    const int cg = kSJ * c + j;
    return lds_frag(b_nxt + (cg >> 2) * kBlockBytes, cg & 3, ch, ks, lane);
  };
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    const int ks = n >> 2, rh = (n >> 1) & 1, ch = n & 1, q = 2 * rh + ch;
    {
      const v4i z = {0, 0, 0, 0};
      st.P[u & 1][q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
          st.aq[si & 1][rh][ks], st.bq[sj][ch][ks], ks ? st.P[u & 1][q] : (kBiased ? magic : z), 0, 0, 0);
      // B operand (ch, ks) was used for the last time in the slot with rh = 1
      const bool b_done = rh == 1;
      // the other four slots (rh = 0) carry a load each into a free buffer: operand i = 0..3
      const int i = 2 * ks + ch, irh = i >> 1, iks = i & 1;
      // A operands of the next si go into the other aq buffer a whole unit before their use
      if (si + 1 < G::kSI && sj == 0 && !b_done)
        st.aq[(si + 1) & 1][irh][iks] = lds_frag(a_cur + G::a_block(h, si + 1) * kBlockBytes,
                                                 G::a_group(h, si + 1), irh, iks, lane);
      // the last two units (same si, odd: they use aq[1]) fetch the next item's first operands
      if (u == kUnits - 2) {
        if (b_done) st.bq[sj][ch][ks] = b_frag(sj, ch, ks);
        else st.aq[0][irh][iks] = lds_frag(a_nxt + G::a_block(h, 0) * kBlockBytes,
                                           G::a_group(h, 0), irh, iks, lane);
      }
      if (u == kUnits - 1) {
        if (b_done) st.bq[sj][ch][ks] = b_frag(sj, ch, ks);
        else if (kSJ == 3) st.bq[0][irh][iks] = b_frag(0, irh, iks);
      }
      pin(st.P[u & 1][q]);
    }
    __builtin_amdgcn_sched_barrier(0);   // MFMA first: its destination must not alias live tiles
#ifndef FQ_ABLATE_NO_DEQUANT
    if constexpr (kBiased) {
      constexpr int kLastSi = G::kSI - 1;
      constexpr int fu = u - 1;
      constexpr bool prev = fu < 0;                     // the last unit of the previous item
      constexpr int pu = fu + kUnits;
      constexpr int fsi = prev ? kLastSi : fu / kSJ, fsj = prev ? pu % kSJ : fu % kSJ;
      const float s = prev ? sp[G::kSP - 1] : sc.s[G::kSC == 1 ? 0 : fsj];
      const int fe = 2 * n;
      st.acc[fsi][fsj][fe] = __builtin_fmaf(
          __int_as_float(st.P[(u - 1) & 1][n >> 1][2 * (n & 1)]), s, st.acc[fsi][fsj][fe]);
      st.acc[fsi][fsj][fe + 1] = __builtin_fmaf(
          __int_as_float(st.P[(u - 1) & 1][n >> 1][2 * (n & 1) + 1]), s, st.acc[fsi][fsj][fe + 1]);
      pin(st.acc[fsi][fsj][fe], st.acc[fsi][fsj][fe + 1]);
      __builtin_amdgcn_sched_barrier(0);
    } else {
      // FMAs of the 2 elements converted in the previous slot (unit u-1, or u-2 for n = 0);
      // negative units are the last two units of the previous item
      constexpr int kLastSi = G::kSI - 1;
      const int fu = n ? u - 1 : u - 2, fe = n ? 2 * (n - 1) : 14;
      const bool prev = fu < 0;
      const int pu = fu + kUnits;                       // unit index in the previous item
      const int fsi = prev ? kLastSi : fu / kSJ, fsj = prev ? pu % kSJ : fu % kSJ;
      const float s = prev ? sp[G::kSP == 1 ? 0 : pu - (kUnits - 2)]
                           : sc.s[G::kSC == 1 ? 0 : fsj];
      st.acc[fsi][fsj][fe] = __builtin_fmaf(st.T[0], s, st.acc[fsi][fsj][fe]);
      st.acc[fsi][fsj][fe + 1] = __builtin_fmaf(st.T[1], s, st.acc[fsi][fsj][fe + 1]);
      pin(st.acc[fsi][fsj][fe], st.acc[fsi][fsj][fe + 1]);
    }
    if constexpr (!kBiased) {
      __builtin_amdgcn_sched_barrier(0);   // FMAs before converts
      st.T[0] = (float)st.P[(u - 1) & 1][n >> 1][2 * (n & 1)];
      st.T[1] = (float)st.P[(u - 1) & 1][n >> 1][2 * (n & 1) + 1];
      pin(st.T[0], st.T[1]);
      __builtin_amdgcn_sched_barrier(0);
    }
#endif
  }
}

// Units [kFrom, kTo) of one item, in order.
template <class G, int kFrom, int kTo, bool kBiased>
__device__ __forceinline__ void run_units_range(WaveState<G>& st, const int8_t* a_cur,
                                                const int8_t* a_nxt, const int8_t* b_nxt, int h,
                                                int c, int lane, const ItemScales<G>& sc,
                                                const float (&sp)[G::kSP], const v4i& magic) {
  if constexpr (kFrom < kTo) {
    run_unit<G, kFrom, kBiased>(st, a_cur, a_nxt, b_nxt, h, c, lane, sc, sp, magic);
    run_units_range<G, kFrom + 1, kTo, kBiased>(st, a_cur, a_nxt, b_nxt, h, c, lane, sc, sp, magic);
  }
}

// Folds the last two units of the last item (scales sp) into the accumulators.
template <class G, bool kBiased>
__device__ __forceinline__ void drain(WaveState<G>& st, const float (&sp)[G::kSP]) {
  constexpr int kLastSi = G::kSI - 1, kSJ = G::kSJ, kP = (G::kUnits - 1) & 1;
  if constexpr (kBiased) {      // only the last unit is pending: all 16 elements of its biased tile
    const float s = sp[G::kSP - 1];
#pragma unroll
    for (int e = 0; e < 16; ++e)
      st.acc[kLastSi][kSJ - 1][e] =
          __builtin_fmaf(__int_as_float(st.P[kP][e >> 2][e & 3]), s, st.acc[kLastSi][kSJ - 1][e]);
    return;
  }
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    const int fsj = n ? kSJ - 1 : kSJ - 2, fe = n ? 2 * (n - 1) : 14;
    const float s = sp[G::kSP == 1 ? 0 : (n ? 1 : 0)];
    st.acc[kLastSi][fsj][fe] = __builtin_fmaf(st.T[0], s, st.acc[kLastSi][fsj][fe]);
    st.acc[kLastSi][fsj][fe + 1] = __builtin_fmaf(st.T[1], s, st.acc[kLastSi][fsj][fe + 1]);
    st.T[0] = (float)st.P[kP][n >> 1][2 * (n & 1)];
    st.T[1] = (float)st.P[kP][n >> 1][2 * (n & 1) + 1];
  }
  const float s = sp[G::kSP - 1];
  st.acc[kLastSi][kSJ - 1][14] = __builtin_fmaf(st.T[0], s, st.acc[kLastSi][kSJ - 1][14]);
  st.acc[kLastSi][kSJ - 1][15] = __builtin_fmaf(st.T[1], s, st.acc[kLastSi][kSJ - 1][15]);
}

// Scalars of one k-block: residual slots and scales of the tile's A blocks, scales of the (up
// to two) B blocks this wave's columns lie in.
template <class G>
struct KRec {
  int slot[G::kBI];
  float sa[G::kBI];
  float rs[G::kBI];   // residual scales (valid where the slot is >= 0)
  float sb[2];
};

}  // namespace

namespace {

// One output tile of geometry G whose first blocks are (ib_first, jb_first).  Blocks beyond
// the matrix repeat the last valid one (their products are never stored).
// kBiased: the tolerance variant.  Every item adds (1.25 * 2^23 + P) * s instead of P * s to the
// accumulators; the wavefront keeps the sum of the scales it has used per scale column and,
// after every kBiasWindow items it took part in (and at the end), folds the pending unit and
// subtracts 1.25 * 2^23 times that sum with one FMA per accumulator.  The window bounds the
// magnitude the accumulators carry, and with it the rounding error of the additions, whatever K.
constexpr int kBiasWindow = 4;
constexpr int kMagicBits = 0x4B200000;          // 1.25 * 2^23 as binary32: with |P| <= 128 * 127^2 < 2^21 the sum
                                                // stays inside [2^23, 2^24), where one ulp is 1
constexpr float kMagic = 10485760.0f;

template <class G, bool kBiased>
__device__ __forceinline__ void tile_body(const GemmParams& p, int ib_first, int jb_first,
                                          int8_t* lds) {
  constexpr int kBI = G::kBI, kBJ = G::kBJ, kSI = G::kSI, kSJ = G::kSJ, kUnits = G::kUnits;
#ifdef FQ_ABLATE_TEAM_SKEW
  constexpr bool kSkew = kBI == 2 && kBJ == 2;
#else
  constexpr bool kSkew = false;
#endif
  int8_t* const a_ring = lds;                    // [2][kBI blocks]
  int8_t* const b_ring = lds + 2 * G::kASet;     // [2][kBJ blocks]

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = w >> 2, c = w & 3;

  int ib[kBI], jbt[kBJ];
#pragma unroll
  for (int i = 0; i < kBI; ++i) ib[i] = min(ib_first + i, p.nib - 1);
#pragma unroll
  for (int j = 0; j < kBJ; ++j) jbt[j] = min(jb_first + j, p.njb - 1);
  // the (up to two) j-blocks this wave's columns lie in, as indices into the tile's blocks
  const int jlo = (kSJ * c) >> 2, jhi = (kSJ * c + kSJ - 1) >> 2;

  // ---- what this wave stages: 8 KiB (half a block) per item; the first 2*kBI waves the A
  // blocks, the others the B blocks
#ifdef FQ_ABLATE_ONE_STAGER
  const bool stager = w < 4;                      // whole blocks: A blocks first, then B blocks
  const bool stage_a = w < kBI;
  const int sidx = stage_a ? w : (w - kBI) & 3;
  const int spart = 0;
#else
  const bool stage_a = w < 2 * kBI;
  const int sidx = stage_a ? (w >> 1) : ((w - 2 * kBI) >> 1);   // which block of the set
  const int spart = (w & 1) * (kBlockBytes / 2);
#endif
  int sblk = 0;
#pragma unroll
  for (int i = 0; i < kBI; ++i) if (stage_a && sidx == i) sblk = ib[i];
#pragma unroll
  for (int j = 0; j < kBJ; ++j) if (!stage_a && sidx == j) sblk = jbt[j];
  const int soff = sidx * kBlockBytes + spart;
  const int8_t* const smain = (stage_a ? p.a_codes : p.b_codes) +
                              (int64_t)sblk * p.nkb * kBlockBytes + spart;

  // Scales and slots are read-only for the whole kernel: reading them through the constant
  // address space makes them scalar loads, which do not share a counter with the vector loads.
  typedef const __attribute__((address_space(4))) float cfloat;
  typedef const __attribute__((address_space(4))) int32_t cint;
  cfloat* const a_sc = (cfloat*)p.a_scales;
  cfloat* const b_sc = (cfloat*)p.b_scales;
  cfloat* const r_sc = (cfloat*)p.a_res_scales;
  cint* const a_sl = (cint*)p.a_slot;
  const bool has_fb = p.a_slot != nullptr;
  int ia[kBI];
#pragma unroll
  for (int i = 0; i < kBI; ++i) ia[i] = ib[i] * p.a_si;
  int jlo_blk = jbt[0], jhi_blk = jbt[0];
#pragma unroll
  for (int j = 0; j < kBJ; ++j) {
    if (jlo == j) jlo_blk = jbt[j];
    if (jhi == j) jhi_blk = jbt[j];
  }
  const int ibj_lo = jlo_blk * p.b_sj, ibj_hi = jhi_blk * p.b_sj;
  const int nkb = p.nkb;

  auto load_rec = [&](int k) -> KRec<G> {
    KRec<G> r;
#pragma unroll
    for (int i = 0; i < kBI; ++i) { r.slot[i] = -1; r.sa[i] = 0.0f; r.rs[i] = 0.0f; }
    r.sb[0] = r.sb[1] = 0.0f;
    if (k < nkb) {
#pragma unroll
      for (int i = 0; i < kBI; ++i) {
        if (has_fb) r.slot[i] = a_sl[ia[i] + k * p.a_sk];
        r.sa[i] = a_sc[ia[i] + k * p.a_sk];
      }
      r.sb[0] = b_sc[ibj_lo + k * p.b_sk];
      if (G::kSC > 1) r.sb[1] = b_sc[ibj_hi + k * p.b_sk];
    }
    return r;
  };
  // Residual scales depend on the slots, so they are fetched one step after the record itself:
  // by then the slots have arrived and the dependent load does not stall the wavefront.
  auto load_res_scales = [&](KRec<G>& r) {
#pragma unroll
    for (int i = 0; i < kBI; ++i) if (r.slot[i] >= 0) r.rs[i] = r_sc[r.slot[i]];
  };
  auto any_flagged = [&](const KRec<G>& r) {
    bool f = false;
#pragma unroll
    for (int i = 0; i < kBI; ++i) f |= r.slot[i] >= 0;
    return f;
  };
  // Stages this wave's 8 KiB share of item (k, res) into ring slot `asel` (A) / k & 1 (B).
  auto stage_item = [&](int k, int res, const KRec<G>& r, int asel, bool new_b) {
#ifdef FQ_ABLATE_ONE_STAGER
    if (!stager) return;
#endif
    if (stage_a) {
      const int8_t* src;
      if (res) {
        int s = -1;
#pragma unroll
        for (int i = 0; i < kBI; ++i) if (sidx == i) s = r.slot[i];
        if (s < 0) return;   // unflagged block: nothing to bring (its wavefronts skip the item)
        src = p.a_res + (int64_t)s * kBlockBytes + spart;
      } else {
        src = smain + (int64_t)k * kBlockBytes;
      }
#ifdef FQ_ABLATE_DMA_HOT
      src = p.a_codes + (reinterpret_cast<uintptr_t>(src) & 0xFE000u);
#endif
      stage_half_block(src, a_ring + asel * G::kASet + soff, lane);
#ifdef FQ_ABLATE_ONE_STAGER
      stage_half_block(src + kBlockBytes / 2, a_ring + asel * G::kASet + soff + kBlockBytes / 2, lane);
#endif
    } else if (new_b) {
#ifdef FQ_ABLATE_DMA_HOT
      stage_half_block(p.a_codes + (reinterpret_cast<uintptr_t>(smain + (int64_t)k * kBlockBytes) & 0xFE000u),
                       b_ring + (k & 1) * G::kBSet + soff, lane);
#else
      stage_half_block(smain + (int64_t)k * kBlockBytes, b_ring + (k & 1) * G::kBSet + soff, lane);
#endif
#ifdef FQ_ABLATE_ONE_STAGER
      stage_half_block(smain + (int64_t)k * kBlockBytes + kBlockBytes / 2,
                       b_ring + (k & 1) * G::kBSet + soff + kBlockBytes / 2, lane);
#endif
    }
  };
  // kSkew: this wavefront's share of item (k, res) when the two teams (h = 0, 1: the wavefronts
  // of i-block h, one per SIMD each) run half an item apart: a quarter of its own team's A block,
  // and for team 0 half a B block as well.
  auto stage_team = [&](int k, int res, const KRec<G>& r, int asel, bool new_b) {
    int blk = ib[0], s = r.slot[0];
#pragma unroll
    for (int i = 1; i < kBI; ++i) if (h == i) { blk = ib[i]; s = r.slot[i]; }
    const int quarter = c * (kBlockBytes / 4);
    int8_t* const dst = a_ring + asel * G::kASet + h * kBlockBytes + quarter;
    if (!res) stage_quarter_block(p.a_codes + ((int64_t)blk * p.nkb + k) * kBlockBytes + quarter, dst, lane);
    else if (s >= 0) stage_quarter_block(p.a_res + (int64_t)s * kBlockBytes + quarter, dst, lane);
    if (h == 0 && new_b) {
      int jb = jbt[0];
#pragma unroll
      for (int j = 1; j < kBJ; ++j) if ((c >> 1) == j) jb = jbt[j];
      const int part = (c >> 1) * kBlockBytes + (c & 1) * (kBlockBytes / 2);
      stage_half_block(p.b_codes + ((int64_t)jb * p.nkb + k) * kBlockBytes + (c & 1) * (kBlockBytes / 2),
                       b_ring + (k & 1) * G::kBSet + part, lane);
    }
  };
  // scale column sc belongs to the wave's second j-block?
  auto sc_is_hi = [&](int scol) { return ((kSJ * c + scol) >> 2) != jlo; };

  WaveState<G> st;
#pragma unroll
  for (int si = 0; si < kSI; ++si)
#pragma unroll
    for (int sj = 0; sj < kSJ; ++sj)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.acc[si][sj][r] = 0.0f;
  bool poison = false;           // this wavefront's i-block has a flagged block without a slot
  v4i magic = {kMagicBits, kMagicBits, kMagicBits, kMagicBits};
  if (kBiased) asm volatile("" : "+v"(magic));   // stays in registers: an MFMA operand cannot be a literal
  float bias_s[G::kSC];          // kBiased: sum of the scales used since the bias was last removed
#pragma unroll
  for (int q = 0; q < G::kSC; ++q) bias_s[q] = 0.0f;
  int bias_items = 0;
  // removes the bias accumulated so far; the pipeline must have been drained
  auto remove_bias = [&]() {
#pragma unroll
    for (int si = 0; si < kSI; ++si)
#pragma unroll
      for (int sj = 0; sj < kSJ; ++sj)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          st.acc[si][sj][e] = __builtin_fmaf(bias_s[G::kSC == 1 ? 0 : sj], -kMagic, st.acc[si][sj][e]);
#pragma unroll
    for (int q = 0; q < G::kSC; ++q) bias_s[q] = 0.0f;
    bias_items = 0;
  };

  if (nkb > 0) {
    // ---- prologue: items 0 and 1 into the two ring slots
    // records are fetched two k-blocks ahead so that no scalar load is waited for in the loop
    KRec<G> r0 = load_rec(0), r1 = load_rec(1), r2 = load_rec(2);
    int k = 0, res = 0, t = 0;
    if constexpr (kSkew) {
      stage_team(0, 0, r0, 0, true);
      if (any_flagged(r0)) stage_team(0, 1, r0, 1, false);
      else if (1 < nkb) stage_team(1, 0, r1, 1, true);
    } else {
      stage_item(0, 0, r0, 0, true);
      if (any_flagged(r0)) stage_item(0, 1, r0, 1, false);
      else if (1 < nkb) stage_item(1, 0, r1, 1, true);
    }
    load_res_scales(r0);
    load_res_scales(r1);
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0): this wave's direct-to-LDS loads landed
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      st.aq[0][i >> 1][i & 1] = lds_frag(a_ring + G::a_block(h, 0) * kBlockBytes, G::a_group(h, 0),
                                         i >> 1, i & 1, lane);
#pragma unroll
      for (int j = 0; j < kSJ; ++j) {
        const int cg = kSJ * c + j;
        st.bq[j][i >> 1][i & 1] =
            lds_frag(b_ring + (cg >> 2) * kBlockBytes, cg & 3, i >> 1, i & 1, lane);
      }
    }
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) st.P[1][qd] = v4i{0, 0, 0, 0};
    st.T[0] = st.T[1] = 0.0f;
    float sp[G::kSP];                      // scales of the previous item's last two units
#pragma unroll
    for (int i = 0; i < G::kSP; ++i) sp[i] = 0.0f;

    int late_b_k = -1;     // B stagers: k-block whose B set is still to be requested (-1: none)
    if (kSkew && h == 1) asm volatile("s_barrier" ::: "memory");   // team 1 starts one barrier later
    for (;;) {
      // The B stagers request their blocks here, two units after the barrier that freed the
      // ring slot, not right behind it: right after the barrier the four A stagers (one per
      // SIMD) are blocked on their eight load instructions each, and while they wait for the
      // address unit to take them, the B stagers, which share their SIMDs, run the last two
      // units of the item.  With all 64 loads issued at once, both wavefronts of every SIMD sat
      // blocked and the matrix cores idled for about a fifth of every item.
      if (late_b_k >= 0) {
#ifdef FQ_ABLATE_DMA_HOT
        stage_half_block(p.a_codes + (reinterpret_cast<uintptr_t>(smain + (int64_t)late_b_k * kBlockBytes) & 0xFE000u),
                         b_ring + (late_b_k & 1) * G::kBSet + soff, lane);
#else
        stage_half_block(smain + (int64_t)late_b_k * kBlockBytes, b_ring + (late_b_k & 1) * G::kBSet + soff, lane);
#endif
      }
      late_b_k = -1;
      // ---- the items after this one (all wave-uniform scalar logic)
      const bool n1res = !res && any_flagged(r0);
      const int n1k = n1res ? k : k + 1;
      const bool has1 = n1k < nkb;
      const bool n2res = !n1res && any_flagged(r1);
      const int n2k = (n1res || n2res) ? k + 1 : k + 2;
      const bool has2 = n2k < nkb;

      // ---- this wavefront's i-block in this item: its slot, scale, and whether there is work
      int my_slot = r0.slot[0];
      float my_sa = res ? r0.rs[0] : r0.sa[0];
#pragma unroll
      for (int i = 1; i < kBI; ++i)
        if (G::a_block(h, 0) == i) {
          my_slot = r0.slot[i];
          my_sa = res ? r0.rs[i] : r0.sa[i];
        }
      if (!res) poison |= my_slot == -2;
      // a residual item is work only for the wavefronts whose i-block is flagged at this k
#ifdef FQ_ABLATE_NO_MULTIPLY
      const bool active = p.M < 0;
#else
      const bool active = !res || my_slot >= 0;
#endif
      ItemScales<G> sc;
#pragma unroll
      for (int q = 0; q < G::kSC; ++q)
        sc.s[q] = my_sa * ((G::kSC > 1 && sc_is_hi(q)) ? r0.sb[1] : r0.sb[0]);

      const int8_t* const a_cur = a_ring + (t & 1) * G::kASet;
      const int8_t* const a_nxt = a_ring + ((t + 1) & 1) * G::kASet;
      const int8_t* const b_nxt = b_ring + (n1k & 1) * G::kBSet;

      if constexpr (kSkew) {
        // two barriers per item: this one is the other team's item boundary, in the middle of ours
        if (active) run_units_range<G, 0, 2, kBiased>(st, a_cur, a_nxt, b_nxt, h, c, lane, sc, sp, magic);
        // Behind this barrier team 0 may overwrite the B set this wavefront took its operands
        // from.  An active wavefront has multiplied with all of them by now; one that skips the
        // item has not used them yet and waits for the reads here.
        else __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
        asm volatile("s_barrier" ::: "memory");
        if (active) run_units_range<G, 2, kUnits - 2, kBiased>(st, a_cur, a_nxt, b_nxt, h, c, lane, sc, sp, magic);
      } else {
        if (active) run_units_range<G, 0, kUnits - 2, kBiased>(st, a_cur, a_nxt, b_nxt, h, c, lane, sc, sp, magic);
      }

      // All LDS reads of this item are issued (the last two units run from registers).  Wait
      // for them and for the next item's direct-to-LDS loads, then the barrier publishes the
      // next item and frees this item's ring slots for the item after it.
      __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
      __syncthreads();
#ifdef FQ_ABLATE_EXTRA_SALU
      {
        int chain = k;
#pragma unroll
        for (int i = 0; i < FQ_ABLATE_EXTRA_SALU; ++i) asm volatile("s_add_i32 %0, %0, 1" : "+s"(chain));
        asm volatile("" :: "s"(chain));
      }
#endif
#ifdef FQ_ABLATE_ONE_STAGER
      if (has2) {
        if (n2res) stage_item(k + 1, 1, r1, t & 1, false);
        else stage_item(n2k, 0, r1, t & 1, n2k != n1k);
      }
#else
      if (has2) {
        if constexpr (kSkew) {
          if (n2res) stage_team(k + 1, 1, r1, t & 1, false);
          else stage_team(n2k, 0, r1, t & 1, n2k != n1k);
        } else if (stage_a) {
          if (n2res) stage_item(k + 1, 1, r1, t & 1, false);
          else stage_item(n2k, 0, r1, t & 1, false);
        } else if (!n2res && n2k != n1k) {
          late_b_k = n2k;
        }
      }
#endif

      if (active) {
        run_units_range<G, kUnits - 2, kUnits, kBiased>(st, a_cur, a_nxt, b_nxt, h, c, lane, sc, sp, magic);
#pragma unroll
        for (int i = 0; i < G::kSP; ++i) sp[i] = sc.s[G::kSC == 1 ? 0 : kSJ - 2 + i];
        if constexpr (kBiased) {
#pragma unroll
          for (int q = 0; q < G::kSC; ++q) bias_s[q] += sc.s[q];
          if (++bias_items == kBiasWindow) {
            // fold the pending unit, take the bias out, and restart the pipeline: the next unit 0
            // folds the same tile again with scale 0, which adds nothing
            drain<G, true>(st, sp);
            remove_bias();
#pragma unroll
            for (int i = 0; i < G::kSP; ++i) sp[i] = 0.0f;
          }
        }
      } else {
        // nothing to multiply in this item: the pipeline state (the pending tile of the last
        // active item and its scale) stays as it is; only fetch the next item's first operands,
        // which the last two units would have done
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          st.aq[0][i >> 1][i & 1] = lds_frag(a_nxt + G::a_block(h, 0) * kBlockBytes, G::a_group(h, 0),
                                             i >> 1, i & 1, lane);
#pragma unroll
          for (int j = 0; j < kSJ; ++j) {
            const int cg = kSJ * c + j;
            st.bq[j][i >> 1][i & 1] =
                lds_frag(b_nxt + (cg >> 2) * kBlockBytes, cg & 3, i >> 1, i & 1, lane);
          }
        }
      }
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
    if (kSkew && h == 0) asm volatile("s_barrier" ::: "memory");   // team 1's last item boundary
    drain<G, kBiased>(st, sp);
    if constexpr (kBiased) remove_bias();
  }

  // ---- epilogue.  The MFMA result layout (lane = column, registers = rows) would give 32-byte
  // global stores; instead each wavefront transposes its tile through a private LDS patch
  // (32 rows x 32*kSJ columns of FP32 at a time, row pitch + 4 floats) and writes whole row
  // segments with 16-byte stores.
  __syncthreads();   // every wavefront is done reading the operand rings
  float* const stg = reinterpret_cast<float*>(lds + w * G::kStageBytesPerWave);
  const int col0 = jb_first * kBlock + c * G::kStageCols;   // first column of this wave's tile
#pragma unroll
  for (int si = 0; si < kSI; ++si) {
    // a flagged block whose residual found no slot cannot be computed: poison its rows
    const bool bad = poison;
#pragma unroll
    for (int sj = 0; sj < kSJ; ++sj)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rl = 16 * (e >> 3) + 4 * (lane >> 4) + (e & 3);
        const int cl = sj * 32 + 16 * ((e >> 2) & 1) + (lane & 15);
        stg[rl * G::kStagePitch + cl] = bad ? __int_as_float(0x7FC00000) : st.acc[si][sj][e];
      }
    const int row0 = (ib_first + G::a_block(h, si)) * kBlock + G::a_group(h, si) * 32;
    if (p.out_bf16) {
      uint16_t* const C = reinterpret_cast<uint16_t*>(p.c);
      constexpr int kChunks = G::kStageCols / 8;         // 16-byte chunks per row
#pragma unroll
      for (int it = 0; it < 32 * kChunks / 64; ++it) {
        const int idx = it * 64 + lane;
        const int rl = idx / kChunks, c8 = (idx % kChunks) * 8;
        const int row = row0 + rl, col = col0 + c8;
        const float4 lo = *reinterpret_cast<const float4*>(stg + rl * G::kStagePitch + c8);
        const float4 hi = *reinterpret_cast<const float4*>(stg + rl * G::kStagePitch + c8 + 4);
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
      constexpr int kChunks = G::kStageCols / 4;
#pragma unroll
      for (int it = 0; it < 32 * kChunks / 64; ++it) {
        const int idx = it * 64 + lane;
        const int rl = idx / kChunks, c4 = (idx % kChunks) * 4;
        const int row = row0 + rl, col = col0 + c4;
        const float4 v = *reinterpret_cast<const float4*>(stg + rl * G::kStagePitch + c4);
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

// Workgroups are dealt to the 8 XCDs round-robin by id, and each XCD has its own L2.  Remap ids
// so that one XCD works through a contiguous run of tiles, and order the tiles in groups of
// kGroupN tile-columns walked row by row: the ~32 tiles resident on an XCD then form a patch
// that shares its A and B blocks through that L2.  Grouping by columns (not rows) gives every
// XCD tiles from all tile-rows, so fallback blocks clustered in a few block-rows (the worst
// case of Sec. 6.3) load the XCDs evenly.  b in [0, tiles_i * tiles_j) -> (ti, tj), a bijection.
__device__ __forceinline__ void tile_of(int b, int tiles_i, int tiles_j, int& ti, int& tj) {
  const int total = tiles_i * tiles_j;
  const int xcd = b % kXcds, l = b / kXcds;
  const int q = total / kXcds, rem = total % kXcds;
  const int L = xcd * q + min(xcd, rem) + l;
  const int group = kGroupN * tiles_i;
  const int g0 = (L / group) * kGroupN;
  const int gn = min(kGroupN, tiles_j - g0);
  const int within = L - (L / group) * group;
  tj = g0 + within % gn;
  ti = within / gn;
}

}  // namespace

// Grid: p.n_main workgroups compute 2 x 2-block tiles covering block columns [0, 2*main_tj),
// the rest 1 x 3-block tiles covering block columns [2*main_tj, njb).
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int ti, tj;
  if ((int)blockIdx.x < p.n_main) {
    tile_of(blockIdx.x, (p.nib + 1) >> 1, p.main_tj, ti, tj);
    tile_body<Geo<2, 2>, false>(p, 2 * ti, 2 * tj, lds);
  } else {
    tile_of(blockIdx.x - p.n_main, p.nib, p.tail_tj, ti, tj);
    tile_body<Geo<1, 3>, false>(p, ti, 2 * p.main_tj + 3 * tj, lds);
  }
}

// The tolerance variant of gemm_kernel: same tiles, same k-loop, same order of the terms, but the
// INT32 block products are folded into the FP32 accumulators without being converted: the first
// MFMA of every 16 x 16 quadrant accumulates onto the bit pattern of 1.25 * 2^23, so that the
// finished INT32 value read as binary32 is exactly 1.25 * 2^23 + P (|P| <= 128 * 127^2 < 2^21), one
// FMA per element adds (1.25 * 2^23 + P) * s, and the bias 1.25 * 2^23 * (sum of the scales used) is
// taken out every kBiasWindow items.  Half the vector-ALU instructions of Eq. (1) (the two left per
// MFMA are the ones its issue leaves free); the additions round at the magnitude of the biased
// sums, so results differ from gemm_kernel's by up to about 2e-4 of max |C|, whatever K.
__global__ __launch_bounds__(kThreads, 2) void gemm_biased_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int ti, tj;
  if ((int)blockIdx.x < p.n_main) {
    tile_of(blockIdx.x, (p.nib + 1) >> 1, p.main_tj, ti, tj);
    tile_body<Geo<2, 2>, true>(p, 2 * ti, 2 * tj, lds);
  } else {
    tile_of(blockIdx.x - p.n_main, p.nib, p.tail_tj, ti, tj);
    tile_body<Geo<1, 3>, true>(p, ti, 2 * p.main_tj + 3 * tj, lds);
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

namespace {

struct TilePlan {
  int n_main;    // workgroups computing 2 x 2-block tiles
  int main_tj;   // tile columns they cover (block columns [0, 2*main_tj))
  int tail_tj;   // 1 x 3-block tile columns covering the remaining block columns
};

// All of the output in 2 x 2-block tiles, unless their number leaves the last round of the
// chip mostly idle: then the last block columns are cut into 1 x 3-block tiles (3/4 of the work
// of a 2 x 2 tile each) so that the final round is shorter.  Costs are in units of one 2 x 2
// tile per compute unit.
TilePlan plan_tiles(int nib, int njb, int cus) {
  const int tiles_i = (nib + 1) / 2, tiles_j = (njb + 1) / 2;
  const int total = tiles_i * tiles_j;
  const TilePlan all{total, tiles_j, 0};
  if (cus <= 0 || total <= cus || total % cus == 0) return all;
  const int rounds = total / cus;
  const int cm = std::min(tiles_j, rounds * cus / tiles_i);
  const int tail_cols = njb - 2 * cm;
  if (cm <= 0 || tail_cols <= 0) return all;
  const int tail_tj = (tail_cols + 2) / 3;
  const int n_tail = nib * tail_tj;
  const double cost_all = (total + cus - 1) / cus;
  const double cost_split = (cm * tiles_i + cus - 1) / cus + 0.75 * ((n_tail + cus - 1) / cus);
  if (cost_split + 0.05 < cost_all) return TilePlan{cm * tiles_i, cm, tail_tj};
  return all;
}

// Compute units the planner assumes: the device's, or the value of the environment variable
// FQ_GEMM_CUS when it is set to a positive number (tuning and tests: a small value makes small
// problems take the mixed-geometry path).
int planning_cus() {
  if (const char* e = std::getenv("FQ_GEMM_CUS")) {
    const int v = std::atoi(e);
    if (v > 0) return v;
  }
  // per device, filled on first use (a race between threads only repeats the query)
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return -1;
  if (dev < 0 || dev >= kMaxDevices) dev = 0;
  int v = cached[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    hipDeviceProp_t prop;
    v = hipGetDeviceProperties(&prop, dev) == hipSuccess ? prop.multiProcessorCount : -1;
    cached[dev].store(v, std::memory_order_relaxed);
  }
  return v;
}

}  // namespace

void gemm_tile_plan(int nib, int njb, int cus, int out[3]) {
  const TilePlan plan = plan_tiles(nib, njb, cus > 0 ? cus : planning_cus());
  out[0] = plan.n_main;
  out[1] = plan.main_tj;
  out[2] = plan.tail_tj;
}

hipError_t launch_gemm(const GemmParams& p_in, bool debug, hipStream_t st) {
  if (debug) {
    if (p_in.nib * p_in.njb == 0) return hipSuccess;
    hipLaunchKernelGGL(partials_kernel, dim3(p_in.nib * p_in.njb), dim3(256), 0, st, p_in);
    return hipGetLastError();
  }
  if (p_in.nib == 0 || p_in.njb == 0) return hipSuccess;
  GemmParams p = p_in;
  const TilePlan plan = plan_tiles(p.nib, p.njb, planning_cus());
  p.n_main = plan.n_main;
  p.main_tj = plan.main_tj;
  p.tail_tj = plan.tail_tj;
  const int grid = plan.n_main + p.nib * plan.tail_tj;
  // the kernel needs more dynamic LDS than the default limit: raise it once per device
  static std::atomic<bool> attr_set[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
  if (!attr_set[dev].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_biased_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set[dev].store(true, std::memory_order_release);
  }
  if (p.biased) hipLaunchKernelGGL(gemm_biased_kernel, dim3(grid), dim3(kThreads), kLdsBytes, st, p);
  else hipLaunchKernelGGL(gemm_kernel, dim3(grid), dim3(kThreads), kLdsBytes, st, p);
  return hipGetLastError();
}

}  // namespace fq
