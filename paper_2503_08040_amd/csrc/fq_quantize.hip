// Fused block quantizer: abs-max, INT8 codes, fallback decision, residual
// quantization, slot allocation and the compact list of flagged blocks in one
// kernel launch, one pass over the bf16 input.
//
// Paper: Sec. 3.1 (a = max|G|/127, Q^ = round(G/a); round-to-nearest or, for gradients and
// stored contexts, stochastic rounding, Sec. 5.1), Sec. 4.4
// (u = [max|G| > theta]), Sec. 4.3 (second step on the residual G - a Q^),
// Sec. 5.3 (the fallback decision is fused into the quantization kernel).
//
// One 256-thread workgroup owns one 128x128 block (32 KiB of bf16).  Thread t
// holds 4 rows x 16 consecutive columns in registers: column chunk t%8, rows
// t/8 + 32*p.  A 16-column chunk is exactly one lane's 16 bytes of a tile-order
// fragment, so codes leave as 16-byte stores.
#include <type_traits>

#include "fq_device.h"
#include "fq_kernels.h"

namespace fq {

namespace {

constexpr int kThreads = 256;

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// max over the workgroup; every thread gets the result.  red: 4 floats of LDS.
__device__ inline float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();  // red may still be read from a previous call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// sums of two binary64 values over the workgroup; every thread gets both.  red: 8 doubles.
__device__ inline void block_sum2(double& a, double& b, double* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    a += __shfl_xor(a, off, 64);
    b += __shfl_xor(b, off, 64);
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) {
    red[threadIdx.x >> 6] = a;
    red[4 + (threadIdx.x >> 6)] = b;
  }
  __syncthreads();
  a = (red[0] + red[1]) + (red[2] + red[3]);
  b = (red[4] + red[5]) + (red[6] + red[7]);
}

// Philox4x32-10 (Salmon et al., SC'11): counter (c0, c1, 0, 0), key (k0, k1).
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1,
                                     uint32_t (&out)[4]) {
  uint32_t c2 = 0, c3 = 0;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    // one 32 x 32 -> 64-bit multiplication per product (a single instruction on this target)
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t h0 = (uint32_t)(p0 >> 32), l0 = (uint32_t)p0;
    const uint32_t h1 = (uint32_t)(p1 >> 32), l1 = (uint32_t)p1;
    c0 = h1 ^ c1 ^ k0;
    c1 = l1;
    c2 = h0 ^ c3 ^ k1;
    c3 = l0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Stochastic rounding of x/a with the 32-bit random word w: floor + [top 24 bits < fraction].
__device__ inline int quantize_one_sr(float x, float a, uint32_t w) {
  const float t = __fdiv_rn(x, a);
  const float lo = floorf(t);
  const float frac = t - lo;
  float v = lo + (((float)(w >> 8) < frac * 16777216.0f) ? 1.0f : 0.0f);
  v = fminf(fmaxf(v, -127.0f), 127.0f);
  return (int)v;
}

// Register state of a thread: its 4 x 16 input values stay in the packed bf16 form they were
// loaded in (raw[pz][half][dword], two values per dword, low half first) and its codes in
// packed bytes (4 per dword).  Keeping both packed holds the kernel under 128 VGPRs, i.e. four
// workgroups per compute unit: on the tensors this kernel sees (a thousand blocks or so) that
// is the difference between one round of workgroups and a second, nearly empty one.
__device__ inline float x_at(const v4i (&raw)[4][2], int pz, int e) {
  const uint32_t w = (uint32_t)raw[pz][e >> 3][(e & 7) >> 1];
  return __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
}

__device__ inline int code_at(const v4i (&q)[4], int pz, int e) {
  return (int)(int8_t)((uint32_t)q[pz][e >> 2] >> (8 * (e & 3)));
}

// Makes the packed inputs opaque to the optimizer at this point, so that values unpacked
// before it are not kept alive across it (they are cheap to unpack again); emits no code.
__device__ __forceinline__ void forget_unpacked(v4i (&raw)[4][2]) {
#pragma unroll
  for (int pz = 0; pz < 4; ++pz) asm volatile("" : "+v"(raw[pz][0]), "+v"(raw[pz][1]));
}

// Round-to-nearest codes are packed without leaving the float domain: k is an integer-valued
// float in [-127, 127] (rint_quotient clamps where a clamp can matter), k + 128 is exact and lies in [1, 255], and the pack-to-byte
// conversion drops it into byte e % 4 of the row's dword.  finish_codes then turns the four
// bytes of each dword into two's complement: k + 128 and k mod 256 differ in bit 7 only.
__device__ __forceinline__ void put_code_f(v4i& q, int e, float k) {
  q[e >> 2] = (int)__builtin_amdgcn_cvt_pk_u8_f32(k + 128.0f, e & 3,
                                                  (e & 3) ? (unsigned)q[e >> 2] : 0u);
}
__device__ __forceinline__ void finish_codes(v4i& q) {
#pragma unroll
  for (int d = 0; d < 4; ++d) q[d] ^= (int)0x80808080u;
}

__device__ inline void put_code(v4i& q, int e, int code) {
  const int sh = 8 * (e & 3);
  if (sh == 0) q[e >> 2] = code & 0xFF;          // first byte of the dword: no read-modify
  else q[e >> 2] |= (code & 0xFF) << sh;
}

// Writes this thread's 4x16 codes into an LDS image of the transposed block in
// tile order, then the workgroup copies the image out linearly.
__device__ inline void store_transposed(const v4i (&q)[4], int rp, int cc, int8_t* img,
                                        int8_t* dst) {
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int r = p * 32 + rp;
#pragma unroll
    for (int e = 0; e < 16; ++e) img[tile_offset(cc * 16 + e, r)] = (int8_t)code_at(q, p, e);
  }
  __syncthreads();
  const v4i* src = reinterpret_cast<const v4i*>(img);
  v4i* out = reinterpret_cast<v4i*>(dst);
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i * kThreads + threadIdx.x] = src[i * kThreads + threadIdx.x];
}

// Thread (rp, cc) of the workgroup that owns block (bi, bk) loads its 4 x 16 bf16 values
// (rows rp + 32 pz, columns 16 cc ...), zero outside the matrix.
__device__ __forceinline__ void load_block(const QuantParams& p, int bi, int bk, int rp, int cc,
                                  v4i (&raw)[4][2]) {
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

// max |G| of this thread's values
__device__ __forceinline__ float thread_absmax(const v4i (&raw)[4][2]) {
  float m = 0.0f;
#pragma unroll
  for (int pz = 0; pz < 4; ++pz)
#pragma unroll
    for (int e = 0; e < 16; ++e) m = fmaxf(m, fabsf(x_at(raw, pz, e)));
  return m;
}

// The bits block b contributes to its group's word: "decided" and, if u, "flagged".
__device__ inline unsigned long long my_bits(int b, bool u) {
  return (1ull << (b & 31)) | ((u ? 1ull : 0ull) << (32 + (b & 31)));
}

// The ascending list of flagged block ids (the compaction step of the quantizer).  Every
// workgroup records its decision with one 64-bit atomic OR into the word of its group of 32
// blocks (bit b % 32: "decided", bit 32 + b % 32: "flagged"), issued as soon as the decision is
// known so that its round trip hides behind the quantization of the block.  The workgroup whose
// OR completes a group counts the group; the one that counts the last group knows that every
// word is final (each OR was performed before the count it led to) and writes the list from the
// words, which it then clears for the next call.  No fence is needed: the words are only ever
// touched by device-scope atomics.  The list holds the lowest `capacity` ids when more blocks
// are flagged than that.
__device__ inline void write_fb_list(unsigned long long* words, int nb, int capacity,
                                     int32_t* fb_list, int* wave_sum /* LDS, 4 ints */,
                                     int* base_sh /* LDS, 1 int */) {
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int n_words = (nb + 31) >> 5;
  if (t == 0) *base_sh = 0;
  for (int first = 0; first < n_words; first += kThreads) {
    const int wi = first + t;
    uint32_t f = 0;
    if (wi < n_words) {
      f = (uint32_t)(__hip_atomic_load(words + wi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32);
      __hip_atomic_store(words + wi, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int mine = __popc(f);
    int incl = mine;      // inclusive prefix over the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    __syncthreads();   // base_sh / wave_sum of the previous trip have been read
    if (lane == 63) wave_sum[w] = incl;
    __syncthreads();
    int pos = *base_sh + incl - mine;
    for (int j = 0; j < w; ++j) pos += wave_sum[j];
    while (f) {
      const int bit = __ffs(f) - 1;
      f &= f - 1;
      if (pos < capacity) fb_list[pos] = wi * 32 + bit;
      ++pos;
    }
    __syncthreads();
    if (t == 0) *base_sh += wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
  }
}

}  // namespace

// kErr: the fallback decision uses a block quantization-error metric (criteria 3, 4), which
// needs the residual of every block, not only of the flagged ones.
// (The error-metric variants need the block's residuals and two binary64 sums on top of the
// packed state: under the 128-register limit of four workgroups per compute unit they spill,
// and run a quarter faster with two workgroups and no spills.)
template <bool kWantT, bool kStochastic, bool kErr>
__global__ __launch_bounds__(kThreads, kErr ? 2 : 4)
void quantize_kernel(QuantParams p) {
  __shared__ float red[4];
  __shared__ double redd[kErr ? 8 : 1];
  __shared__ int slot_sh, last_sh, scan_base_sh;
  __shared__ int scan_sh[4];
  __shared__ __attribute__((aligned(16))) int8_t img[kWantT ? kBlockBytes : 16];

  const int blk = blockIdx.x;
  const int bi = blk / p.nbc, bk = blk - bi * p.nbc;
  const int t = threadIdx.x;
  const int cc = t & 7, rp = t >> 3;
  const int row0 = bi * kBlock, col0 = bk * kBlock + cc * 16;

  v4i raw[4][2];
  load_block(p, bi, bk, rp, cc, raw);

  // ---- step 1: a = max|G| / 127, codes = round(G / a)           (Sec. 3.1)
  const float m = thread_absmax(raw);
  const float amax = block_max(m, red);
  const float a = __fdiv_rn(amax, 127.0f);
  const float a_rcp = fast_recip(a);
  forget_unpacked(raw);

  // The abs-max decision is known now: take the residual slot right away, so that the round
  // trip of the atomic is hidden behind the quantization of the block.          (Sec. 4.4)
  // a tensor without residual slots has no list to write (nothing can fall back into it)
  const bool want_list = p.capacity > 0;
  bool u = false;
  int slot_early = -1;
  unsigned long long group_before = 0;   // thread 0: the group's word before this block's bits
  if (!kErr) {
    // criterion 5: the decision was taken by topk_select_kernel and is read from the mask
    u = p.crit == 2 || (p.crit == 1 && amax > p.theta) || (p.crit == 5 && p.mask[blk] != 0);
    if (t == 0) {
      if (u) slot_early = atomicAdd(p.fb_count, 1);
      if (want_list) group_before = atomicOr(p.fb_words + (blk >> 5), my_bits(blk, u));
    }
    // a flagged block has twice the work of the others and ends the kernel: it goes first
    if (u) __builtin_amdgcn_s_setprio(3);
  }

  v4i q[4];
  if (!kStochastic) {
#pragma unroll
    for (int pz = 0; pz < 4; ++pz) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        put_code_f(q[pz], e, (a == 0.0f) ? 0.0f : rint_quotient(x_at(raw, pz, e), a, a_rcp, 127.0f));
        // eight elements in flight at a time: bounds the live temporaries
        if ((e & 7) == 7) __builtin_amdgcn_sched_barrier(0);
      }
      finish_codes(q[pz]);
    }
  } else {
    // element (r, c) uses word (r*cols + c) & 3 of the Philox block with counter (r*cols + c) >> 2.
    // A thread's 16 consecutive elements of a row start at word `off` of a block and span 4
    // blocks (off = 0) or 5; off is the same for its four rows (they are 32*cols elements apart).
    const uint32_t k0 = (uint32_t)p.seed, k1 = (uint32_t)(p.seed >> 32);
    auto rows_at = [&](auto off_c) {
      constexpr int off = decltype(off_c)::value;
      constexpr int kBlocks = off ? 5 : 4;
#pragma unroll
      for (int pz = 0; pz < 4; ++pz) {
        const uint64_t e0 = (uint64_t)(row0 + pz * 32 + rp) * (uint64_t)p.cols + (uint64_t)col0;
#pragma unroll
        for (int b = 0; b < kBlocks; ++b) {
          uint32_t w[4];
          const uint64_t ctr = (e0 >> 2) + b;
          philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), k0, k1, w);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int e = 4 * b + i - off;      // compile-time after unrolling
            if (e >= 0 && e < 16)
              put_code(q[pz], e, (a == 0.0f) ? 0 : quantize_one_sr(x_at(raw, pz, e), a, w[i]));
          }
        }
      }
    };
    switch ((int)(((uint64_t)(row0 + rp) * (uint64_t)p.cols + (uint64_t)col0) & 3)) {
      case 0: rows_at(std::integral_constant<int, 0>{}); break;
      case 1: rows_at(std::integral_constant<int, 1>{}); break;
      case 2: rows_at(std::integral_constant<int, 2>{}); break;
      default: rows_at(std::integral_constant<int, 3>{}); break;
    }
  }

  // ---- the block's residual slot, known to the whole workgroup before the codes are stored (the
  // atomic issued after the decision has had the whole quantization to come back; an unflagged
  // block does not look at it at all); with an error-based criterion the decision is only known
  // after the codes, so this runs there.
  int slot = -1;
  auto record_block = [&]() {
    if (t == 0) {
      int slot0 = -1;
      if (u) {
        asm volatile("" : "+v"(slot_early));     // keeps the wait for the atomic inside this branch
        slot0 = (slot_early < p.capacity) ? slot_early : -2;
      }
      slot_sh = slot0;
    }
    __syncthreads();
    slot = slot_sh;
  };
  // ---- per-block outputs: scale, mask, slot.  Stored last, when the wavefront has nothing left
  // to compute: a register that held store data is not reused before the store has completed,
  // and behind these small stores that wait sat in the middle of the quantization.
  auto store_block_record = [&]() {
    if (t == 0) {
      p.scales[blk] = a;
      p.mask[blk] = u ? 1 : 0;
      p.fb_slot[blk] = slot;
      if (blk == 0) *p.fb_count_next = 0;   // ready for the next call into this tensor
    }
  };
  // ---- the list of flagged blocks: the workgroup whose decision completed a group of 32 counts
  // the group, the one that counts the last group writes the list.  Runs when the workgroup has
  // issued all its stores, so that nobody's codes wait for the round trip of the counter.
  auto finish_list = [&]() {
    if (!want_list) return;       // uniform over the grid
    if (t == 0) {
      const int nb = (int)gridDim.x, g = blk >> 5;
      const uint32_t full = (nb - 32 * g >= 32) ? 0xFFFFFFFFu : ((1u << (nb - 32 * g)) - 1u);
      // (both halves of the returned word are named here: a half that nothing reads gives its
      // register away at once, and the write to that register would wait for the atomic)
      asm volatile("" ::"v"(group_before));
      const uint32_t decided = (uint32_t)group_before | (1u << (blk & 31));
      bool last = false;
      if (decided == full) last = atomicAdd(p.fb_groups_done, 1) == ((nb + 31) >> 5) - 1;
      last_sh = last;
    }
    __syncthreads();
    if (last_sh) {      // uniform over the workgroup
      write_fb_list(p.fb_words, (int)gridDim.x, p.capacity, p.fb_list, scan_sh, &scan_base_sh);
      if (t == 0) *p.fb_groups_done = 0;    // ready for the next call
    }
  };
  if (!kErr) record_block();

  forget_unpacked(raw);
  int8_t* cdst = p.codes + (int64_t)blk * kBlockBytes;
#pragma unroll
  for (int pz = 0; pz < 4; ++pz)
    *reinterpret_cast<v4i*>(cdst + tile_offset(pz * 32 + rp, cc * 16)) = q[pz];
  if (kWantT)
    store_transposed(q, rp, cc, img, p.codes_t + ((int64_t)bk * p.nbr + bi) * kBlockBytes);

  // the residual G - a*codes of element (pz, e): one fused multiply-add, single rounding
  auto residual = [&](int pz, int e) {
    return __builtin_fmaf(-(float)code_at(q, pz, e), a, x_at(raw, pz, e));
  };

  // ---- fallback decision by a quantization-error metric          (Sec. 4.4)
  if (kErr) {
    // L1 = sum |G - Q(G)| over the block, L1-Rel = L1 / sum |G|; the sums are binary64
    // accumulations of the binary32 terms (order unspecified), compared with theta in binary64
    double l1 = 0.0, l1x = 0.0;
#pragma unroll
    for (int pz = 0; pz < 4; ++pz)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        l1x += (double)fabsf(x_at(raw, pz, e));
        l1 += (double)fabsf(residual(pz, e));
      }
    block_sum2(l1, l1x, redd);
    if (p.crit == 3) u = l1 > (double)p.theta;
    else u = l1x > 0.0 && l1 / l1x > (double)p.theta;
    if (t == 0) {
      if (u) slot_early = atomicAdd(p.fb_count, 1);
      if (want_list) group_before = atomicOr(p.fb_words + (blk >> 5), my_bits(blk, u));
    }
  }

  if (kErr) record_block();
  if (slot < 0) {        // uniform over the workgroup
    store_block_record();
    finish_list();
    return;
  }

  // ---- step 2: quantize the residual G - a*codes                 (Sec. 4.3)
  // (the residual is recomputed where it is needed instead of being kept in 64 registers)
  float rm = 0.0f;
#pragma unroll
  for (int pz = 0; pz < 4; ++pz)
#pragma unroll
    for (int e = 0; e < 16; ++e) rm = fmaxf(rm, fabsf(residual(pz, e)));
  const float rmax = block_max(rm, red);
  const float ra = __fdiv_rn(rmax, 127.0f);
  const float ra_rcp = fast_recip(ra);
  forget_unpacked(raw);
  v4i rq[4];
#pragma unroll
  for (int pz = 0; pz < 4; ++pz) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      put_code_f(rq[pz], e, (ra == 0.0f) ? 0.0f : rint_quotient(residual(pz, e), ra, ra_rcp, 127.0f));
      if ((e & 7) == 7) __builtin_amdgcn_sched_barrier(0);
    }
    finish_codes(rq[pz]);
  }

  int8_t* rdst = p.res_codes + (int64_t)slot * kBlockBytes;
#pragma unroll
  for (int pz = 0; pz < 4; ++pz)
    *reinterpret_cast<v4i*>(rdst + tile_offset(pz * 32 + rp, cc * 16)) = rq[pz];
  if (kWantT) store_transposed(rq, rp, cc, img, p.res_codes_t + (int64_t)slot * kBlockBytes);
  if (t == 0) p.res_scales[slot] = ra;
  store_block_record();
  finish_list();
}

// ---- TopK AbsMax selection (Sec. 4.4), in three launches: the abs-max of every block, the
// tensor-wide choice of the k largest, then quantize_kernel with that choice as its decision.

// max |G| of each block into amax[nbr * nbc] (the tensor's scale array serves as that buffer
// until quantize_kernel overwrites it with the scales).
__global__ __launch_bounds__(kThreads, 4) void block_absmax_kernel(QuantParams p) {
  __shared__ float red[4];
  const int blk = blockIdx.x;
  const int bi = blk / p.nbc, bk = blk - bi * p.nbc;
  v4i raw[4][2];
  load_block(p, bi, bk, threadIdx.x >> 3, threadIdx.x & 7, raw);
  const float amax = block_max(thread_absmax(raw), red);
  if (threadIdx.x == 0) p.scales[blk] = amax;
}

constexpr int kSelectThreads = 1024;

// mask[b] = 1 for the k blocks with the largest amax (0 < k < nb), equal values in ascending
// block order.  One workgroup: a radix select over the bit patterns (non-negative binary32
// values order like unsigned integers) finds the k-th largest value T in four passes of 8
// bits; then everything above T is flagged, and of the blocks equal to T the first ones in
// index order, as many as are still missing.
__global__ __launch_bounds__(kSelectThreads) void topk_select_kernel(const float* amax, int nb,
                                                                    int k, uint8_t* mask) {
  __shared__ int hist[256], suffix[256];
  __shared__ int sel_bin, sel_want;
  __shared__ int wave_total[kSelectThreads / 64];
  __shared__ int running;
  const int t = threadIdx.x;
  uint32_t prefix = 0, known = 0;
  int want = k;            // the value looked for is the want-th largest among those matching prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (t < 256) hist[t] = 0;
    __syncthreads();
    for (int i = t; i < nb; i += kSelectThreads) {
      const uint32_t b = __float_as_uint(amax[i]);
      if ((b & known) == prefix) atomicAdd(&hist[(b >> shift) & 255], 1);
    }
    __syncthreads();
    // the bin holding the want-th largest candidate: the one whose count of candidates in
    // bins >= it reaches `want` while the count in bins above it does not.  suffix[b] = sum of
    // hist[b..255] by a 256-wide parallel scan.
    if (t < 256) suffix[t] = hist[t];
    __syncthreads();
    for (int step = 1; step < 256; step <<= 1) {
      int add = 0;
      if (t < 256 && t + step < 256) add = suffix[t + step];
      __syncthreads();
      if (t < 256) suffix[t] += add;
      __syncthreads();
    }
    if (t < 256) {
      const int above = t < 255 ? suffix[t + 1] : 0;
      if (suffix[t] >= want && above < want) {
        sel_bin = t;
        sel_want = want - above;
      }
    }
    __syncthreads();
    prefix |= (uint32_t)sel_bin << shift;
    known |= 255u << shift;
    want = sel_want;
    __syncthreads();       // sel_* and hist are rewritten in the next pass
  }
  const uint32_t T = prefix;     // `want` of the blocks equal to T are taken
  if (t == 0) running = 0;
  __syncthreads();
  const int lane = t & 63, w = t >> 6;
  for (int base = 0; base < nb; base += kSelectThreads) {
    const int i = base + t;
    const uint32_t b = i < nb ? __float_as_uint(amax[i]) : 0u;
    const bool eq = i < nb && b == T;
    const unsigned long long ballot = __ballot(eq);
    const int before_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
    if (lane == 0) wave_total[w] = __popcll(ballot);
    __syncthreads();
    int before = running, chunk = 0;
    for (int j = 0; j < kSelectThreads / 64; ++j) {
      if (j < w) before += wave_total[j];
      chunk += wave_total[j];
    }
    if (i < nb) mask[i] = (b > T || (eq && before + before_in_wave < want)) ? 1 : 0;
    __syncthreads();
    if (t == 0) running += chunk;
    __syncthreads();
  }
}

// mask[b] = v for every block (k <= 0 or k >= number of blocks).
__global__ void fill_mask_kernel(uint8_t* mask, int nb, int v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nb) mask[i] = (uint8_t)v;
}

// Clears both slot counters: first use of a tensor, or an empty input.
__global__ void clear_counters_kernel(int32_t* live, int32_t* next, int32_t* groups_done,
                                      unsigned long long* words, int n_words) {
  if (threadIdx.x == 0) {
    *live = 0;
    *next = 0;
    *groups_done = 0;
  }
  for (int i = threadIdx.x; i < n_words; i += blockDim.x) words[i] = 0;
}

// Tile order -> dense row-major (inspection / tests).
__global__ void untile_kernel(const int8_t* tiled, int rows, int cols, int nbc, int8_t* dense) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows * cols) return;
  const int r = (int)(idx / cols), c = (int)(idx - (int64_t)r * cols);
  const int64_t blk = (int64_t)(r >> 7) * nbc + (c >> 7);
  dense[idx] = tiled[blk * kBlockBytes + tile_offset(r & 127, c & 127)];
}

hipError_t launch_quantize(const QuantParams& p, hipStream_t st) {
  if (p.clear_both)
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(256), 0, st, p.fb_count, p.fb_count_next,
                       p.fb_groups_done, p.fb_words, (p.nbr * p.nbc + 31) / 32);
  const int nb = p.nbr * p.nbc;
  if (nb > 0 && p.crit == 5) {
    if (p.topk <= 0 || p.topk >= nb) {
      hipLaunchKernelGGL(fill_mask_kernel, dim3((nb + 255) / 256), dim3(256), 0, st, p.mask, nb,
                         p.topk > 0 ? 1 : 0);
    } else {
      hipLaunchKernelGGL(block_absmax_kernel, dim3(nb), dim3(kThreads), 0, st, p);
      hipLaunchKernelGGL(topk_select_kernel, dim3(1), dim3(kSelectThreads), 0, st, p.scales, nb,
                         p.topk, p.mask);
    }
  }
  if (nb > 0) {
    const dim3 grid(nb), block(kThreads);
    const bool err = p.crit == 3 || p.crit == 4;
    if (p.stochastic) {
      if (p.codes_t) hipLaunchKernelGGL((quantize_kernel<true, true, false>), grid, block, 0, st, p);
      else hipLaunchKernelGGL((quantize_kernel<false, true, false>), grid, block, 0, st, p);
    } else if (err) {
      if (p.codes_t) hipLaunchKernelGGL((quantize_kernel<true, false, true>), grid, block, 0, st, p);
      else hipLaunchKernelGGL((quantize_kernel<false, false, true>), grid, block, 0, st, p);
    } else {
      if (p.codes_t) hipLaunchKernelGGL((quantize_kernel<true, false, false>), grid, block, 0, st, p);
      else hipLaunchKernelGGL((quantize_kernel<false, false, false>), grid, block, 0, st, p);
    }
  }
  return hipGetLastError();
}

hipError_t launch_untile(const int8_t* tiled, int rows, int cols, int8_t* dense, hipStream_t st) {
  const int64_t n = (int64_t)rows * cols;
  if (n == 0) return hipSuccess;
  const int nbc = (cols + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(untile_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, tiled,
                     rows, cols, nbc, dense);
  return hipGetLastError();
}

}  // namespace fq
