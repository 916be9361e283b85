/*
 * fq_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, single-source CPU statement of what Fallback Quantization
 * computes on the linear-layer GEMM path.  It exists so that the HIP library
 * can be checked against something written straight from the paper.  Nothing
 * in the product path may call it; only the test-suite, the smoke check and
 * the benchmark's CPU-baseline leg load this file's shared object.  It shares
 * no source, header, table or helper with the HIP library.
 *
 * What follows which passage of the paper (arXiv 2503.08040):
 *   - block quantization  a = max|G| / 127,  Q^(G) = round(G / a),
 *     dequantization Q(G) = a * Q^(G)                     : Sec. 3.1
 *   - round = round-to-nearest (ties to even)             : Sec. 3.1
 *   - two-step fallback quantization: quantize G, then quantize the residual
 *     dQ(G) = G - Q(G) with a scale of its own            : Sec. 4.3
 *   - fallback indicator u(i,k) = [max|G_ik| > theta]      : Sec. 4.4
 *     (and the selectors the section compares it with: the TopK blocks by
 *     max|G|, and the two error-based ones, L1 = sum|G - Q(G)| and
 *     L1-Rel = L1 / sum|G|, each against theta)
 *   - block GEMM, INT8 x INT8 -> INT32, dequantized by a^A * a^B and
 *     accumulated in FP32                                  : Sec. 4.2, Eq. (1)
 *   - fallback GEMM: k ascending; main term, then, if u(i,k)=1, the residual
 *     term against the same B block                        : Sec. 4.3, Alg. 1
 *   - the three linear-layer products  Y = X W^T,  dX = dY W,  dW = dY^T X
 *                                                          : Sec. 3.2
 *
 * Arithmetic: the paper fixes INT8 codes, INT32 block products and an FP32
 * accumulator.  It does not fix the precision in which a code is decided.
 * Reading taken here: Sec. 3.1 prints a = max|G| / L and round(G / a) as two
 * operations on scale factors it stores in full precision next to bf16 data,
 * so each printed operation is one IEEE binary32 operation (the inputs widen
 * to binary32 exactly), round-to-nearest-even, no contraction (build with
 * -ffp-contract=off), no flush-to-zero:
 *     a  = amax / 127.0f            one division
 *     q  = clamp(rintf(x / a))      one division, one rounding, clamp +-127
 *     r  = fmaf(-(float)q, a, x)    residual, single rounding
 *     a~ = max|r| / 127.0f ;  q~ = clamp(rintf(r / a~))
 *     s  = a^A * a^B                one multiplication
 *     acc = fmaf((float)P, s, acc)  P the exact INT32 block product
 * An all-zero block has a = 0 and all codes 0 (no division is performed).
 * Behaviour on NaN/Inf inputs is not defined by the paper: parity unpinned
 * for non-finite inputs, and they are excluded from every test.
 *
 * Layouts (all host memory, all row-major, caller-allocated):
 *   x_bf16     [rows, ld]            bf16 bit patterns (uint16)
 *   codes      [rows, cols] int8     Q^(G)
 *   scales     [nbr, nbc]   float    a_{i,k},  nbr = ceil(rows/g), nbc = ceil(cols/g)
 *   mask       [nbr, nbc]   uint8    u(i,k)
 *   res_codes  [rows, cols] int8     Q^(dQ(G)); zero outside flagged blocks
 *   res_scales [nbr, nbc]   float    a~_{i,k}; zero outside flagged blocks
 *   fb_list    [nbr*nbc]    int32    ascending ids (bi*nbc+bk) of flagged blocks
 *   fb_count   [1]          int32
 * Ragged edges: an edge block is the elements that exist.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#define FQO_CRIT_NONE 0      /* u == 0 everywhere: plain block INT8, Eq. (1) */
#define FQO_CRIT_ABSMAX_GT 1 /* u = [max|G| > theta], Sec. 4.4            */
#define FQO_CRIT_ALL 2       /* u == 1 everywhere                           */
#define FQO_CRIT_L1_GT 3     /* u = [sum|G - Q(G)| > theta], Sec. 4.4       */
#define FQO_CRIT_L1REL_GT 4  /* u = [sum|G - Q(G)| / sum|G| > theta], Sec. 4.4 */
#define FQO_CRIT_GIVEN 5     /* internal: u is read from `mask` (fqo_quantize_topk) */

#define FQO_OP_NT 0 /* C[M,N] = A[M,K] * B[N,K]^T   (Y  = X  W^T) */
#define FQO_OP_NN 1 /* C[M,K] = A[M,N] * B[N,K]     (dX = dY W)   */
#define FQO_OP_TN 2 /* C[N,K] = A[M,N]^T * B[M,K]   (dW = dY^T X) */

static float bf16_to_f32(uint16_t h) {
  uint32_t w = (uint32_t)h << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return f;
}

/* fp32 -> bf16, round to nearest even (finite inputs). */
static uint16_t f32_to_bf16_rne(float f) {
  uint32_t w;
  memcpy(&w, &f, sizeof w);
  uint32_t lsb = (w >> 16) & 1u;
  w += 0x7FFFu + lsb;
  return (uint16_t)(w >> 16);
}

static int8_t quantize_one(float x, float a) {
  float t = rintf(x / a); /* current rounding mode is the default: ties to even */
  if (t > 127.0f) t = 127.0f;
  if (t < -127.0f) t = -127.0f;
  return (int8_t)t;
}

/* Sec. 3.1 (block quantization), Sec. 4.3 (residual step), Sec. 4.4 (u). */
static int quantize_blocks(const uint16_t *x_bf16, int rows, int cols, long ld, int g,
                           int crit, float theta, int8_t *codes, float *scales,
                           uint8_t *mask, int8_t *res_codes, float *res_scales,
                           int32_t *fb_list, int32_t *fb_count) {
  if (!x_bf16 || !codes || !scales || !mask || !res_codes || !res_scales ||
      !fb_list || !fb_count)
    return -1;
  if (rows < 0 || cols < 0 || g < 1 || ld < cols) return -2;
  if (crit < 0 || crit > FQO_CRIT_GIVEN) return -4;
  int nbr = (rows + g - 1) / g, nbc = (cols + g - 1) / g;
  int n_fb = 0;
  for (int bi = 0; bi < nbr; ++bi) {
    for (int bk = 0; bk < nbc; ++bk) {
      int r0 = bi * g, r1 = r0 + g < rows ? r0 + g : rows;
      int c0 = bk * g, c1 = c0 + g < cols ? c0 + g : cols;
      /* step 1: a = max|G| / L */
      float amax = 0.0f;
      for (int r = r0; r < r1; ++r)
        for (int c = c0; c < c1; ++c) {
          float v = fabsf(bf16_to_f32(x_bf16[(size_t)r * ld + c]));
          if (v > amax) amax = v;
        }
      float a = amax / 127.0f;
      for (int r = r0; r < r1; ++r)
        for (int c = c0; c < c1; ++c) {
          float x = bf16_to_f32(x_bf16[(size_t)r * ld + c]);
          codes[(size_t)r * cols + c] = (a == 0.0f) ? 0 : quantize_one(x, a);
        }
      scales[bi * nbc + bk] = a;
      /* fallback decision */
      int u;
      if (crit == FQO_CRIT_NONE) u = 0;
      else if (crit == FQO_CRIT_ALL) u = 1;
      else if (crit == FQO_CRIT_ABSMAX_GT) u = (amax > theta) ? 1 : 0;
      else if (crit == FQO_CRIT_GIVEN) u = mask[bi * nbc + bk] ? 1 : 0;
      else {
        /* block quantization error L1 = sum |G - Q(G)| and sum |G|, summed in binary64 over
         * the binary32 residuals (the same residual the second step quantizes) */
        double l1 = 0.0, l1x = 0.0;
        for (int r = r0; r < r1; ++r)
          for (int c = c0; c < c1; ++c) {
            float x = bf16_to_f32(x_bf16[(size_t)r * ld + c]);
            float res = fmaf(-(float)codes[(size_t)r * cols + c], a, x);
            l1 += (double)fabsf(res);
            l1x += (double)fabsf(x);
          }
        if (crit == FQO_CRIT_L1_GT) u = (l1 > (double)theta) ? 1 : 0;
        else u = (l1x > 0.0 && l1 / l1x > (double)theta) ? 1 : 0; /* all-zero block: never flagged */
      }
      mask[bi * nbc + bk] = (uint8_t)u;
      /* step 2 (flagged blocks only): quantize the residual G - Q(G) */
      float ra = 0.0f;
      if (u) {
        float rmax = 0.0f;
        for (int r = r0; r < r1; ++r)
          for (int c = c0; c < c1; ++c) {
            float x = bf16_to_f32(x_bf16[(size_t)r * ld + c]);
            float res = fmaf(-(float)codes[(size_t)r * cols + c], a, x);
            float v = fabsf(res);
            if (v > rmax) rmax = v;
          }
        ra = rmax / 127.0f;
        for (int r = r0; r < r1; ++r)
          for (int c = c0; c < c1; ++c) {
            float x = bf16_to_f32(x_bf16[(size_t)r * ld + c]);
            float res = fmaf(-(float)codes[(size_t)r * cols + c], a, x);
            res_codes[(size_t)r * cols + c] =
                (ra == 0.0f) ? 0 : quantize_one(res, ra);
          }
        fb_list[n_fb++] = bi * nbc + bk;
      } else {
        for (int r = r0; r < r1; ++r)
          for (int c = c0; c < c1; ++c) res_codes[(size_t)r * cols + c] = 0;
      }
      res_scales[bi * nbc + bk] = ra;
    }
  }
  *fb_count = n_fb;
  return 0;
}

int fqo_quantize(const uint16_t *x_bf16, int rows, int cols, long ld, int g,
                 int crit, float theta, int8_t *codes, float *scales,
                 uint8_t *mask, int8_t *res_codes, float *res_scales,
                 int32_t *fb_list, int32_t *fb_count) {
  if (crit < 0 || crit > FQO_CRIT_L1REL_GT) return -4;
  return quantize_blocks(x_bf16, rows, cols, ld, g, crit, theta, codes, scales, mask,
                         res_codes, res_scales, fb_list, fb_count);
}

/*
 * TopK AbsMax selection (Sec. 4.4): the k blocks with the largest max|G| fall back
 * (all of them if k is at least the number of blocks, none if k <= 0).  The paper does
 * not say what happens among equal values: here the block with the lower index
 * (bi*nbc + bk) goes first, which makes the selection unique.  Written as k rounds of
 * "take the largest block not taken yet"; everything else is fqo_quantize.
 */
int fqo_quantize_topk(const uint16_t *x_bf16, int rows, int cols, long ld, int g, int k,
                      int8_t *codes, float *scales, uint8_t *mask, int8_t *res_codes,
                      float *res_scales, int32_t *fb_list, int32_t *fb_count) {
  if (!x_bf16 || !mask) return -1;
  if (rows < 0 || cols < 0 || g < 1 || ld < cols) return -2;
  int nbr = (rows + g - 1) / g, nbc = (cols + g - 1) / g, nb = nbr * nbc;
  float *amax = (float *)malloc(sizeof(float) * (size_t)(nb > 0 ? nb : 1));
  if (!amax) return -7;
  for (int bi = 0; bi < nbr; ++bi)
    for (int bk = 0; bk < nbc; ++bk) {
      int r1 = (bi + 1) * g < rows ? (bi + 1) * g : rows;
      int c1 = (bk + 1) * g < cols ? (bk + 1) * g : cols;
      float m = 0.0f;
      for (int r = bi * g; r < r1; ++r)
        for (int c = bk * g; c < c1; ++c) {
          float v = fabsf(bf16_to_f32(x_bf16[(size_t)r * ld + c]));
          if (v > m) m = v;
        }
      amax[bi * nbc + bk] = m;
    }
  for (int b = 0; b < nb; ++b) mask[b] = 0;
  for (int n = 0; n < k && n < nb; ++n) {
    int best = -1;
    for (int b = 0; b < nb; ++b)
      if (!mask[b] && (best < 0 || amax[b] > amax[best])) best = b;
    mask[best] = 1;
  }
  free(amax);
  return quantize_blocks(x_bf16, rows, cols, ld, g, FQO_CRIT_GIVEN, 0.0f, codes, scales, mask,
                         res_codes, res_scales, fb_list, fb_count);
}

/*
 * A quantized operand as the GEMM sees it.  `codes`/`res_codes` are the
 * [rows, cols] arrays written by fqo_quantize; rows/cols are those of the
 * stored matrix (before any transposition the op implies).
 */
typedef struct {
  int rows, cols;
  const int8_t *codes;
  const float *scales;
  const uint8_t *mask;      /* may be NULL for the B operand */
  const int8_t *res_codes;  /* may be NULL when mask is NULL */
  const float *res_scales;
} fqo_operand;

/* Output shape and contraction length of each product. */
static int op_dims(int op, const fqo_operand *A, const fqo_operand *B, int *Mo,
                   int *No, int *Kc) {
  switch (op) {
  case FQO_OP_NT:
    if (A->cols != B->cols) return -2;
    *Mo = A->rows; *No = B->rows; *Kc = A->cols; return 0;
  case FQO_OP_NN:
    if (A->cols != B->rows) return -2;
    *Mo = A->rows; *No = B->cols; *Kc = A->cols; return 0;
  case FQO_OP_TN:
    if (A->rows != B->rows) return -2;
    *Mo = A->cols; *No = B->cols; *Kc = A->rows; return 0;
  default:
    return -4;
  }
}

/* Element (i, t) of the left factor and (t, j) of the right factor, where i, j
 * index the output and t the contraction; and the block-grid index of the
 * quantization block that element lies in. */
static size_t a_elem(int op, const fqo_operand *A, int i, int t) {
  return op == FQO_OP_TN ? (size_t)t * A->cols + i : (size_t)i * A->cols + t;
}
static int a_block(int op, const fqo_operand *A, int g, int i, int t) {
  int nbc = (A->cols + g - 1) / g;
  return op == FQO_OP_TN ? (t / g) * nbc + i / g : (i / g) * nbc + t / g;
}
static size_t b_elem(int op, const fqo_operand *B, int t, int j) {
  return op == FQO_OP_NT ? (size_t)j * B->cols + t : (size_t)t * B->cols + j;
}
static int b_block(int op, const fqo_operand *B, int g, int t, int j) {
  int nbc = (B->cols + g - 1) / g;
  return op == FQO_OP_NT ? (j / g) * nbc + t / g : (t / g) * nbc + j / g;
}

/*
 * Alg. 1 for output rows [i0,i1) and columns [j0,j1).  Output elements are
 * independent, so the tile loops of Alg. 1 are written per element; the
 * k-block loop, the order of the two "+=" inside it and the FP32 accumulator
 * are the algorithm's.  c_f32 (and c_bf16 if not NULL) are full [Mo, No]
 * arrays; only the requested window is written.
 */
int fqo_gemm(int op, const fqo_operand *A, const fqo_operand *B, int g,
             int i0, int i1, int j0, int j1, float *c_f32, uint16_t *c_bf16) {
  if (!A || !B || !c_f32 || !A->codes || !A->scales || !B->codes || !B->scales)
    return -1;
  if (A->mask && (!A->res_codes || !A->res_scales)) return -1;
  if (g < 1) return -3;
  int Mo, No, Kc, rc = op_dims(op, A, B, &Mo, &No, &Kc);
  if (rc) return rc;
  if (i0 < 0 || i1 > Mo || j0 < 0 || j1 > No) return -2;
  int nkb = (Kc + g - 1) / g;
#pragma omp parallel for schedule(dynamic, 8)
  for (int i = i0; i < i1; ++i) {
    for (int j = j0; j < j1; ++j) {
      float acc = 0.0f;
      for (int kb = 0; kb < nkb; ++kb) {
        int t0 = kb * g, t1 = t0 + g < Kc ? t0 + g : Kc;
        int ab = a_block(op, A, g, i, t0), bb = b_block(op, B, g, t0, j);
        int32_t P = 0;
        for (int t = t0; t < t1; ++t)
          P += (int32_t)A->codes[a_elem(op, A, i, t)] *
               (int32_t)B->codes[b_elem(op, B, t, j)];
        float s = A->scales[ab] * B->scales[bb];
        acc = fmaf((float)P, s, acc);
        if (A->mask && A->mask[ab]) {
          int32_t Pr = 0;
          for (int t = t0; t < t1; ++t)
            Pr += (int32_t)A->res_codes[a_elem(op, A, i, t)] *
                  (int32_t)B->codes[b_elem(op, B, t, j)];
          float sr = A->res_scales[ab] * B->scales[bb];
          acc = fmaf((float)Pr, sr, acc);
        }
      }
      c_f32[(size_t)i * No + j] = acc;
      if (c_bf16) c_bf16[(size_t)i * No + j] = f32_to_bf16_rne(acc);
    }
  }
  return 0;
}

/* The INT32 block product of one k-block (main or residual term) for the
 * window [i0,i1) x [j0,j1); p_out is a full [Mo, No] array.  The residual
 * product of an unflagged block is 0. */
int fqo_gemm_partials(int op, const fqo_operand *A, const fqo_operand *B, int g,
                      int kb, int residual_term, int i0, int i1, int j0,
                      int j1, int32_t *p_out) {
  if (!A || !B || !p_out || !A->codes || !B->codes) return -1;
  if (residual_term && (!A->mask || !A->res_codes)) return -1;
  if (g < 1) return -3;
  int Mo, No, Kc, rc = op_dims(op, A, B, &Mo, &No, &Kc);
  if (rc) return rc;
  int nkb = (Kc + g - 1) / g;
  if (kb < 0 || kb >= nkb) return -2;
  if (i0 < 0 || i1 > Mo || j0 < 0 || j1 > No) return -2;
  int t0 = kb * g, t1 = t0 + g < Kc ? t0 + g : Kc;
  const int8_t *ac = residual_term ? A->res_codes : A->codes;
  for (int i = i0; i < i1; ++i)
    for (int j = j0; j < j1; ++j) {
      int32_t P = 0;
      if (!residual_term || A->mask[a_block(op, A, g, i, t0)])
        for (int t = t0; t < t1; ++t)
          P += (int32_t)ac[a_elem(op, A, i, t)] *
               (int32_t)B->codes[b_elem(op, B, t, j)];
      p_out[(size_t)i * No + j] = P;
    }
  return 0;
}

/* ------------------------------------------------------------------------
 * Stochastic rounding (Sec. 3.1: round x up to ceil(x) with probability
 * x - floor(x), down otherwise; E[Q_s(x)] = x) for the tensors the paper
 * quantizes that way: the output gradient dY and the stored activation
 * context X (Sec. 5.1, Sec. 5.3), both plain block INT8 without fallback.
 *
 * The paper does not say where the random numbers come from.  Reading used
 * here: element (r, c) of the matrix draws one 32-bit word from the
 * counter-based generator Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel
 * random numbers: as easy as 1, 2, 3", SC'11) with key = the 64-bit seed and
 * counter = (e >> 2) for e = r*cols + c, taking output word e & 3; its top 24
 * bits u are compared with the fraction:  q = floor(t) + [u < (t-floor(t))*2^24],
 * t = x/a in binary32 (all operations exact or single IEEE operations).
 * Parity unpinned for non-finite inputs, as for round-to-nearest.
 * ------------------------------------------------------------------------ */
static void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                          uint32_t k0, uint32_t k1, uint32_t out[4]) {
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Exposed so that the generator itself can be pinned to published test vectors. */
void fqo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1], out);
}

static uint32_t sr_word(uint64_t seed, uint64_t e) {
  uint32_t o[4];
  uint64_t ctr = e >> 2;
  philox4x32_10((uint32_t)ctr, (uint32_t)(ctr >> 32), 0u, 0u, (uint32_t)seed,
                (uint32_t)(seed >> 32), o);
  return o[e & 3];
}

int fqo_quantize_sr(const uint16_t *x_bf16, int rows, int cols, long ld, int g,
                    uint64_t seed, int8_t *codes, float *scales) {
  if (!x_bf16 || !codes || !scales) return -1;
  if (rows < 0 || cols < 0 || g < 1 || ld < cols) return -2;
  int nbr = (rows + g - 1) / g, nbc = (cols + g - 1) / g;
  for (int bi = 0; bi < nbr; ++bi)
    for (int bk = 0; bk < nbc; ++bk) {
      int r0 = bi * g, r1 = r0 + g < rows ? r0 + g : rows;
      int c0 = bk * g, c1 = c0 + g < cols ? c0 + g : cols;
      float amax = 0.0f;
      for (int r = r0; r < r1; ++r)
        for (int c = c0; c < c1; ++c) {
          float v = fabsf(bf16_to_f32(x_bf16[(size_t)r * ld + c]));
          if (v > amax) amax = v;
        }
      float a = amax / 127.0f;
      scales[bi * nbc + bk] = a;
      for (int r = r0; r < r1; ++r)
        for (int c = c0; c < c1; ++c) {
          int8_t q = 0;
          if (a != 0.0f) {
            float t = bf16_to_f32(x_bf16[(size_t)r * ld + c]) / a;
            float lo = floorf(t);
            float frac = t - lo;                       /* exact */
            uint32_t u = sr_word(seed, (uint64_t)r * (uint64_t)cols + (uint64_t)c) >> 8;
            float v = lo + (((float)u < frac * 16777216.0f) ? 1.0f : 0.0f);
            if (v > 127.0f) v = 127.0f;
            if (v < -127.0f) v = -127.0f;
            q = (int8_t)v;
          }
          codes[(size_t)r * cols + c] = q;
        }
    }
  return 0;
}

/* ------------------------------------------------------------------------
 * Delay Threshold (App. D, Alg. 2): after a training step, a layer's threshold
 * is divided by alpha if its fallback rate was below r_min, multiplied by alpha
 * if it was above r_max, left alone otherwise.  theta starts at 1.
 * ------------------------------------------------------------------------ */
float fqo_threshold_update(float theta, int n_fallback, int n_blocks, float r_min,
                           float r_max, float alpha) {
  if (n_blocks <= 0) return theta;
  /* the rate is formed in binary32 like the bounds it is compared with, so that a rate of
   * exactly r_min or r_max (e.g. 10 of 100 blocks against 0.1f) counts as inside the range */
  float rate = (float)n_fallback / (float)n_blocks;
  if (rate < r_min) return theta / alpha;
  if (rate > r_max) return theta * alpha;
  return theta;
}

/* ------------------------------------------------------------------------
 * Activation-context compression for non-linear layers (Sec. 5.2, 5.3): the
 * input of a normalization / activation function is kept for the backward pass
 * as 10-bit integers with one scale per 1 x 128 group (one token, 128 channels),
 * "5/8 of BF16", and dequantized again in the backward pass.
 *   a = max|G| / 511,  q = round-to-nearest-even(x / a) in [-511, 511]  (Sec. 3.1 with L = 511;
 *   the paper does not state the rounding of contexts: round-to-nearest is the reading here),
 *   dequantized value = a * q, rounded to bf16 (the layers work in bf16).
 * Packed format (not fixed by the paper): a group is 160 bytes, value i (two's complement,
 * 10 bits) occupies bits [10 i, 10 i + 10) of the group's little-endian bit string; row r,
 * group j starts at byte (r * ngroups + j) * 160; absent elements of a ragged last group are 0.
 * Arithmetic in binary32 as for the block quantizer.
 * ------------------------------------------------------------------------ */
int fqo_ctx_quantize(const uint16_t *x_bf16, int rows, int cols, long ld, uint8_t *packed,
                     float *scales) {
  if (!x_bf16 || !packed || !scales) return -1;
  if (rows < 0 || cols < 0 || ld < cols) return -2;
  const int G = 128, ng = (cols + G - 1) / G;
  for (int r = 0; r < rows; ++r)
    for (int j = 0; j < ng; ++j) {
      int c0 = j * G, c1 = c0 + G < cols ? c0 + G : cols;
      float amax = 0.0f;
      for (int c = c0; c < c1; ++c) {
        float v = fabsf(bf16_to_f32(x_bf16[(size_t)r * ld + c]));
        if (v > amax) amax = v;
      }
      float a = amax / 511.0f;
      scales[(size_t)r * ng + j] = a;
      uint8_t *dst = packed + ((size_t)r * ng + j) * 160;
      memset(dst, 0, 160);
      for (int c = c0; c < c1; ++c) {
        int q = 0;
        if (a != 0.0f) {
          float t = rintf(bf16_to_f32(x_bf16[(size_t)r * ld + c]) / a);
          if (t > 511.0f) t = 511.0f;
          if (t < -511.0f) t = -511.0f;
          q = (int)t;
        }
        uint32_t bits = (uint32_t)q & 0x3FFu;
        int pos = (c - c0) * 10;
        for (int b = 0; b < 10; ++b)
          if (bits & (1u << b)) dst[(pos + b) >> 3] |= (uint8_t)(1u << ((pos + b) & 7));
      }
    }
  return 0;
}

int fqo_ctx_dequantize(const uint8_t *packed, const float *scales, int rows, int cols,
                       uint16_t *out_bf16, long ldo) {
  if (!packed || !scales || !out_bf16) return -1;
  if (rows < 0 || cols < 0 || ldo < cols) return -2;
  const int G = 128, ng = (cols + G - 1) / G;
  for (int r = 0; r < rows; ++r)
    for (int c = 0; c < cols; ++c) {
      int j = c / G, pos = (c - j * G) * 10;
      const uint8_t *src = packed + ((size_t)r * ng + j) * 160;
      uint32_t bits = 0;
      for (int b = 0; b < 10; ++b)
        if (src[(pos + b) >> 3] & (1u << ((pos + b) & 7))) bits |= 1u << b;
      int q = (bits & 0x200u) ? (int)bits - 1024 : (int)bits;   /* sign-extend 10 bits */
      float v = scales[(size_t)r * ng + j] * (float)q;
      out_bf16[(size_t)r * ldo + c] = f32_to_bf16_rne(v);
    }
  return 0;
}

/*
 * Gated linear unit y = sigma(x1) * x2 with sigma = SiLU, sigma(x) = x / (1 + e^-x) (Sec. 4.1),
 * as a non-linear layer of Sec. 5.2: bf16 inputs and output; what it keeps for the backward
 * pass are the INT10 1 x 128 contexts of x1 and x2 (fqo_ctx_quantize), which the backward pass
 * dequantizes (Sec. 5.3).  The function values are evaluated in binary64 and rounded once to
 * bf16.
 */
static uint16_t f64_to_bf16_rne(double v) {
  /* a double rounded once to bf16 (8 significant bits, ties to even; below 2^-126 the spacing
   * is 2^-133); finite inputs.  rint() uses the default rounding mode: ties to even. */
  if (v == 0.0) return signbit(v) ? 0x8000u : 0u;
  int e;
  (void)frexp(fabs(v), &e);                        /* |v| = m * 2^e, 0.5 <= m < 1 */
  int quantum = e - 8 < -133 ? -133 : e - 8;       /* exponent of the bf16 spacing at |v| */
  double r = ldexp(rint(ldexp(fabs(v), -quantum)), quantum);
  return f32_to_bf16_rne((float)copysign(r, v));   /* r is a bf16 value: both conversions exact */
}

int fqo_glu_forward(const uint16_t *x1_bf16, const uint16_t *x2_bf16, int rows, int cols,
                    long ld, uint16_t *y_bf16, long ldy) {
  if (!x1_bf16 || !x2_bf16 || !y_bf16) return -1;
  if (rows < 0 || cols < 0 || ld < cols || ldy < cols) return -2;
  for (int r = 0; r < rows; ++r)
    for (int c = 0; c < cols; ++c) {
      double x1 = (double)bf16_to_f32(x1_bf16[(size_t)r * ld + c]);
      double x2 = (double)bf16_to_f32(x2_bf16[(size_t)r * ld + c]);
      double silu = x1 / (1.0 + exp(-x1));
      y_bf16[(size_t)r * ldy + c] = f64_to_bf16_rne(silu * x2);
    }
  return 0;
}

/* Value of element (r, c) of an INT10 context: scale * code, one binary32 multiplication. */
static float ctx_value(const uint8_t *packed, const float *scales, int ng, int r, int c) {
  const int G = 128, j = c / G, pos = (c - j * G) * 10;
  const uint8_t *src = packed + ((size_t)r * ng + j) * 160;
  uint32_t bits = 0;
  for (int b = 0; b < 10; ++b)
    if (src[(pos + b) >> 3] & (1u << ((pos + b) & 7))) bits |= 1u << b;
  int q = (bits & 0x200u) ? (int)bits - 1024 : (int)bits;
  return scales[(size_t)r * ng + j] * (float)q;
}

/* dx2 = dy * silu(x1~), dx1 = dy * x2~ * silu'(x1~), silu'(x) = s (1 + x (1 - s)), s = 1/(1+e^-x),
 * with x1~, x2~ the dequantized contexts; binary64 evaluation, one rounding to bf16. */
int fqo_glu_backward(const uint16_t *dy_bf16, long ld_dy, const uint8_t *packed1,
                     const float *scales1, const uint8_t *packed2, const float *scales2,
                     int rows, int cols, uint16_t *dx1_bf16, uint16_t *dx2_bf16, long ldo) {
  if (!dy_bf16 || !packed1 || !scales1 || !packed2 || !scales2 || !dx1_bf16 || !dx2_bf16)
    return -1;
  if (rows < 0 || cols < 0 || ld_dy < cols || ldo < cols) return -2;
  const int ng = (cols + 127) / 128;
  for (int r = 0; r < rows; ++r)
    for (int c = 0; c < cols; ++c) {
      double dy = (double)bf16_to_f32(dy_bf16[(size_t)r * ld_dy + c]);
      double x1 = (double)ctx_value(packed1, scales1, ng, r, c);
      double x2 = (double)ctx_value(packed2, scales2, ng, r, c);
      double s = 1.0 / (1.0 + exp(-x1));
      double silu = x1 * s, dsilu = s * (1.0 + x1 * (1.0 - s));
      dx2_bf16[(size_t)r * ldo + c] = f64_to_bf16_rne(dy * silu);
      dx1_bf16[(size_t)r * ldo + c] = f64_to_bf16_rne(dy * x2 * dsilu);
    }
  return 0;
}

/*
 * RMS normalization y = x * rstd * w, rstd = 1 / sqrt(mean(x^2) + eps) per row, as a non-linear
 * layer of Sec. 5.2: bf16 input, gain and output; what it keeps for the backward pass is the
 * INT10 1 x 128 context of x (fqo_ctx_quantize) and rstd per row (binary32).  Evaluated in
 * binary64, each result rounded once.
 */
int fqo_rmsnorm_forward(const uint16_t *x_bf16, const uint16_t *w_bf16, int rows, int cols,
                        long ld, double eps, uint16_t *y_bf16, long ldy, float *rstd) {
  if (!x_bf16 || !w_bf16 || !y_bf16 || !rstd) return -1;
  if (rows < 0 || cols < 1 || ld < cols || ldy < cols) return -2;
  for (int r = 0; r < rows; ++r) {
    double ss = 0.0;
    for (int c = 0; c < cols; ++c) {
      double x = (double)bf16_to_f32(x_bf16[(size_t)r * ld + c]);
      ss += x * x;
    }
    double rs = 1.0 / sqrt(ss / (double)cols + eps);
    rstd[r] = (float)rs;
    for (int c = 0; c < cols; ++c) {
      double x = (double)bf16_to_f32(x_bf16[(size_t)r * ld + c]);
      double w = (double)bf16_to_f32(w_bf16[c]);
      y_bf16[(size_t)r * ldy + c] = f64_to_bf16_rne(x * rs * w);
    }
  }
  return 0;
}

/*
 * Backward of the RMS normalization from dy, the INT10 context of x, the stored rstd and the
 * gain: with x~ the dequantized context, xh = x~ * rstd, g = dy * w,
 *   dx = rstd * (g - xh * mean(g * xh)),     dw[c] = sum over rows of dy * xh.
 * Binary64 evaluation; dx rounded once to bf16, dw to binary32.
 */
int fqo_rmsnorm_backward(const uint16_t *dy_bf16, long ld_dy, const uint8_t *packed,
                         const float *scales, const float *rstd, const uint16_t *w_bf16,
                         int rows, int cols, uint16_t *dx_bf16, long ldo, float *dw) {
  if (!dy_bf16 || !packed || !scales || !rstd || !w_bf16 || !dx_bf16 || !dw) return -1;
  if (rows < 0 || cols < 1 || ld_dy < cols || ldo < cols) return -2;
  const int ng = (cols + 127) / 128;
  double *acc = (double *)calloc((size_t)cols, sizeof(double));
  if (!acc) return -7;
  for (int r = 0; r < rows; ++r) {
    const double rs = (double)rstd[r];
    double m = 0.0;
    for (int c = 0; c < cols; ++c) {
      double xh = (double)ctx_value(packed, scales, ng, r, c) * rs;
      double g = (double)bf16_to_f32(dy_bf16[(size_t)r * ld_dy + c]) * (double)bf16_to_f32(w_bf16[c]);
      m += g * xh;
    }
    m /= (double)cols;
    for (int c = 0; c < cols; ++c) {
      double xh = (double)ctx_value(packed, scales, ng, r, c) * rs;
      double dy = (double)bf16_to_f32(dy_bf16[(size_t)r * ld_dy + c]);
      double g = dy * (double)bf16_to_f32(w_bf16[c]);
      dx_bf16[(size_t)r * ldo + c] = f64_to_bf16_rne(rs * (g - xh * m));
      acc[c] += dy * xh;
    }
  }
  for (int c = 0; c < cols; ++c) dw[c] = (float)acc[c];
  free(acc);
  return 0;
}

/* Number of OpenMP threads fqo_gemm will use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int fqo_num_threads(void) { return omp_get_max_threads(); }
#else
int fqo_num_threads(void) { return 1; }
#endif
