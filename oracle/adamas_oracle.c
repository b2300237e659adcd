/*
 * adamas_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, scalar CPU statement of what the Adamas decode-time sparse
 * attention path computes (Algorithm 1 of the paper), written from the
 * paper's definitions.  It exists only so that tests, the smoke check and
 * the bench's cpu_baseline leg have something independent to compare the
 * GPU library against.  It shares no code, header, table or constant with
 * the HIP path and must never be called from it.
 *
 * Every stage is the plain definition, not a fast algorithm:
 *   - Hadamard matrix: Kronecker recursion from H_2 (Section 2, Eq. 2),
 *     kept as integer +-1 entries; the 1/sqrt(d) normalisation is applied to
 *     the thresholds instead of to every coefficient.  For d = 2^n * m with
 *     m = 12 or 20 the recursion starts from a Hadamard matrix of order m
 *     (Section 2, the construction H_d = H_{2^n} (x) H_m under Eq. 2); the paper
 *     names no H_12 / H_20, this file uses Paley's (see oracle_hadamard_matrix).
 *   - Transform: dense d-term sums y_j = sum_i x_i * H[i][j] in double
 *     (Section 3.2, Eq. 4).
 *   - Bucketize: code = number of thresholds strictly below the value
 *     (Eq. 5).
 *   - Compress: 2-bit codes, eight per 16 bits, 32 bytes per 128-d vector
 *     (Section 3.2, paragraph after Eq. 5).  Bit placement is this build's
 *     reading: the paper does not give one.
 *   - Manhattan distance on the unpacked codes (Eq. 6).
 *   - Top-k: k smallest distances by a full sort, ties to the lower index
 *     (Algorithm 1, top-k step; the tie rule is this build's, the paper has none).
 *   - Sparse attention: Eq. 1 on the original q, K, V restricted to the
 *     selected rows (Algorithm 1, gather and attention steps), in double.
 *
 * Pins (see tests/test_oracle_*.py): H H^T = d I, H[i][j] = (-1)^popcount(i&j),
 * transform twice = d * identity exactly, Parseval, (QH)(KH)^T = d QK^T,
 * scipy's Hadamard matrix, brute-force subset enumeration for top-k,
 * k = L reduces to full attention, closed forms for one row / equal scores.
 * Parity with the authors' own cache bytes is UNPINNED: thresholds and bit
 * order are not in the paper.
 *
 * Exactness precondition for the transform (so that the dense double sums
 * are the exact real-arithmetic values and bucket decisions do not depend on
 * summation order): all inputs finite, and within one vector the exponents
 * of the largest and the smallest non-zero magnitude differ by at most 38.
 * oracle_encode() checks this per vector and fails (-2) when it is violated.
 */

#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/*
 * Head dimension.  The paper's models have d = 128 and that is the default;
 * Section 2 builds the transform for any power of two (H_{2n} from H_n) and
 * for d = 2^n * m with m the order of a known Hadamard matrix, and
 * oracle_set_head_dim() switches every function below to another supported d
 * (test code sets it before a group of calls and restores 128 afterwards; it
 * is process-wide state, only read inside the calls).  A 2-bit code row then
 * has d / 4 bytes: d / 32 words of two 32-bit planes, so d must be a multiple
 * of 32.
 */
#define ORACLE_MAX_D 256
static int oracle_head_dim = 128;
#define ORACLE_D (oracle_head_dim)
#define ORACLE_ROW_BYTES (oracle_head_dim / 4)

/* m with d = 2^n * m, m in {1, 12, 20}; 0 if d is not of that form. */
static int hadamard_base_order(int d) {
  if (d < 1) return 0;
  while (d % 2 == 0 && d != 12 && d != 20) d /= 2;
  return (d == 1 || d == 12 || d == 20) ? d : 0;
}

int oracle_set_head_dim(int d) {
  if (d < 32 || d > ORACLE_MAX_D || d % 32 != 0 || hadamard_base_order(d) == 0) return -1;
  oracle_head_dim = d;
  return 0;
}

int oracle_get_head_dim(void) { return oracle_head_dim; }

enum {
  ORACLE_OK = 0,
  ORACLE_BAD_ARG = -1,
  ORACLE_PRECONDITION = -2,
  ORACLE_NOMEM = -3
};

/* ------------------------------------------------------------------ bf16 */

/* A bf16 value is the top 16 bits of an IEEE binary32: widening is exact. */
static double bf16_to_double(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* --------------------------------------------------- Hadamard matrix, Eq. 2 */

/*
 * Paley's Hadamard matrix of order m = q + 1 for a prime q = 3 (mod 4) (q = 11
 * and 19 give the orders 12 and 20 that Section 2's construction needs; the
 * paper does not say which H_12 / H_20 its authors use, so this choice is this
 * build's):  with chi the quadratic character mod q (chi(0) = 0, +1 for the
 * non-zero squares, -1 otherwise),
 *     P[0][0] = 1,  P[0][j] = 1,  P[i][0] = -1,  P[i][i] = 1,
 *     P[i][j] = chi(i - j)   for i != j, i, j >= 1.
 * P P^T = m I because the q x q matrix chi(i - j) is antisymmetric for
 * q = 3 (mod 4) and has Q Q^T = q I - J, Q J = 0.  P is not symmetric.
 */
static void paley_matrix(int q, int8_t *P, int stride) {
  int m = q + 1;
  int8_t chi[32];
  for (int a = 0; a < q; ++a) chi[a] = -1;
  chi[0] = 0;
  for (int a = 1; a < q; ++a) chi[(a * a) % q] = 1; /* the non-zero squares */
  for (int i = 0; i < m; ++i) {
    for (int j = 0; j < m; ++j) {
      int8_t v;
      if (i == 0) v = 1;
      else if (j == 0) v = -1;
      else if (i == j) v = 1;
      else v = chi[(((i - j) % q) + q) % q];
      P[i * stride + j] = v;
    }
  }
}

/*
 * Fills H (d*d, row-major, entries +1/-1).  d = 2^n: the Kronecker recursion
 * H_{2k} = H_2 (x) H_k = [[H_k, H_k], [H_k, -H_k]] from H_1 = [1] (Eq. 2).
 * d = 2^n * 12 or 2^n * 20: the same recursion started from Paley's matrix of
 * order 12 / 20, which is H_{2^n} (x) H_m (Section 2, under Eq. 2):
 *     H[a * m + b][a' * m + b'] = H_{2^n}[a][a'] * H_m[b][b'].
 * The factor 1/sqrt(2) per level (1/sqrt(d) in all) is left out: the
 * orthonormal matrix is H / sqrt(d).
 */
int oracle_hadamard_matrix(int d, int8_t *H) {
  int m = hadamard_base_order(d);
  if (m == 0 || !H) return ORACLE_BAD_ARG;
  if (m == 1) H[0] = 1;
  else paley_matrix(m - 1, H, d);
  for (int n = m; n < d; n *= 2) {
    /* grow the n x n block in the top-left corner (stride d) to 2n x 2n */
    for (int i = 0; i < n; ++i) {
      for (int j = 0; j < n; ++j) {
        int8_t v = H[i * d + j];
        H[i * d + (j + n)] = v;
        H[(i + n) * d + j] = v;
        H[(i + n) * d + (j + n)] = (int8_t)(-v);
      }
    }
  }
  return ORACLE_OK;
}

/* ------------------------------------------------ transform, Eq. 4 (dense) */

/*
 * y = x H with the +-1 matrix: y_j = sum_i x_i H[i][j], i ascending, double.
 * The orthonormal transform of the paper is y / sqrt(d).
 */
int oracle_hadamard_transform(int d, const double *x, double *y) {
  if (hadamard_base_order(d) == 0 || !x || !y) return ORACLE_BAD_ARG;
  int8_t *H = (int8_t *)malloc((size_t)d * d);
  if (!H) return ORACLE_NOMEM;
  oracle_hadamard_matrix(d, H);
  for (int j = 0; j < d; ++j) {
    double s = 0.0;
    for (int i = 0; i < d; ++i) s += x[i] * (double)H[i * d + j];
    y[j] = s;
  }
  free(H);
  return ORACLE_OK;
}

/* ---------------------------------------------------------- bucketize, Eq. 5 */

/*
 * Thresholds are given on the orthonormal scale (thr[0] < thr[1] < thr[2]);
 * the n values y are unnormalised sums of a transform of order d, so each
 * threshold is scaled once by sqrt(d) in double:
 * tau_i = (double)thr[i] * sqrt((double)d).
 * code = #{ i : y > tau_i }  (strict: y == tau_i falls in the lower bucket).
 */
#define ORACLE_MAX_THR 7 /* 3-bit codes */

static void scaled_thresholds(int d, const float *thr, int nthr, double *tau) {
  double root = sqrt((double)d);
  for (int i = 0; i < nthr; ++i) tau[i] = (double)thr[i] * root;
}

static int increasing(const float *thr, int nthr) {
  for (int i = 0; i + 1 < nthr; ++i)
    if (!(thr[i] < thr[i + 1])) return 0;
  return thr[0] == thr[0]; /* not NaN */
}

/* Eq. 5 with nthr thresholds (1, 3 or 7 for the 1-, 2-, 3-bit codes of Section 4.4). */
int oracle_bucketize_n(int64_t n, const double *y, int d, const float *thr, int nthr,
                       uint8_t *code) {
  if (n < 0 || d < 1 || !y || !thr || !code || nthr < 1 || nthr > ORACLE_MAX_THR)
    return ORACLE_BAD_ARG;
  if (!increasing(thr, nthr)) return ORACLE_BAD_ARG;
  double tau[ORACLE_MAX_THR];
  scaled_thresholds(d, thr, nthr, tau);
  for (int64_t j = 0; j < n; ++j) {
    int c = 0;
    for (int i = 0; i < nthr; ++i)
      if (y[j] > tau[i]) ++c;
    code[j] = (uint8_t)c;
  }
  return ORACLE_OK;
}

int oracle_bucketize(int64_t n, const double *y, int d, const float thr[3], uint8_t *code) {
  return oracle_bucketize_n(n, y, d, thr, 3, code);
}

/* ------------------------------------------------------------------ compress */

/*
 * Row layout (this build's reading; the paper fixes only the density of
 * eight codes per 16 bits): 32 bytes = four little-endian 64-bit words.
 * Word g holds dimensions 32g .. 32g+31: bit j is the low bit of the code of
 * dimension 32g+j, bit 32+j its high bit.
 */
int oracle_pack_row(const uint8_t *code, uint8_t *row) {
  if (!code || !row) return ORACLE_BAD_ARG;
  memset(row, 0, ORACLE_ROW_BYTES);
  for (int dim = 0; dim < ORACLE_D; ++dim) {
    if (code[dim] > 3) return ORACLE_BAD_ARG;
    int g = dim / 32, j = dim % 32;
    int low = code[dim] & 1, high = (code[dim] >> 1) & 1;
    int bit_low = j, bit_high = 32 + j; /* bit positions inside the 64-bit word */
    if (low) row[g * 8 + bit_low / 8] |= (uint8_t)(1u << (bit_low % 8));
    if (high) row[g * 8 + bit_high / 8] |= (uint8_t)(1u << (bit_high % 8));
  }
  return ORACLE_OK;
}

int oracle_unpack_row(const uint8_t *row, uint8_t *code) {
  if (!code || !row) return ORACLE_BAD_ARG;
  for (int dim = 0; dim < ORACLE_D; ++dim) {
    int g = dim / 32, j = dim % 32;
    int bit_low = j, bit_high = 32 + j;
    int low = (row[g * 8 + bit_low / 8] >> (bit_low % 8)) & 1;
    int high = (row[g * 8 + bit_high / 8] >> (bit_high % 8)) & 1;
    code[dim] = (uint8_t)(low + 2 * high);
  }
  return ORACLE_OK;
}

/*
 * The same layout for the 1-bit and 3-bit codes of the bucketization ablation
 * (Section 4.4): a row is 16 * bits bytes = four words of `bits` little-endian
 * 32-bit planes; plane p of word g holds, at bit j, bit p of the code of
 * dimension 32g + j.  bits = 2 gives exactly the 32-byte row above.
 */
int oracle_pack_row_bits(const uint8_t code[ORACLE_MAX_D], int bits, uint8_t *row) {
  if (!code || !row || bits < 1 || bits > 3) return ORACLE_BAD_ARG;
  memset(row, 0, (size_t)(ORACLE_D / 8) * bits);
  for (int dim = 0; dim < ORACLE_D; ++dim) {
    if (code[dim] >> bits) return ORACLE_BAD_ARG;
    int g = dim / 32, j = dim % 32;
    for (int p = 0; p < bits; ++p)
      if ((code[dim] >> p) & 1) row[(g * bits + p) * 4 + j / 8] |= (uint8_t)(1u << (j % 8));
  }
  return ORACLE_OK;
}

int oracle_unpack_row_bits(const uint8_t *row, int bits, uint8_t code[ORACLE_MAX_D]) {
  if (!code || !row || bits < 1 || bits > 3) return ORACLE_BAD_ARG;
  for (int dim = 0; dim < ORACLE_D; ++dim) {
    int g = dim / 32, j = dim % 32, c = 0;
    for (int p = 0; p < bits; ++p) c |= ((row[(g * bits + p) * 4 + j / 8] >> (j % 8)) & 1) << p;
    code[dim] = (uint8_t)c;
  }
  return ORACLE_OK;
}

/* ------------------------------------- encode = transform + bucketize + pack */

/*
 * x: n vectors of 128 bf16 bit patterns, contiguous.  Writes, when non-NULL,
 * codes (n*128 bytes, values 0..3) and rows (n*32 bytes, packed).
 * Returns ORACLE_PRECONDITION if a vector holds NaN/Inf or its exponent
 * spread is too large for the double sums to be exact (see file header).
 */
int oracle_encode_variant(const uint16_t *x, int64_t n, const float thr[3], int use_hadamard,
                          uint8_t *codes, uint8_t *rows);
int oracle_encode_bits(const uint16_t *x, int64_t n, const float *thr, int bits, int use_hadamard,
                       uint8_t *codes, uint8_t *rows);

int oracle_encode(const uint16_t *x, int64_t n, const float thr[3],
                  uint8_t *codes, uint8_t *rows) {
  return oracle_encode_variant(x, n, thr, 1, codes, rows);
}

/*
 * use_hadamard != 0: the method (Eq. 4 then Eq. 5).  use_hadamard == 0: the
 * ablation "without the Hadamard transform" (Section 4.4): Eq. 5 is applied
 * to the raw vector, code_j = #{ i : x_j > thr[i] }, thresholds as given.
 */
int oracle_encode_variant(const uint16_t *x, int64_t n, const float thr[3], int use_hadamard,
                          uint8_t *codes, uint8_t *rows) {
  return oracle_encode_bits(x, n, thr, 2, use_hadamard, codes, rows);
}

/*
 * bits = 1, 2, 3: the bucketization granularities of Section 4.4, with
 * 2^bits - 1 thresholds and rows of 16 * bits bytes (oracle_pack_row_bits).
 */
int oracle_encode_bits(const uint16_t *x, int64_t n, const float *thr, int bits, int use_hadamard,
                       uint8_t *codes, uint8_t *rows) {
  if (!x || n < 0 || !thr || bits < 1 || bits > 3) return ORACLE_BAD_ARG;
  const int nthr = (1 << bits) - 1;
  if (!increasing(thr, nthr)) return ORACLE_BAD_ARG;
  int8_t *H = (int8_t *)malloc((size_t)ORACLE_D * ORACLE_D);
  if (!H) return ORACLE_NOMEM;
  oracle_hadamard_matrix(ORACLE_D, H);
  double tau[ORACLE_MAX_THR];
  if (use_hadamard) {
    scaled_thresholds(ORACLE_D, thr, nthr, tau);
  } else {
    for (int i = 0; i < nthr; ++i) tau[i] = (double)thr[i];
  }
  int status = ORACLE_OK;
#pragma omp parallel for schedule(static)
  for (int64_t v = 0; v < n; ++v) {
    double xv[ORACLE_MAX_D], y[ORACLE_MAX_D];
    uint8_t code[ORACLE_MAX_D];
    int emax = -100000, emin = 100000, bad = 0;
    for (int i = 0; i < ORACLE_D; ++i) {
      xv[i] = bf16_to_double(x[v * ORACLE_D + i]);
      if (!isfinite(xv[i])) bad = 1;
      if (xv[i] != 0.0 && isfinite(xv[i])) {
        int e;
        frexp(xv[i], &e);
        if (e > emax) emax = e;
        if (e < emin) emin = e;
      }
    }
    if (bad || (emax > -100000 && emax - emin > 38)) {
#pragma omp atomic write
      status = ORACLE_PRECONDITION;
      continue;
    }
    for (int j = 0; j < ORACLE_D; ++j) {
      if (use_hadamard) {
        double s = 0.0;
        for (int i = 0; i < ORACLE_D; ++i) s += xv[i] * (double)H[i * ORACLE_D + j];
        y[j] = s;
      } else {
        y[j] = xv[j];
      }
    }
    for (int j = 0; j < ORACLE_D; ++j) {
      int c = 0;
      for (int i = 0; i < nthr; ++i)
        if (y[j] > tau[i]) ++c;
      code[j] = (uint8_t)c;
    }
    if (codes) memcpy(codes + v * ORACLE_D, code, ORACLE_D);
    if (rows) oracle_pack_row_bits(code, bits, rows + v * (int64_t)(ORACLE_D / 8) * bits);
  }
  free(H);
  return status;
}

/* ------------------------------------------------- Manhattan distance, Eq. 6 */

/* D[t] = sum_j |qcode_j - kcodes[t][j]| over unpacked codes, t < L. */
int oracle_manhattan(const uint8_t *qcode, const uint8_t *kcodes, int64_t L,
                     int32_t *D) {
  if (!qcode || (!kcodes && L > 0) || L < 0 || (!D && L > 0)) return ORACLE_BAD_ARG;
  for (int64_t t = 0; t < L; ++t) {
    int32_t s = 0;
    for (int j = 0; j < ORACLE_D; ++j) {
      int diff = (int)qcode[j] - (int)kcodes[t * ORACLE_D + j];
      s += diff < 0 ? -diff : diff;
    }
    D[t] = s;
  }
  return ORACLE_OK;
}

/*
 * Ablation "with L2 distance" (Section 4.4): the estimator of Eq. 6 with the
 * absolute difference replaced by its square, D[t] = sum_j (qcode_j - kcodes[t][j])^2.
 * (The square root is monotone and would not change any ranking; it is left out,
 * which keeps the distances integers.)
 */
int oracle_squared_distance(const uint8_t *qcode, const uint8_t *kcodes, int64_t L,
                            int32_t *D) {
  if (!qcode || (!kcodes && L > 0) || L < 0 || (!D && L > 0)) return ORACLE_BAD_ARG;
  for (int64_t t = 0; t < L; ++t) {
    int32_t s = 0;
    for (int j = 0; j < ORACLE_D; ++j) {
      int diff = (int)qcode[j] - (int)kcodes[t * ORACLE_D + j];
      s += diff * diff;
    }
    D[t] = s;
  }
  return ORACLE_OK;
}

/* --------------------------------------------------- top-k (Algorithm 1, selection step) */

typedef struct {
  int32_t dist;
  int32_t tok;
} dist_tok;

static int cmp_dist_then_tok(const void *a, const void *b) {
  const dist_tok *x = (const dist_tok *)a, *y = (const dist_tok *)b;
  if (x->dist != y->dist) return x->dist < y->dist ? -1 : 1;
  if (x->tok != y->tok) return x->tok < y->tok ? -1 : 1;
  return 0;
}

static int cmp_int32(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

/*
 * The min(k, L) tokens of smallest distance; equal distances are ranked by
 * token index, lower first.  Output: those token indices in ascending order,
 * then -1 up to k entries.
 */
int oracle_topk(const int32_t *D, int64_t L, int32_t k, int32_t *idx) {
  if (L < 0 || k < 1 || !idx || (!D && L > 0)) return ORACLE_BAD_ARG;
  for (int32_t i = 0; i < k; ++i) idx[i] = -1;
  if (L == 0) return ORACLE_OK;
  dist_tok *all = (dist_tok *)malloc((size_t)L * sizeof *all);
  if (!all) return ORACLE_NOMEM;
  for (int64_t t = 0; t < L; ++t) {
    all[t].dist = D[t];
    all[t].tok = (int32_t)t;
  }
  qsort(all, (size_t)L, sizeof *all, cmp_dist_then_tok);
  int32_t n = (int64_t)k < L ? k : (int32_t)L;
  for (int32_t i = 0; i < n; ++i) idx[i] = all[i].tok;
  qsort(idx, (size_t)n, sizeof *idx, cmp_int32);
  free(all);
  return ORACLE_OK;
}

/* ------------------------------------------------------- attention, Eq. 1 */

/*
 * o = softmax(q K_s^T * scale) V_s over the rows listed in idx (entries < 0
 * are skipped), in the order listed.  q: 128 bf16; K, V: rows of 128 bf16,
 * row r at K + r*128.  All arithmetic in double; result rounded to float.
 * No valid row -> zeros.
 */
int oracle_sparse_attention(const uint16_t *q, const uint16_t *K,
                            const uint16_t *V, const int32_t *idx, int32_t k,
                            double scale, float *out) {
  if (!q || !K || !V || !idx || k < 0 || !out) return ORACLE_BAD_ARG;
  double *s = (double *)malloc((size_t)(k > 0 ? k : 1) * sizeof *s);
  if (!s) return ORACLE_NOMEM;
  double m = -INFINITY;
  int any = 0;
  for (int32_t i = 0; i < k; ++i) {
    if (idx[i] < 0) continue;
    const uint16_t *row = K + (int64_t)idx[i] * ORACLE_D;
    double dot = 0.0;
    for (int j = 0; j < ORACLE_D; ++j)
      dot += bf16_to_double(q[j]) * bf16_to_double(row[j]);
    s[i] = dot * scale;
    if (s[i] > m) m = s[i];
    any = 1;
  }
  double acc[ORACLE_MAX_D];
  for (int j = 0; j < ORACLE_D; ++j) acc[j] = 0.0;
  double denom = 0.0;
  for (int32_t i = 0; i < k && any; ++i) {
    if (idx[i] < 0) continue;
    double p = exp(s[i] - m);
    denom += p;
    const uint16_t *row = V + (int64_t)idx[i] * ORACLE_D;
    for (int j = 0; j < ORACLE_D; ++j) acc[j] += p * bf16_to_double(row[j]);
  }
  for (int j = 0; j < ORACLE_D; ++j) out[j] = any ? (float)(acc[j] / denom) : 0.0f;
  free(s);
  return ORACLE_OK;
}

/* Eq. 1 over every cached row 0..L-1: written out separately on purpose. */
int oracle_full_attention(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                          int64_t L, double scale, float *out) {
  if (!q || L < 0 || (L > 0 && (!K || !V)) || !out) return ORACLE_BAD_ARG;
  if (L == 0) {
    for (int j = 0; j < ORACLE_D; ++j) out[j] = 0.0f;
    return ORACLE_OK;
  }
  double *p = (double *)malloc((size_t)L * sizeof *p);
  if (!p) return ORACLE_NOMEM;
  double m = -INFINITY;
  for (int64_t t = 0; t < L; ++t) {
    double dot = 0.0;
    for (int j = 0; j < ORACLE_D; ++j)
      dot += bf16_to_double(q[j]) * bf16_to_double(K[t * ORACLE_D + j]);
    p[t] = dot * scale;
    if (p[t] > m) m = p[t];
  }
  double denom = 0.0;
  for (int64_t t = 0; t < L; ++t) {
    p[t] = exp(p[t] - m);
    denom += p[t];
  }
  for (int j = 0; j < ORACLE_D; ++j) {
    double a = 0.0;
    for (int64_t t = 0; t < L; ++t) a += p[t] * bf16_to_double(V[t * ORACLE_D + j]);
    out[j] = (float)(a / denom);
  }
  free(p);
  return ORACLE_OK;
}

/* ------------------------------------------- whole decode step, Algorithm 1 */

/*
 * One decode step of one attention layer over a ragged batch.
 *
 * Pools (host memory, caller-owned): K, V bf16 [Hkv][pool_tokens][128];
 * code_rows uint8 [Hkv][pool_tokens][32].  Sequence b owns pool rows
 * seq_start[b] .. seq_start[b]+seq_len[b]-1 of every KV head; seq_len counts
 * the appended token when k_new/v_new are given.  q: bf16 [B][Hq][128];
 * k_new, v_new: bf16 [B][Hkv][128] or both NULL.  Query head h reads KV head
 * h / (Hq/Hkv).
 *
 * Steps, in the order of Algorithm 1: (1-3) encode q and, when appending,
 * k_new; (4) write k_new, v_new and the new code row at the sequence's last
 * row; (5) distances to every cached row; (6) top-k; (7-8) attention over
 * the selected rows of the original K, V.
 *
 * Outputs: out fp32 [B][Hq][128]; idx int32 [B][Hq][k] (ascending, -1
 * padded); dist (nullable) int32 [B][Hq][max_seq_len], entries past
 * seq_len[b] untouched.  Parallel over (b, query head) when built with
 * OpenMP.
 */
int oracle_decode_step_variant(int32_t Hq, int32_t Hkv, int64_t pool_tokens,
                               const float thr_q[3], const float thr_k[3], double scale,
                               const uint16_t *q, const uint16_t *k_new,
                               const uint16_t *v_new, uint16_t *K, uint16_t *V,
                               uint8_t *code_rows, const int64_t *seq_start,
                               const int32_t *seq_len, int32_t B, int32_t k, float *out,
                               int32_t *idx, int32_t *dist, int64_t max_seq_len,
                               int use_hadamard, int squared_distance);
int oracle_decode_step_bits(int32_t Hq, int32_t Hkv, int64_t pool_tokens,
                            const float *thr_q, const float *thr_k, int bits, double scale,
                            const uint16_t *q, const uint16_t *k_new,
                            const uint16_t *v_new, uint16_t *K, uint16_t *V,
                            uint8_t *code_rows, const int64_t *seq_start,
                            const int32_t *seq_len, int32_t B, int32_t k, float *out,
                            int32_t *idx, int32_t *dist, int64_t max_seq_len,
                            int use_hadamard, int squared_distance);

int oracle_decode_step(int32_t Hq, int32_t Hkv, int64_t pool_tokens,
                       const float thr_q[3], const float thr_k[3], double scale,
                       const uint16_t *q, const uint16_t *k_new,
                       const uint16_t *v_new, uint16_t *K, uint16_t *V,
                       uint8_t *code_rows, const int64_t *seq_start,
                       const int32_t *seq_len, int32_t B, int32_t k, float *out,
                       int32_t *idx, int32_t *dist, int64_t max_seq_len) {
  return oracle_decode_step_variant(Hq, Hkv, pool_tokens, thr_q, thr_k, scale, q, k_new, v_new, K,
                                    V, code_rows, seq_start, seq_len, B, k, out, idx, dist,
                                    max_seq_len, 1, 0);
}

/*
 * The same step for the ablation variants of Section 4.4: use_hadamard == 0
 * encodes query and appended key without the transform; squared_distance != 0
 * ranks by the squared-difference estimator instead of Eq. 6.  (1, 0) is the
 * method itself.  code_rows must have been encoded with the same use_hadamard.
 */
int oracle_decode_step_variant(int32_t Hq, int32_t Hkv, int64_t pool_tokens,
                               const float thr_q[3], const float thr_k[3], double scale,
                               const uint16_t *q, const uint16_t *k_new,
                               const uint16_t *v_new, uint16_t *K, uint16_t *V,
                               uint8_t *code_rows, const int64_t *seq_start,
                               const int32_t *seq_len, int32_t B, int32_t k, float *out,
                               int32_t *idx, int32_t *dist, int64_t max_seq_len,
                               int use_hadamard, int squared_distance) {
  return oracle_decode_step_bits(Hq, Hkv, pool_tokens, thr_q, thr_k, 2, scale, q, k_new, v_new, K,
                                 V, code_rows, seq_start, seq_len, B, k, out, idx, dist,
                                 max_seq_len, use_hadamard, squared_distance);
}

/*
 * The step with `bits`-bit codes (Section 4.4, bucketization ablation):
 * thr_q, thr_k hold 2^bits - 1 thresholds, code_rows has 16 * bits bytes per
 * row.  bits = 2 is the method.
 */
int oracle_decode_step_bits(int32_t Hq, int32_t Hkv, int64_t pool_tokens,
                            const float *thr_q, const float *thr_k, int bits, double scale,
                            const uint16_t *q, const uint16_t *k_new,
                            const uint16_t *v_new, uint16_t *K, uint16_t *V,
                            uint8_t *code_rows, const int64_t *seq_start,
                            const int32_t *seq_len, int32_t B, int32_t k, float *out,
                            int32_t *idx, int32_t *dist, int64_t max_seq_len,
                            int use_hadamard, int squared_distance) {
  if (bits < 1 || bits > 3) return ORACLE_BAD_ARG;
  const int64_t row_bytes = (int64_t)(ORACLE_D / 8) * bits;
  if (Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || B < 1 || k < 1) return ORACLE_BAD_ARG;
  if (!q || !K || !V || !code_rows || !seq_start || !seq_len || !out || !idx)
    return ORACLE_BAD_ARG;
  if ((k_new == NULL) != (v_new == NULL)) return ORACLE_BAD_ARG;
  const int group = Hq / Hkv;
  int status = ORACLE_OK;

  /* Algorithm 1, encode and cache-update steps for the appended key */
  if (k_new) {
    for (int32_t b = 0; b < B; ++b) {
      if (seq_len[b] < 1) continue;
      int64_t row = seq_start[b] + seq_len[b] - 1;
      if (row < 0 || row >= pool_tokens) return ORACLE_BAD_ARG;
      for (int32_t h = 0; h < Hkv; ++h) {
        const uint16_t *kn = k_new + ((int64_t)b * Hkv + h) * ORACLE_D;
        const uint16_t *vn = v_new + ((int64_t)b * Hkv + h) * ORACLE_D;
        int64_t off = (int64_t)h * pool_tokens + row;
        memcpy(K + off * ORACLE_D, kn, ORACLE_D * sizeof(uint16_t));
        memcpy(V + off * ORACLE_D, vn, ORACLE_D * sizeof(uint16_t));
        int rc = oracle_encode_bits(kn, 1, thr_k, bits, use_hadamard, NULL,
                                    code_rows + off * row_bytes);
        if (rc != ORACLE_OK) return rc;
      }
    }
  }

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int32_t b = 0; b < B; ++b) {
    for (int32_t h = 0; h < Hq; ++h) {
      const int32_t kvh = h / group;
      const int64_t L = seq_len[b];
      const int64_t base = (int64_t)kvh * pool_tokens + seq_start[b];
      const uint16_t *qv = q + ((int64_t)b * Hq + h) * ORACLE_D;
      float *o = out + ((int64_t)b * Hq + h) * ORACLE_D;
      int32_t *sel = idx + ((int64_t)b * Hq + h) * k;
      uint8_t qcode[ORACLE_MAX_D];
      int rc = oracle_encode_bits(qv, 1, thr_q, bits, use_hadamard, qcode, NULL);
      uint8_t *kc = (uint8_t *)malloc((size_t)(L > 0 ? L : 1) * ORACLE_D);
      int32_t *D = (int32_t *)malloc((size_t)(L > 0 ? L : 1) * sizeof(int32_t));
      if (!kc || !D) rc = ORACLE_NOMEM;
      if (rc == ORACLE_OK) {
        for (int64_t t = 0; t < L; ++t)
          oracle_unpack_row_bits(code_rows + (base + t) * row_bytes, bits, kc + t * ORACLE_D);
        if (squared_distance) oracle_squared_distance(qcode, kc, L, D);
        else oracle_manhattan(qcode, kc, L, D);
        if (dist)
          memcpy(dist + ((int64_t)b * Hq + h) * max_seq_len, D, (size_t)L * sizeof(int32_t));
        rc = oracle_topk(D, L, k, sel);
      }
      if (rc == ORACLE_OK)
        rc = oracle_sparse_attention(qv, K + base * ORACLE_D, V + base * ORACLE_D, sel, k,
                                     scale, o);
      free(kc);
      free(D);
      if (rc != ORACLE_OK) {
#pragma omp atomic write
        status = rc;
      }
    }
  }
  return status;
}

/* ------------------------------------------------------- paged cache layout */

/*
 * The same step on a paged cache, the layout of the serving engines the paper
 * compares with (Section 4.1).  The pools are cut into pages of page_tokens
 * rows; token t of sequence b lives in pool row
 *   page_table[b * max_pages + t / page_tokens] * page_tokens + t % page_tokens
 * of every KV head.  Nothing new is computed: every sequence's rows are copied
 * into a contiguous scratch cache through the page table, the contiguous step
 * above runs on that copy, and the appended row (K, V, code row) is copied back
 * to its page.  idx holds token positions, as in the contiguous step.
 */
int oracle_decode_step_paged(int32_t Hq, int32_t Hkv, int64_t pool_tokens,
                             const float thr_q[3], const float thr_k[3], double scale,
                             const uint16_t *q, const uint16_t *k_new,
                             const uint16_t *v_new, uint16_t *K, uint16_t *V,
                             uint8_t *code_rows, const int32_t *page_table,
                             int32_t max_pages, int32_t page_tokens,
                             const int32_t *seq_len, int32_t B, int32_t k, float *out,
                             int32_t *idx, int use_hadamard, int squared_distance) {
  if (Hq < 1 || Hkv < 1 || B < 1 || k < 1 || !page_table || max_pages < 1 || page_tokens < 1)
    return ORACLE_BAD_ARG;
  if (!q || !K || !V || !code_rows || !seq_len || !out || !idx) return ORACLE_BAD_ARG;
  int64_t total = 0, max_len = 1;
  for (int32_t b = 0; b < B; ++b) {
    if (seq_len[b] < 0 || (int64_t)seq_len[b] > (int64_t)max_pages * page_tokens)
      return ORACLE_BAD_ARG;
    total += seq_len[b];
    if (seq_len[b] > max_len) max_len = seq_len[b];
  }
  int64_t pool2 = total > 0 ? total : 1;
  uint16_t *K2 = (uint16_t *)malloc((size_t)Hkv * pool2 * ORACLE_D * sizeof(uint16_t));
  uint16_t *V2 = (uint16_t *)malloc((size_t)Hkv * pool2 * ORACLE_D * sizeof(uint16_t));
  uint8_t *R2 = (uint8_t *)malloc((size_t)Hkv * pool2 * ORACLE_ROW_BYTES);
  int64_t *start2 = (int64_t *)malloc((size_t)B * sizeof(int64_t));
  if (!K2 || !V2 || !R2 || !start2) {
    free(K2); free(V2); free(R2); free(start2);
    return ORACLE_NOMEM;
  }
  int rc = ORACLE_OK;
  int64_t at = 0;
  for (int32_t b = 0; b < B && rc == ORACLE_OK; ++b) {
    start2[b] = at;
    for (int64_t t = 0; t < seq_len[b]; ++t) {
      int64_t page = page_table[(int64_t)b * max_pages + t / page_tokens];
      int64_t row = page * page_tokens + t % page_tokens;
      if (page < 0 || row >= pool_tokens) { rc = ORACLE_BAD_ARG; break; }
      for (int32_t h = 0; h < Hkv; ++h) {
        int64_t src = (int64_t)h * pool_tokens + row, dst = (int64_t)h * pool2 + at + t;
        memcpy(K2 + dst * ORACLE_D, K + src * ORACLE_D, ORACLE_D * sizeof(uint16_t));
        memcpy(V2 + dst * ORACLE_D, V + src * ORACLE_D, ORACLE_D * sizeof(uint16_t));
        memcpy(R2 + dst * ORACLE_ROW_BYTES, code_rows + src * ORACLE_ROW_BYTES, ORACLE_ROW_BYTES);
      }
    }
    at += seq_len[b];
  }
  if (rc == ORACLE_OK)
    rc = oracle_decode_step_variant(Hq, Hkv, pool2, thr_q, thr_k, scale, q, k_new, v_new, K2, V2,
                                    R2, start2, seq_len, B, k, out, idx, NULL, max_len,
                                    use_hadamard, squared_distance);
  if (rc == ORACLE_OK && k_new) {
    for (int32_t b = 0; b < B; ++b) {
      if (seq_len[b] < 1) continue;
      int64_t t = seq_len[b] - 1;
      int64_t row = (int64_t)page_table[(int64_t)b * max_pages + t / page_tokens] * page_tokens +
                    t % page_tokens;
      for (int32_t h = 0; h < Hkv; ++h) {
        int64_t dst = (int64_t)h * pool_tokens + row, src = (int64_t)h * pool2 + start2[b] + t;
        memcpy(K + dst * ORACLE_D, K2 + src * ORACLE_D, ORACLE_D * sizeof(uint16_t));
        memcpy(V + dst * ORACLE_D, V2 + src * ORACLE_D, ORACLE_D * sizeof(uint16_t));
        memcpy(code_rows + dst * ORACLE_ROW_BYTES, R2 + src * ORACLE_ROW_BYTES, ORACLE_ROW_BYTES);
      }
    }
  }
  free(K2); free(V2); free(R2); free(start2);
  return rc;
}

/* ---------------------------------------------------------- thread control */

#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of host threads the parallel loops above may use (1 without OpenMP). */
int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}
