/*
 * Sanitizer run of the CPU oracle (test infrastructure): compiled together with
 * oracle/adamas_oracle.c under -fsanitize=address,undefined by
 * tests/test_oracle_sanitizers.py and run as a plain program.  It drives every
 * oracle function at every head dimension on small seeded inputs -- ragged
 * batches with an empty sequence, appends, paged caches, all code widths and
 * both estimators -- so that an out-of-bounds access, a leak, a signed overflow
 * or a misaligned access anywhere in the oracle aborts the program.  A few
 * invariants are checked on the way (H H^T = d I, pack/unpack round trip,
 * top-k order); the numerical pins live in tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_set_head_dim(int d);
int oracle_hadamard_matrix(int d, int8_t *H);
int oracle_hadamard_transform(int d, const double *x, double *y);
int oracle_bucketize_n(int64_t n, const double *y, int d, const float *thr, int nthr, uint8_t *code);
int oracle_pack_row_bits(const uint8_t *code, int bits, uint8_t *row);
int oracle_unpack_row_bits(const uint8_t *row, int bits, uint8_t *code);
int oracle_pack_row(const uint8_t *code, uint8_t *row);
int oracle_unpack_row(const uint8_t *row, uint8_t *code);
int oracle_encode_bits(const uint16_t *x, int64_t n, const float *thr, int bits, int use_hadamard,
                       uint8_t *codes, uint8_t *rows);
int oracle_manhattan(const uint8_t *qcode, const uint8_t *kcodes, int64_t L, int32_t *D);
int oracle_squared_distance(const uint8_t *qcode, const uint8_t *kcodes, int64_t L, int32_t *D);
int oracle_topk(const int32_t *D, int64_t L, int32_t k, int32_t *idx);
int oracle_sparse_attention(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                            const int32_t *idx, int32_t k, double scale, float *out);
int oracle_full_attention(const uint16_t *q, const uint16_t *K, const uint16_t *V, int64_t L,
                          double scale, float *out);
int oracle_decode_step_variant(int32_t Hq, int32_t Hkv, int64_t pool_tokens, const float thr_q[3],
                               const float thr_k[3], double scale, const uint16_t *q,
                               const uint16_t *k_new, const uint16_t *v_new, uint16_t *K,
                               uint16_t *V, uint8_t *code_rows, const int64_t *seq_start,
                               const int32_t *seq_len, int32_t B, int32_t k, float *out,
                               int32_t *idx, int32_t *dist, int64_t max_seq_len, int use_hadamard,
                               int squared_distance);
int oracle_decode_step_bits(int32_t Hq, int32_t Hkv, int64_t pool_tokens, const float *thr_q,
                            const float *thr_k, int bits, double scale, const uint16_t *q,
                            const uint16_t *k_new, const uint16_t *v_new, uint16_t *K, uint16_t *V,
                            uint8_t *code_rows, const int64_t *seq_start, const int32_t *seq_len,
                            int32_t B, int32_t k, float *out, int32_t *idx, int32_t *dist,
                            int64_t max_seq_len, int use_hadamard, int squared_distance);
int oracle_decode_step_paged(int32_t Hq, int32_t Hkv, int64_t pool_tokens, const float thr_q[3],
                             const float thr_k[3], double scale, const uint16_t *q,
                             const uint16_t *k_new, const uint16_t *v_new, uint16_t *K, uint16_t *V,
                             uint8_t *code_rows, const int32_t *page_table, int32_t max_pages,
                             int32_t page_tokens, const int32_t *seq_len, int32_t B, int32_t k,
                             float *out, int32_t *idx, int use_hadamard, int squared_distance);

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      fprintf(stderr, "oracle_sanitize: %s failed (line %d)\n", #cond, __LINE__); \
      exit(1);                                                               \
    }                                                                        \
  } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return rng_state >> 8;
}
/* a bf16 bit pattern of modest magnitude: sign, exponent 120..129, 7 mantissa bits */
static uint16_t rnd_bf16(void) {
  uint32_t r = rnd();
  return (uint16_t)(((r & 1u) << 15) | ((120u + (r >> 1) % 10u) << 7) | ((r >> 8) & 0x7fu));
}
static void fill_bf16(uint16_t *p, size_t n) {
  for (size_t i = 0; i < n; ++i) p[i] = rnd_bf16();
}

static void run_head_dim(int d) {
  CHECK(oracle_set_head_dim(d) == 0);
  const float thr1[1] = {0.f}, thr3[3] = {-1.f, 0.f, 1.f};
  const float thr7[7] = {-1.5f, -1.f, -0.5f, 0.f, 0.5f, 1.f, 1.5f};
  /* matrix and transform */
  int8_t *H = malloc((size_t)d * d);
  CHECK(H && oracle_hadamard_matrix(d, H) == 0);
  for (int i = 0; i < d; i += 7)
    for (int j = 0; j < d; j += 5) {
      int s = 0;
      for (int c = 0; c < d; ++c) s += H[i * d + c] * H[j * d + c];
      CHECK(s == (i == j ? d : 0));
    }
  double *x = malloc(sizeof(double) * d), *y = malloc(sizeof(double) * d);
  for (int i = 0; i < d; ++i) x[i] = (double)((int)(rnd() % 21) - 10);
  CHECK(oracle_hadamard_transform(d, x, y) == 0);
  uint8_t *code = malloc(d), *code2 = malloc(d), *row = malloc((size_t)d / 8 * 3);
  CHECK(oracle_bucketize_n(d, y, d, thr7, 7, code) == 0);
  for (int bits = 1; bits <= 3; ++bits) {
    for (int i = 0; i < d; ++i) code2[i] = (uint8_t)(code[i] & ((1 << bits) - 1));
    CHECK(oracle_pack_row_bits(code2, bits, row) == 0);
    memset(code, 0xff, d);
    CHECK(oracle_unpack_row_bits(row, bits, code) == 0);
    CHECK(memcmp(code, code2, d) == 0);
  }
  (void)oracle_pack_row(code2, row); /* the 3-bit values are refused (BAD_ARG): no fault either way */
  free(H); free(x); free(y); free(code); free(code2); free(row);

  /* a ragged cache: three sequences (one empty), gaps, append */
  enum { B = 3, Hq = 4, Hkv = 2, K_ = 9 };
  const int32_t len[B] = {37, 0, 130};
  const int64_t start[B] = {0, 40, 45};
  const int64_t pool = 45 + 130;
  size_t kv = (size_t)Hkv * pool * d;
  uint16_t *K = malloc(kv * 2), *V = malloc(kv * 2), *q = malloc((size_t)B * Hq * d * 2);
  uint16_t *kn = malloc((size_t)B * Hkv * d * 2), *vn = malloc((size_t)B * Hkv * d * 2);
  fill_bf16(K, kv); fill_bf16(V, kv); fill_bf16(q, (size_t)B * Hq * d);
  fill_bf16(kn, (size_t)B * Hkv * d); fill_bf16(vn, (size_t)B * Hkv * d);
  float *out = malloc(sizeof(float) * B * Hq * d);
  int32_t *idx = malloc(sizeof(int32_t) * B * Hq * K_), *dist = malloc(sizeof(int32_t) * B * Hq * 130);
  for (int bits = 1; bits <= 3; ++bits) {
    const float *thr = bits == 1 ? thr1 : bits == 2 ? thr3 : thr7;
    size_t rb = (size_t)d / 8 * bits;
    uint8_t *rows = malloc((size_t)Hkv * pool * rb), *codes = malloc((size_t)Hkv * pool * d);
    for (int had = 0; had <= 1; ++had) {
      CHECK(oracle_encode_bits(K, Hkv * pool, thr, bits, had, codes, rows) == 0);
      CHECK(oracle_decode_step_bits(Hq, Hkv, pool, thr, thr, bits, 1.0 / sqrt((double)d), q, kn, vn,
                                    K, V, rows, start, len, B, K_, out, idx, dist, 130, had, 0) == 0);
      for (int h = 0; h < Hq; ++h) { /* empty sequence: no index, zero output */
        for (int i = 0; i < K_; ++i) CHECK(idx[(1 * Hq + h) * K_ + i] == -1);
        for (int i = 1; i < K_; ++i) {
          int a = idx[(2 * Hq + h) * K_ + i - 1], b = idx[(2 * Hq + h) * K_ + i];
          CHECK(a >= 0 && a < b && b < 130);
        }
      }
    }
    if (bits == 2) {
      CHECK(oracle_decode_step_variant(Hq, Hkv, pool, thr3, thr3, 0.1, q, NULL, NULL, K, V, rows,
                                       start, len, B, K_, out, idx, NULL, 130, 1, 1) == 0);
      int32_t D1[130], D2[130];
      CHECK(oracle_manhattan(codes, codes + (size_t)45 * d, 130, D1) == 0);
      CHECK(oracle_squared_distance(codes, codes + (size_t)45 * d, 130, D2) == 0);
      for (int t = 0; t < 130; ++t) CHECK(D1[t] <= D2[t] && D2[t] <= 3 * D1[t]);
      int32_t top[200];
      CHECK(oracle_topk(D1, 130, 200, top) == 0);
      CHECK(top[129] == 129 && top[130] == -1);
      CHECK(oracle_sparse_attention(q, K, V, top, 130, 0.1, out) == 0);
      CHECK(oracle_full_attention(q, K, V, 45, 0.1, out) == 0);
      /* paged: pages of 64 tokens, sequence 2 on pages {2, 0, 1} */
      const int32_t table[B * 3] = {1, -1, -1, -1, -1, -1, 2, 0, 1};
      const int64_t ppool = 3 * 64;
      uint16_t *Kp = malloc((size_t)Hkv * ppool * d * 2), *Vp = malloc((size_t)Hkv * ppool * d * 2);
      uint8_t *rp = malloc((size_t)Hkv * ppool * rb);
      fill_bf16(Kp, (size_t)Hkv * ppool * d); fill_bf16(Vp, (size_t)Hkv * ppool * d);
      CHECK(oracle_encode_bits(Kp, Hkv * ppool, thr3, 2, 1, NULL, rp) == 0);
      const int32_t plen[B] = {37, 0, 130};
      CHECK(oracle_decode_step_paged(Hq, Hkv, ppool, thr3, thr3, 0.1, q, kn, vn, Kp, Vp, rp, table, 3,
                                     64, plen, B, K_, out, idx, 1, 0) == 0);
      free(Kp); free(Vp); free(rp);
    }
    free(rows); free(codes);
  }
  free(K); free(V); free(q); free(kn); free(vn); free(out); free(idx); free(dist);
}

int main(void) {
  const int dims[] = {64, 96, 128, 160, 192, 256};
  for (size_t i = 0; i < sizeof dims / sizeof dims[0]; ++i) run_head_dim(dims[i]);
  int8_t P[20 * 20];
  CHECK(oracle_hadamard_matrix(12, P) == 0 && oracle_hadamard_matrix(20, P) == 0);
  CHECK(oracle_hadamard_matrix(36, P) != 0 && oracle_set_head_dim(80) != 0);
  CHECK(oracle_set_head_dim(128) == 0);
  printf("oracle_sanitize: ok\n");
  return 0;
}
