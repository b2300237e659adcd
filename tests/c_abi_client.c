/*
 * A plain C program that uses the library the way a serving engine without
 * Python would: hipMalloc'ed buffers, adamas.h, nothing else.  TEST CODE: it
 * checks the fused decode step (with append, ragged batch, GQA) against the CPU
 * oracle, which it links as well, then the staged entry points (query codes,
 * distances, top-k, attention) and the step that allocates nothing against the
 * same results.  Exit code 0 = all checks passed.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adamas.h"

/* the oracle's C entry points used here (oracle/adamas_oracle.c) */
int oracle_encode(const uint16_t *x, int64_t n, const float thr[3], uint8_t *codes, uint8_t *rows);
int oracle_decode_step(int32_t Hq, int32_t Hkv, int64_t pool_tokens, const float thr_q[3],
                       const float thr_k[3], double scale, const uint16_t *q,
                       const uint16_t *k_new, const uint16_t *v_new, uint16_t *K, uint16_t *V,
                       uint8_t *code_rows, const int64_t *seq_start, const int32_t *seq_len,
                       int32_t B, int32_t k, float *out, int32_t *idx, int32_t *dist,
                       int64_t max_seq_len);

#define HIP_OK(x)                                                                  \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));               \
      return 2;                                                                    \
    }                                                                              \
  } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static float uniform_pm2(void) { /* 24-bit uniform in [-2, 2) */
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return ((float)(rng_state >> 40) / 16777216.0f) * 4.0f - 2.0f;
}
static uint16_t to_bf16(float f) { /* round to nearest even */
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
static void fill(uint16_t *p, size_t n) {
  for (size_t i = 0; i < n; ++i) p[i] = to_bf16(uniform_pm2());
}

int main(void) {
  enum { B = 2, Hq = 4, Hkv = 2, D = 128, K_BUDGET = 64 };
  const int32_t lens[B] = {3000, 777};          /* after the append */
  const int64_t starts[B] = {0, 3000 + 64};
  const int64_t pool = 3000 + 64 + 777, max_len = 3000;
  const float thr[3] = {-1.0f, 0.0f, 1.0f};
  const size_t n_kv = (size_t)Hkv * pool * D;

  uint16_t *K = malloc(n_kv * 2), *V = malloc(n_kv * 2), *Kref = malloc(n_kv * 2), *Vref = malloc(n_kv * 2);
  uint16_t q[B * Hq * D], kn[B * Hkv * D], vn[B * Hkv * D];
  uint8_t *rows = malloc((size_t)Hkv * pool * 32), *rows_gpu = malloc((size_t)Hkv * pool * 32);
  if (!K || !V || !Kref || !Vref || !rows || !rows_gpu) return 2;
  fill(K, n_kv); fill(V, n_kv); fill(q, B * Hq * D); fill(kn, B * Hkv * D); fill(vn, B * Hkv * D);
  /* make the first query of each sequence a near copy of a cached key: it must be selected */
  for (int b = 0; b < B; ++b)
    memcpy(q + (size_t)b * Hq * D, K + (size_t)(starts[b] + 123) * D, D * 2);
  memcpy(Kref, K, n_kv * 2); memcpy(Vref, V, n_kv * 2);

  adamas_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.head_dim = D; cfg.num_q_heads = Hq; cfg.num_kv_heads = Hkv; cfg.pool_tokens = pool;
  memcpy(cfg.thr_k, thr, sizeof thr); memcpy(cfg.thr_q, thr, sizeof thr);

  void *dK, *dV, *dq, *dkn, *dvn, *dcodes, *dws, *dout, *didx, *dstart, *dlen;
  const size_t ws_bytes = adamas_workspace_bytes(&cfg, B, max_len, K_BUDGET);
  if (ws_bytes == 0) { fprintf(stderr, "workspace size 0\n"); return 1; }
  HIP_OK(hipMalloc(&dK, n_kv * 2)); HIP_OK(hipMalloc(&dV, n_kv * 2));
  HIP_OK(hipMalloc(&dq, sizeof q)); HIP_OK(hipMalloc(&dkn, sizeof kn)); HIP_OK(hipMalloc(&dvn, sizeof vn));
  HIP_OK(hipMalloc(&dcodes, (size_t)Hkv * pool * 32)); HIP_OK(hipMalloc(&dws, ws_bytes));
  HIP_OK(hipMalloc(&dout, B * Hq * D * 4)); HIP_OK(hipMalloc(&didx, B * Hq * K_BUDGET * 4));
  HIP_OK(hipMalloc(&dstart, sizeof starts)); HIP_OK(hipMalloc(&dlen, sizeof lens));
  HIP_OK(hipMemcpy(dK, K, n_kv * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dV, V, n_kv * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dq, q, sizeof q, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dkn, kn, sizeof kn, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dvn, vn, sizeof vn, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dstart, starts, sizeof starts, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dlen, lens, sizeof lens, hipMemcpyHostToDevice));
  HIP_OK(hipMemset(dws, 0xA5, ws_bytes));

  int rc = adamas_encode_keys(&cfg, dK, dcodes, 0, pool, NULL);
  if (rc) { fprintf(stderr, "encode_keys: %s\n", adamas_status_string(rc)); return 1; }
  rc = adamas_decode_step(&cfg, dq, dkn, dvn, dK, dV, dcodes, dstart, dlen, B, K_BUDGET, dout, didx,
                          max_len, dws, ws_bytes, NULL);
  if (rc) { fprintf(stderr, "decode_step: %s\n", adamas_status_string(rc)); return 1; }
  HIP_OK(hipDeviceSynchronize());

  float out[B * Hq * D], ref_out[B * Hq * D];
  int32_t idx[B * Hq * K_BUDGET], ref_idx[B * Hq * K_BUDGET];
  HIP_OK(hipMemcpy(out, dout, sizeof out, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(idx, didx, sizeof idx, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(rows_gpu, dcodes, (size_t)Hkv * pool * 32, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(K, dK, n_kv * 2, hipMemcpyDeviceToHost));

  /* the oracle on the same inputs: encode the cache as it was, then the step (which appends) */
  if (oracle_encode(Kref, (int64_t)Hkv * pool, thr, NULL, rows)) { fprintf(stderr, "oracle encode\n"); return 1; }
  if (oracle_decode_step(Hq, Hkv, pool, thr, thr, 1.0 / sqrt(128.0), q, kn, vn, Kref, Vref, rows,
                         starts, lens, B, K_BUDGET, ref_out, ref_idx, NULL, max_len)) {
    fprintf(stderr, "oracle step\n");
    return 1;
  }
  int bad = 0;
  if (memcmp(idx, ref_idx, sizeof idx)) { fprintf(stderr, "indices differ\n"); bad = 1; }
  if (memcmp(rows_gpu, rows, (size_t)Hkv * pool * 32)) { fprintf(stderr, "code rows differ\n"); bad = 1; }
  if (memcmp(K, Kref, n_kv * 2)) { fprintf(stderr, "appended K rows differ\n"); bad = 1; }
  double worst = 0.0;
  for (int h = 0; h < B * Hq; ++h) {
    double mx = 0.0;
    for (int j = 0; j < D; ++j) mx = fmax(mx, fabs(ref_out[h * D + j]));
    for (int j = 0; j < D; ++j) {
      double r = ref_out[h * D + j], e = fabs(out[h * D + j] - r) / fmax(fabs(r), 1e-3 * mx);
      worst = fmax(worst, e);
    }
  }
  if (!(worst <= 2e-3)) { fprintf(stderr, "attention rel err %g\n", worst); bad = 1; }
  for (int b = 0; b < B; ++b) { /* the copied key (token 123) must be among head 0's selection */
    int found = 0;
    for (int i = 0; i < K_BUDGET; ++i) found |= idx[(b * Hq) * K_BUDGET + i] == 123;
    if (!found) { fprintf(stderr, "sequence %d: token 123 not selected\n", b); bad = 1; }
  }
  /* The staged entry points on the cache as the step left it (new token appended): query codes,
   * distances, top-k, attention over the selected rows; then the step again without an append,
   * through the entry point that allocates nothing.  Indices must equal the fused step's bit for
   * bit, outputs must meet the same bound against the oracle. */
  void *dqcodes, *ddist, *didx2, *dout2;
  HIP_OK(hipMalloc(&dqcodes, B * Hq * 32)); HIP_OK(hipMalloc(&ddist, (size_t)B * Hq * max_len * 2));
  HIP_OK(hipMalloc(&didx2, sizeof idx)); HIP_OK(hipMalloc(&dout2, sizeof out));
  HIP_OK(hipMemset(ddist, 0xEE, (size_t)B * Hq * max_len * 2));
  rc = adamas_encode_query(&cfg, dq, dqcodes, B, NULL);
  if (!rc) rc = adamas_manhattan_distance(&cfg, dqcodes, dcodes, dstart, dlen, B, ddist, max_len, NULL);
  if (!rc) rc = adamas_select_topk(&cfg, dqcodes, dcodes, dstart, dlen, B, K_BUDGET, didx2, NULL, max_len,
                                   dws, ws_bytes, NULL);
  if (!rc) rc = adamas_sparse_attn(&cfg, dq, dK, dV, dstart, didx2, B, K_BUDGET, dout2, max_len, dws,
                                   ws_bytes, NULL);
  if (rc) { fprintf(stderr, "staged calls: %s\n", adamas_status_string(rc)); return 1; }
  HIP_OK(hipDeviceSynchronize());
  float out2[B * Hq * D];
  int32_t idx2[B * Hq * K_BUDGET];
  uint16_t *dist = malloc((size_t)B * Hq * max_len * 2);
  if (!dist) return 2;
  HIP_OK(hipMemcpy(out2, dout2, sizeof out2, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(idx2, didx2, sizeof idx2, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(dist, ddist, (size_t)B * Hq * max_len * 2, hipMemcpyDeviceToHost));
  if (memcmp(idx2, ref_idx, sizeof idx2)) { fprintf(stderr, "staged indices differ\n"); bad = 1; }
  double worst2 = 0.0;
  for (int h = 0; h < B * Hq; ++h) {
    double mx = 0.0;
    for (int j = 0; j < D; ++j) mx = fmax(mx, fabs(ref_out[h * D + j]));
    for (int j = 0; j < D; ++j) {
      double r = ref_out[h * D + j];
      worst2 = fmax(worst2, fabs(out2[h * D + j] - r) / fmax(fabs(r), 1e-3 * mx));
    }
  }
  if (!(worst2 <= 2e-3)) { fprintf(stderr, "staged attention rel err %g\n", worst2); bad = 1; }
  for (int b = 0; b < B; ++b) { /* distances: 0..384 inside the sequence, untouched behind it; the copied key is nearest */
    for (int h = 0; h < Hq; ++h) {
      const uint16_t *dr = dist + ((size_t)b * Hq + h) * max_len;
      for (int t = 0; t < max_len; ++t) {
        if (t < lens[b] ? dr[t] > 384 : dr[t] != 0xEEEE) { fprintf(stderr, "distance [%d][%d][%d] = %u\n", b, h, t, dr[t]); bad = 1; t = max_len; }
      }
    }
    if (dist[(size_t)b * Hq * max_len + 123] != 0) { fprintf(stderr, "sequence %d: distance to its own copy is not 0\n", b); bad = 1; }
  }
  HIP_OK(hipMemset(dout2, 0, sizeof out2)); HIP_OK(hipMemset(didx2, 0xFF, sizeof idx2));
  rc = adamas_decode_step_static(&cfg, dq, NULL, NULL, dK, dV, dcodes, dstart, dlen, B, K_BUDGET, dout2, didx2,
                                 max_len, NULL);
  if (rc) { fprintf(stderr, "decode_step_static: %s\n", adamas_status_string(rc)); return 1; }
  HIP_OK(hipDeviceSynchronize());
  HIP_OK(hipMemcpy(out2, dout2, sizeof out2, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(idx2, didx2, sizeof idx2, hipMemcpyDeviceToHost));
  if (memcmp(idx2, idx, sizeof idx2)) { fprintf(stderr, "static step: indices differ\n"); bad = 1; }
  if (memcmp(out2, out, sizeof out2)) { fprintf(stderr, "static step: output differs from the step's\n"); bad = 1; }
  printf("C ABI client: %s (attention max rel err %.3g fused, %.3g staged)\n", bad ? "FAILED" : "OK", worst, worst2);
  return bad;
}
