/*
 * adamas.h -- C ABI of the MI355X (gfx950) implementation of the Adamas
 * decode-time sparse-attention path (Algorithm 1 of the paper):
 *
 *   Hadamard transform of each query / key head vector      (Alg. 1, Eq. 4)
 *   bucketize into 2-bit codes and pack, 32 B per vector    (Alg. 1, Eq. 5)
 *   append K, V and the code row to the cache               (Alg. 1)
 *   Manhattan distance of the query codes to every cached
 *   key's codes                                             (Alg. 1, Eq. 6)
 *   top-k: the k cached tokens of smallest distance         (Alg. 1)
 *   softmax attention of the original q over the selected
 *   rows of the original K, V                               (Alg. 1, Eq. 1)
 *
 * GENERAL CONVENTIONS
 *
 * Pointers.  `cfg` is HOST memory.  Every other pointer is DEVICE memory of
 * the current HIP device, owned by the caller for the whole call and until
 * the enqueued work has finished.  The library never allocates, frees or
 * synchronises: all work is enqueued on `stream` (a hipStream_t passed as
 * void*; NULL is the default stream) and the call returns at once.
 *
 * Cache layout ("pools").  pool_tokens rows per KV head:
 *     K, V   : bf16   [num_kv_heads][pool_tokens][128]
 *     codes  : uint8  [num_kv_heads][pool_tokens][32]
 * Sequence b of a batch owns rows seq_start[b] .. seq_start[b]+seq_len[b]-1
 * of every KV head (ragged batches are packed into one pool).  Token t of
 * sequence b is pool row seq_start[b]+t.  All indices the library returns
 * are token positions t inside the sequence, not pool rows.  Pools must be
 * 16-byte aligned.
 *
 * Heads.  Query head h reads KV head h / (num_q_heads / num_kv_heads).  With
 * grouped-query attention every query head encodes its own query and picks
 * its own top-k from its group's shared code plane.
 *
 * Code row (32 B).  Four little-endian 64-bit words; word g covers transform
 * coefficients 32g..32g+31 (natural/Sylvester order); bit j is the low bit
 * of the 2-bit code of coefficient 32g+j, bit 32+j its high bit.  This keeps
 * the paper's density of eight codes per 16 bits (1/16 of the bf16 K+V
 * bytes); the paper does not fix a bit order.  (Everything here describes
 * the method itself; the ablation switches further down change the code
 * width -- rows of 16 or 48 bytes -- or the distance estimator.)
 *
 * Codes.  code_j = #{ i : y_j > thr[i] } in {0,1,2,3}, strict comparison,
 * where y = x H / sqrt(128) is the orthonormal transform evaluated EXACTLY:
 * the kernels form the +-1 sums in fp64, which is exact when, within one
 * vector, the binary exponents of the largest and smallest non-zero input
 * differ by at most 38, and compare with (double)thr[i] * sqrt(128.0).  (The
 * bulk encode tries fp32 first and keeps a vector's result only where an
 * error bound proves every comparison equal to the exact one; the other
 * vectors are redone in fp64.)
 * Inputs outside that range, NaN or Inf give unspecified codes.
 *
 * Selection.  The min(k, seq_len) tokens of smallest distance, equal
 * distances ranked by token position (lower first).  Written in ascending
 * token position, padded with -1 up to k entries.  Every cached position,
 * including a token appended by the same call, is a candidate.
 *
 * Errors.  Return 0 on success.  A negative return means nothing was
 * enqueued and no output was touched:
 *     ADAMAS_ERR_BAD_ARG      null pointer, non-positive size, heads not
 *                             divisible, thresholds not strictly increasing,
 *                             non-finite scale, misaligned pool, ...
 *     ADAMAS_ERR_UNSUPPORTED  head_dim not one of those listed below,
 *                             k > ADAMAS_MAX_K,
 *                             group size > ADAMAS_MAX_GROUP,
 *                             max_seq_len > ADAMAS_MAX_SEQ_LEN
 *     ADAMAS_ERR_WORKSPACE    workspace_bytes < adamas_workspace_bytes(...)
 *     ADAMAS_ERR_HIP          a launch failed (adamas_last_hip_error() tells)
 * seq_len[b] and seq_start[b] live on the device, so the host cannot reject
 * them: the caller guarantees 0 <= seq_len[b] <= max_seq_len and
 * 0 <= seq_start[b], seq_start[b]+seq_len[b] <= pool_tokens.  The kernels
 * check the same conditions and treat a sequence that violates them as empty
 * (out zeros, idx all -1, nothing appended): no access leaves the pools.
 *
 * Workspace.  Calls that take `workspace` need at least
 * adamas_workspace_bytes(cfg, batch, max_seq_len, k) bytes, 256-byte aligned.
 * Its contents need no initialisation and carry nothing between calls, but
 * two calls that may run concurrently must not share one workspace.
 */
#ifndef ADAMAS_H
#define ADAMAS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADAMAS_HEAD_DIM 128
#define ADAMAS_CODE_ROW_BYTES 32
#define ADAMAS_MAX_DISTANCE 384          /* 3 * 128 (Eq. 6) */
#define ADAMAS_MAX_DISTANCE_L2 1152      /* 9 * 128 (ADAMAS_VARIANT_L2) */
#define ADAMAS_MAX_K 4096                /* largest budget in the paper's tables */
#define ADAMAS_MAX_GROUP 8               /* query heads per KV head */
#define ADAMAS_MAX_SEQ_LEN (1 << 20)

#define ADAMAS_OK 0
#define ADAMAS_ERR_BAD_ARG (-1)
#define ADAMAS_ERR_UNSUPPORTED (-2)
#define ADAMAS_ERR_WORKSPACE (-3)
#define ADAMAS_ERR_HIP (-4)

/*
 * Ablation variants of Section 4.4, as switches on the same kernels.  They
 * apply to every entry point that takes the config; a cache must be encoded
 * and queried with the same ADAMAS_VARIANT_NO_HADAMARD setting.
 *   NO_HADAMARD  Eq. 5 is applied to the raw vector: no transform, thresholds
 *                compared with the elements as given.
 *   L2           tokens are ranked by sum_j (qcode_j - kcode_j)^2 instead of
 *                Eq. 6 (no square root: it would not change the ranking);
 *                distances then range over 0..ADAMAS_MAX_DISTANCE_L2.
 * Other bits -> ADAMAS_ERR_UNSUPPORTED.
 * The bucketization ablation (1-bit and 3-bit codes) is adamas_config.code_bits:
 * 2^code_bits - 1 thresholds, code rows of 16 * code_bits bytes (four words of
 * code_bits 32-bit planes: plane p of word g holds, at bit j, bit p of the code
 * of coefficient 32g + j; for 2 bits that is the 32-byte row described above),
 * distances 0..(2^code_bits - 1) * 128.  Every `codes` / `qcodes` buffer then
 * has rows of that size.  L2 needs 2-bit codes (else ADAMAS_ERR_UNSUPPORTED).
 */
#define ADAMAS_VARIANT_NO_HADAMARD 1u
#define ADAMAS_VARIANT_L2 2u

/*
 * Head dimension d.  The text above and below is written for d = 128, the
 * head dimension of the paper's models.  head_dim 64 and 256 (powers of two:
 * Sylvester's H_d, Eq. 2) and 96, 160, 192 (d = 2^n * m with m = 12 or 20:
 * H_d = H_{2^n} (x) H_m, Section 2 under Eq. 2, with Paley's Hadamard matrix
 * of order m built from the quadratic residues mod m - 1; the paper names no
 * H_12 / H_20, so codes at these dimensions are this library's own) run
 * everything as well: every ablation switch, contiguous or paged cache, every
 * entry point.  Read d for 128 and d/4 for the 32-byte code row (d/32 words of
 * 64 bits, same bit placement; 16 * code_bits * d/128 bytes with the
 * code-width switch), distances 0..3d, sm_scale 0 meaning 1/sqrt(d),
 * thresholds compared with x H / sqrt(d).  Other head dimensions ->
 * ADAMAS_ERR_UNSUPPORTED (a code row needs d to be a multiple of 32).
 */
typedef struct adamas_config {
  int32_t head_dim;      /* 128; or 64, 96, 160, 192, 256 (see above) */
  int32_t num_q_heads;   /* Hq */
  int32_t num_kv_heads;  /* Hkv; Hq % Hkv == 0 */
  uint32_t variant;      /* 0 = the method; else ADAMAS_VARIANT_* flags (Sec. 4.4 ablations) */
  int64_t pool_tokens;   /* rows per KV head in K, V and codes */
  float thr_k[7];        /* key thresholds B1 < B2 < ... of Eq. 5, orthonormal scale; the first
                            2^code_bits - 1 are used (three for the method) */
  float thr_q[7];        /* query thresholds (the paper uses one set: pass the same) */
  float sm_scale;        /* softmax scale of Eq. 1; 0 means 1/sqrt(head_dim) */
  int32_t code_bits;     /* 0 or 2: 2-bit codes (the method); 1, 3: bucketization ablation */
} adamas_config;

/* Human-readable name of a status code; never NULL. */
const char *adamas_status_string(int status);

/* Identifies the build: a hash of the sources and compiler flags the library
 * was made from ("unknown" when built without one).  Never NULL. */
const char *adamas_build_id(void);

/* hipError_t (as int) of the launch that made the last call on this thread
 * return ADAMAS_ERR_HIP; 0 if none. */
int adamas_last_hip_error(void);

/* Bytes of workspace the calls below need for these sizes; 0 if the
 * arguments are invalid or unsupported.  Host-only, enqueues nothing. */
size_t adamas_workspace_bytes(const adamas_config *cfg, int32_t batch,
                              int64_t max_seq_len, int32_t k);

/*
 * Alg. 1, transform / bucketize / pack steps (Eq. 4, Eq. 5), for cached
 * keys (prefill-time bulk encode): for every KV head, transform, bucketize
 * (thr_k) and pack pool rows
 * [row_begin, row_begin + n_rows) of K into the same rows of codes.
 * K: bf16 [Hkv][pool_tokens][128] (read), codes: uint8 [Hkv][pool_tokens][32]
 * (written).  n_rows == 0 is a no-op.
 */
int adamas_encode_keys(const adamas_config *cfg, const void *K, void *codes,
                       int64_t row_begin, int64_t n_rows, void *stream);

/*
 * The same steps of Alg. 1 for queries: q bf16 [batch][Hq][128] -> qcodes
 * uint8 [batch][Hq][32], thresholds thr_q.
 */
int adamas_encode_query(const adamas_config *cfg, const void *q, void *qcodes,
                        int32_t batch, void *stream);

/*
 * Alg. 1, distance step (Eq. 6):
 *   dist_out[b][h][t] = sum_j |qcode[b][h]_j - code[kv(h)][seq_start[b]+t]_j|
 * for t < seq_len[b]; entries t >= seq_len[b] are left untouched.
 * qcodes uint8 [batch][Hq][32]; seq_start int64 [batch]; seq_len int32 [batch];
 * dist_out uint16 [batch][Hq][max_seq_len], values 0..384 (other ranges with
 * the ablation switches: see ADAMAS_VARIANT_L2 and code_bits).
 */
int adamas_manhattan_distance(const adamas_config *cfg, const void *qcodes,
                              const void *codes, const int64_t *seq_start,
                              const int32_t *seq_len, int32_t batch,
                              uint16_t *dist_out, int64_t max_seq_len,
                              void *stream);

/*
 * Alg. 1, distance and top-k steps: distances as above, then the top-k selection described
 * under "Selection".  idx_out int32 [batch][Hq][k].  dist_out may be NULL;
 * otherwise it receives the distances as in adamas_manhattan_distance.
 */
int adamas_select_topk(const adamas_config *cfg, const void *qcodes,
                       const void *codes, const int64_t *seq_start,
                       const int32_t *seq_len, int32_t batch, int32_t k,
                       int32_t *idx_out, uint16_t *dist_out,
                       int64_t max_seq_len, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * Alg. 1, gather and attention steps (Eq. 1): out[b][h] = softmax(q[b][h] . K_s^T * sm_scale) V_s
 * over the rows idx[b][h][0..k) of sequence b (token positions; negative
 * entries are skipped; no valid entry -> zeros).  q bf16 [batch][Hq][128];
 * idx int32 [batch][Hq][k]; out fp32 [batch][Hq][128].  Scores are formed in
 * fp64, weights and weighted sums in fp32; the caller guarantees 0 <= idx < seq_len[b] for non-negative entries.
 * max_seq_len is only used to size the workspace (pass the same value as to
 * adamas_workspace_bytes).
 */
int adamas_sparse_attn(const adamas_config *cfg, const void *q, const void *K,
                       const void *V, const int64_t *seq_start,
                       const int32_t *idx, int32_t batch, int32_t k, float *out,
                       int64_t max_seq_len, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * One whole decode step of one attention layer (all of Alg. 1), fused:
 * encodes q (and k_new), appends, scans, selects and attends.
 *
 * k_new, v_new: bf16 [batch][Hkv][128], or both NULL for "no append".  With
 * an append, seq_len[b] already counts the new token; its K, V and code row
 * are written to pool row seq_start[b]+seq_len[b]-1 before the scan, so it
 * is a candidate like any other (sequences with seq_len[b] == 0 append
 * nothing).  K, V, codes are therefore read AND written.
 * out fp32 [batch][Hq][128]; idx_out int32 [batch][Hq][k] or NULL.
 */
int adamas_decode_step(const adamas_config *cfg, const void *q,
                       const void *k_new, const void *v_new, void *K, void *V,
                       void *codes, const int64_t *seq_start,
                       const int32_t *seq_len, int32_t batch, int32_t k,
                       float *out, int32_t *idx_out, int64_t max_seq_len,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * adamas_decode_step for callers that cannot allocate device memory or pass a
 * workspace along: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and errors as
 * adamas_decode_step, minus `workspace`: the kernels' scratch (distances, tile
 * histograms, attention partials) lives in a device array of
 * ADAMAS_STATIC_SCRATCH_BYTES that is part of the library's code object; every
 * GPU the library runs on holds its own copy until the process ends.  The call
 * allocates and frees nothing.  Sizes whose scratch would exceed the array
 * (adamas_workspace_bytes(cfg, batch, max_seq_len, k) >
 * ADAMAS_STATIC_SCRATCH_BYTES) -> ADAMAS_ERR_WORKSPACE, nothing enqueued.
 * All calls on one GPU share that GPU's array: two calls whose work may overlap
 * on one GPU (different streams, different threads) race; calls on one stream
 * are ordered and safe.  The first call on each device looks the array's
 * address up (a HIP runtime query, no allocation); make that call outside a
 * graph capture.
 */
#define ADAMAS_STATIC_SCRATCH_BYTES (16u << 20)
int adamas_decode_step_static(const adamas_config *cfg, const void *q,
                              const void *k_new, const void *v_new, void *K,
                              void *V, void *codes, const int64_t *seq_start,
                              const int32_t *seq_len, int32_t batch, int32_t k,
                              float *out, int32_t *idx_out, int64_t max_seq_len,
                              void *stream);

/*
 * Profiling hook: adamas_decode_step cut at its one internal kernel
 * boundary.  `stages` is a bit mask; ADAMAS_STAGE_ALL is exactly
 * adamas_decode_step.  ADAMAS_STAGE_SCAN runs Alg. 1 up to the distance
 * step (query encode, append, distance scan; leaves distances and
 * histograms in the workspace, writes neither out nor idx_out).
 * ADAMAS_STAGE_SELECT_ATTN runs the top-k, gather and attention steps on
 * what a preceding ADAMAS_STAGE_SCAN call with the same arguments left in
 * the same workspace; without such a call its outputs are unspecified
 * (all accesses stay in bounds).  Same arguments and errors as
 * adamas_decode_step; stages outside 1..3 -> ADAMAS_ERR_BAD_ARG.
 */
#define ADAMAS_STAGE_SCAN 1u
#define ADAMAS_STAGE_SELECT_ATTN 2u
#define ADAMAS_STAGE_ALL 3u
int adamas_decode_step_stages(const adamas_config *cfg, const void *q,
                              const void *k_new, const void *v_new, void *K,
                              void *V, void *codes, const int64_t *seq_start,
                              const int32_t *seq_len, int32_t batch, int32_t k,
                              float *out, int32_t *idx_out, int64_t max_seq_len,
                              void *workspace, size_t workspace_bytes,
                              void *stream, uint32_t stages);

/*
 * Profiling hook, for libraries built with -DADAMAS_PHASE_TRACE only (an
 * ordinary build returns ADAMAS_ERR_UNSUPPORTED and has no stamping code in
 * its kernels).  After this call every workgroup of the two kernels of
 * adamas_decode_step / _stages / _paged leaves a record of ADAMAS_TRACE_SLOTS
 * uint64 in scan_records / select_records (device memory, n_records records
 * each, indexed by the workgroup's linear index in its grid; workgroups beyond
 * n_records leave nothing; either pointer may be NULL): the 100 MHz wall clock
 * at the kernel's phase boundaries, in the order of enum ScanPhase /
 * SelectPhase of the kernel sources, 0 where a workgroup did not pass a
 * boundary.  NULL, NULL, 0 switches the stamps off.  Process-wide state, not
 * thread-safe; the buffers must stay valid while traced calls run.
 */
#define ADAMAS_TRACE_SLOTS 16
int adamas_phase_trace(void *scan_records, void *select_records, int64_t n_records);

/*
 * adamas_decode_step on a PAGED cache, the layout of the serving engines the
 * paper compares with (Section 4.1): the pools are cut into pages of
 * page_tokens rows (a power of two, 64..4096; pool_tokens a multiple of it)
 * and token t of sequence b lives in pool row
 *     page_table[b * max_pages + t / page_tokens] * page_tokens + t % page_tokens
 * of every KV head.  page_table: device int32 [batch][max_pages]; entries for
 * pages a sequence does not use are never read beyond being clamped into the
 * pool; an entry outside the pool is clamped into it (wrong rows, no fault).
 * With an append the table must already name the page of the new token
 * (position seq_len[b]-1).  idx_out holds token positions, as in
 * adamas_decode_step.  max_seq_len <= max_pages * page_tokens.  stages:
 * ADAMAS_STAGE_ALL, or ADAMAS_STAGE_SCAN to time the scan alone (other values
 * -> ADAMAS_ERR_BAD_ARG).  Everything else (arguments, workspace size, errors,
 * variants) as adamas_decode_step.
 */
int adamas_decode_step_paged(const adamas_config *cfg, const void *q,
                             const void *k_new, const void *v_new, void *K,
                             void *V, void *codes, const int32_t *page_table,
                             int32_t max_pages, int32_t page_tokens,
                             const int32_t *seq_len, int32_t batch, int32_t k,
                             float *out, int32_t *idx_out, int64_t max_seq_len,
                             void *workspace, size_t workspace_bytes,
                             void *stream, uint32_t stages);

/*
 * Comparison point, not a step of the method: Eq. 1 over ALL cached rows of
 * every sequence (dense decode attention), the baseline of the paper's
 * "self-attention speedup" (Sec. 4.3), so that both sides of that ratio can be
 * measured on one GPU.  q bf16 [batch][Hq][128]; K, V pools as above;
 * out fp32 [batch][Hq][128] (zeros for an empty sequence).  Workspace:
 * adamas_full_attn_workspace_bytes(cfg, batch, max_seq_len) bytes, 256-byte
 * aligned, no initialisation needed.  Same argument checks and error codes as
 * adamas_sparse_attn.
 */
size_t adamas_full_attn_workspace_bytes(const adamas_config *cfg, int32_t batch,
                                        int64_t max_seq_len);
int adamas_full_attn(const adamas_config *cfg, const void *q, const void *K,
                     const void *V, const int64_t *seq_start,
                     const int32_t *seq_len, int32_t batch, float *out,
                     int64_t max_seq_len, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * Measurement aid, not a step of the method: reads `bytes` bytes of device
 * memory at `src` once, 32 bytes per lane in the scan's access pattern, does
 * no arithmetic on them and writes nothing (`sink`, device, at least 4 bytes,
 * is only touched if the data's checksum hits one particular value).  Timing
 * it over the code planes gives the streaming-read rate this GPU reaches on
 * the buffers the Eq. 6 scan must read: the achievable ceiling that the scan's
 * time is compared with.  src 16-byte aligned, bytes a multiple of 32;
 * bytes == 0 is a no-op.  ADAMAS_ERR_BAD_ARG otherwise.
 */
int adamas_stream_read(const void *src, size_t bytes, void *sink, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* ADAMAS_H */
