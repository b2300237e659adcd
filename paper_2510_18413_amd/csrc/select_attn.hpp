// Top-k selection from the scan's distances and tile histograms (Algorithm 1,
// top-k step) and softmax attention over the selected rows (its gather and
// attention steps, Eq. 1).
//
// Selection without sorting.  Distances take few values (385 for Eq. 6, 1153
// for the squared-difference variant), so the k-th smallest
// is found from the head's histogram: T = smallest distance whose cumulative
// count reaches kk = min(k, L).  Every token with distance < T is selected,
// plus the first r = kk - #{D < T} tokens (in token order) with distance == T:
// exactly the k smallest under (distance, token position) order.  A selected
// token's slot in the ascending output is the number of selected tokens before
// it, #{D<T before} + min(#{D==T before}, r), which each workgroup gets from
// the tile histograms of earlier tiles plus a prefix scan inside its segment.
//
// One workgroup (256 threads) owns one segment of one (sequence, query head).
// With attention enabled it then gathers the K, V rows it selected, runs a
// one-pass online softmax over them (16 lanes per row, 8 dims per lane, fp32)
// and leaves an (m, l, o[128]) partial.  Inside the fused step the partials of
// a head are combined, in segment order, by whichever of its workgroups
// finishes last (a per-head arrival counter that the scan kernel zeroed).
// Partials and counter are exchanged through device-scope atomic stores, loads
// and one fetch-add, which are coherent across the chip by themselves, so no
// device-scope fence is needed (on this part such a fence walks the XCD's whole
// L2 and costs more than a kernel boundary).  Without a zeroed counter (staged
// calls, stand-alone attention) a small follow-up kernel does the same merge.
#pragma once

#include "device_utils.hpp"

namespace adamas {

constexpr int kSelTokPerThread = 16;
constexpr int kHistBatch = 16;               // tiles whose histograms are loaded together
constexpr int kMaxParts = 16;  // attention partial slots per head in the workspace
constexpr int kMaxK = 4096;
constexpr float kNegBig = -1.0e30f;

struct SelectParams {
  const uint16_t* dist;       // [B*Hq][dist_stride]
  int64_t dist_stride;
  const uint16_t* tilehist;   // [B*Hq][n_tiles][Dist<METRIC>::kStride]
  const int64_t* seq_start;   // [B]
  const int32_t* seq_len;     // [B]
  int32_t* idx_out;           // [B*Hq][k] or null
  const uint16_t* q;          // bf16 [B*Hq][128]
  const uint16_t* K;          // pools
  const uint16_t* V;
  float* out;                 // [B*Hq][128]
  float* partial;             // [B*Hq][kMaxParts][partial_stride(D)]
  uint32_t* arrivals;         // per-head counter of finished segments, zero on entry; null: no in-kernel merge
  int64_t arrivals_stride;
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, Hkv, k;
  int32_t n_tiles, tile_tokens, seg_len;
  double scale_log2e;         // sm_scale * log2(e)
  // Paged cache (PAGED kernels only), as in ScanParams.
  const int32_t* page_table;
  int32_t max_pages, page_shift;
  // Profiling builds only: one record of phase stamps per workgroup (see PhaseTrace).
  uint64_t* trace;
  int64_t trace_records;
};

// Phase stamps of select_kernel, in the order they are taken.
enum SelectPhase {
  kSelStart = 0,      // first instruction
  kSelLoaded,         // distances, tile histograms and the sequence length have arrived
  kSelThreshold,      // T and r known to every thread
  kSelCompacted,      // the segment's selected positions are in LDS / idx_out
  kSelRowsFirst,      // the first batch of K, V rows has arrived
  kSelAttended,       // all rows of the segment consumed
  kSelCombined,       // the row groups' states combined through LDS
  kSelPartialAcked,   // the partial's stores acknowledged
  kSelCounted,        // the arrival counter returned
  kSelMerged,         // (merging workgroup only) partials read back and combined
  kSelEnd
};

// Exclusive prefix sum over a workgroup of THREADS threads (a multiple of 64).
// s_wave must hold THREADS/64 words.  Two barriers inside; all threads call it.
template <int THREADS>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* s_wave, uint32_t& total) {
  constexpr int NW = THREADS / kWave;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_incl_scan_u32(v);
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t x = s_wave[w];
    before += w < wave ? x : 0u;
    all += x;
  }
  total = all;
  __syncthreads();
  return before + incl - v;
}

template <int THREADS, int D = kHeadDim>
struct AttnShared {
  static constexpr int kGroups = THREADS / (D / 8);
  float m[kGroups];
  float l[kGroups];
  float acc[kGroups][D];
};

// Softmax attention (Eq. 1) of one query over the n rows listed in s_sel (token
// positions; Kp, Vp point at the sequence's first row of the right KV head),
// by the whole workgroup: 16 lanes per row, 8 dims per lane, one-pass online
// softmax per 16-lane group in fp32 (exp2 domain), groups combined in fixed
// order through LDS.  Threads 0..127 receive, for output dim tid: M (running
// maximum), lsum (sum of weights) and o (unnormalised weighted sum of V).
// Entries of s_sel are clamped to [0, n_tokens) before use (n_tokens >= 1 when n > 0).
// All threads must call it.
template <int THREADS, int D>
__device__ __forceinline__ void attention_rows(const int32_t* s_sel, int n, int n_tokens,
                                               const uint16_t* __restrict__ q,
                                               const uint16_t* __restrict__ Kp,
                                               const uint16_t* __restrict__ Vp, double scale_log2e,
                                               AttnShared<THREADS, D>& sh, float& M, float& lsum,
                                               float& o, PhaseTrace& trace) {
  // Scores in fp64: products of bf16 values are exact, and so (for all practical
  // purposes) is their sum.  An fp32 dot product of 128 terms is off by about
  // 1e-5 in the exponent of a weight; where the weighted rows nearly cancel that
  // becomes 1e-3 of the output.  Only the difference between a score and the
  // running maximum (itself a float, so that every weight of a head refers to
  // exactly the same number) is rounded to fp32, and rows with equal scores get
  // equal weights.  No implicit FMA contraction in the fp32 part.
#pragma clang fp contract(off)
  constexpr int LPR = D / 8;  // lanes per row: 8 dims each
  constexpr int kGroups = THREADS / LPR;
  const int tid = threadIdx.x, grp = tid / LPR, gl = tid % LPR;

  double qf[8];
  {
    const uint4 qv = *reinterpret_cast<const uint4*>(q + gl * 8);
    qf[0] = bf16_lo(qv.x); qf[1] = bf16_hi(qv.x); qf[2] = bf16_lo(qv.y); qf[3] = bf16_hi(qv.y);
    qf[4] = bf16_lo(qv.z); qf[5] = bf16_hi(qv.z); qf[6] = bf16_lo(qv.w); qf[7] = bf16_hi(qv.w);
  }
  float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;

  constexpr int U = 4;  // rows in flight per 16-lane group
  for (int i0 = grp; i0 < n; i0 += kGroups * U) {
    uint4 kv[U], vv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * kGroups;
      ok[u] = i < n;
      if (ok[u]) {
        // clamped: whatever the list holds, the gather stays inside the sequence
        const int tok = min(max(s_sel[i], 0), n_tokens - 1);
        const int64_t off = (int64_t)tok * D + gl * 8;
        kv[u] = *reinterpret_cast<const uint4*>(Kp + off);
        vv[u] = *reinterpret_cast<const uint4*>(Vp + off);
      } else {
        kv[u] = make_uint4(0, 0, 0, 0);
        vv[u] = make_uint4(0, 0, 0, 0);
      }
    }
    if (i0 == grp) trace.stamp(kSelRowsFirst);
    double sc[U];
    float mn = m;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // two chains of four: the additions of a chain wait for each other
      double s = qf[0] * (double)bf16_lo(kv[u].x), s2 = qf[1] * (double)bf16_hi(kv[u].x);
      s = fma(qf[2], (double)bf16_lo(kv[u].y), s);
      s2 = fma(qf[3], (double)bf16_hi(kv[u].y), s2);
      s = fma(qf[4], (double)bf16_lo(kv[u].z), s);
      s2 = fma(qf[5], (double)bf16_hi(kv[u].z), s2);
      s = fma(qf[6], (double)bf16_lo(kv[u].w), s);
      s2 = fma(qf[7], (double)bf16_hi(kv[u].w), s2);
      s += s2;
      // the row's D / 8 lanes are an aligned group of 8, 16 or 32 lanes
      s = lanes_sum_f64<LPR>(s) * scale_log2e;
      sc[u] = ok[u] ? s : (double)kNegBig;
      mn = fmaxf(mn, (float)sc[u]);
    }
    // one rescale of the running state for the whole batch of rows
    const float corr = exp2f(m - mn);
    m = mn;
    l *= corr;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] *= corr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float pw = ok[u] ? exp2f((float)(sc[u] - (double)mn)) : 0.f;
      l += pw;
      acc[0] = fmaf(pw, bf16_lo(vv[u].x), acc[0]);
      acc[1] = fmaf(pw, bf16_hi(vv[u].x), acc[1]);
      acc[2] = fmaf(pw, bf16_lo(vv[u].y), acc[2]);
      acc[3] = fmaf(pw, bf16_hi(vv[u].y), acc[3]);
      acc[4] = fmaf(pw, bf16_lo(vv[u].z), acc[4]);
      acc[5] = fmaf(pw, bf16_hi(vv[u].z), acc[5]);
      acc[6] = fmaf(pw, bf16_lo(vv[u].w), acc[6]);
      acc[7] = fmaf(pw, bf16_hi(vv[u].w), acc[7]);
    }
  }

  trace.stamp(kSelAttended);
  if (gl == 0) {
    sh.m[grp] = m;
    sh.l[grp] = l;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) sh.acc[grp][gl * 8 + j] = acc[j];
  __syncthreads();

  M = kNegBig;
  lsum = 0.f;
  o = 0.f;
  if (tid < D) {
    for (int g = 0; g < kGroups; ++g) M = fmaxf(M, sh.m[g]);
    for (int g = 0; g < kGroups; ++g) {
      const float w = exp2f(sh.m[g] - M);
      lsum = fmaf(sh.l[g], w, lsum);
      o = fmaf(sh.acc[g][tid], w, o);
    }
  }
}

// Grid (n_segs, Hq, B).  With ATTN a head that has a single segment with
// tokens is finished by that workgroup; otherwise each workgroup leaves an
// (M, lsum, o[128]) partial, merged by the last one to arrive (p.arrivals set)
// or by merge_kernel (p.arrivals null).
template <int THREADS, bool ATTN, int METRIC, bool PAGED, int D>
__global__ __launch_bounds__(THREADS) void select_kernel(const SelectParams p) {
  static_assert(ATTN || !PAGED, "only the gather needs the page table");
  static_assert(THREADS >= D, "one thread per output dimension in the merge");
  constexpr int kNumBins = Dist<METRIC, D>::kBins, kHistStride = Dist<METRIC, D>::kStride;
  constexpr int kPartial = partial_stride(D);
  constexpr int kHistPairs = kHistStride / 2;                      // pairs of uint16 bins per stored row
  constexpr int PP = (kHistPairs + THREADS - 1) / THREADS;         // pairs owned by one thread
  constexpr int BPL = (kNumBins + kWave - 1) / kWave;              // bins per lane in the threshold search
  constexpr int kTot = BPL * kWave;
  constexpr int PASS = THREADS * kSelTokPerThread;           // tokens per pass
  __shared__ uint32_t s_tot[kTot];
  __shared__ uint32_t s_scan[THREADS / kWave];
  __shared__ int32_t s_T, s_cntlt;
  __shared__ uint32_t s_ltb, s_eqb;
  __shared__ int32_t s_sel[ATTN ? kMaxK : 1];
  __shared__ AttnShared<ATTN ? THREADS : D / 8, D> s_attn;

  PhaseTrace trace;
  trace.stamp(kSelStart);
  const int seg = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const int seg_t0 = seg * p.seg_len;

  // Nothing below depends on the sequence length until the loads are issued:
  // the workspace rows exist up to dist_stride / n_tiles whatever L is, and
  // what lies beyond L is masked once L has arrived.
  const uint16_t* drow = p.dist + head * p.dist_stride;
  // distances of this thread for the current pass and the next one (rolling prefetch)
  uint4 cur_a, cur_b, nxt_a, nxt_b;
  {
    const int o0 = tid * kSelTokPerThread, o1 = PASS + tid * kSelTokPerThread;
    if (o0 < p.seg_len && seg_t0 + o0 < p.dist_stride) {
      const uint4* src = reinterpret_cast<const uint4*>(drow + seg_t0 + o0);
      cur_a = src[0];
      cur_b = src[1];
    } else {
      cur_a = cur_b = make_uint4(0, 0, 0, 0);
    }
    if (o1 < p.seg_len && seg_t0 + o1 < p.dist_stride) {
      const uint4* src = reinterpret_cast<const uint4*>(drow + seg_t0 + o1);
      nxt_a = src[0];
      nxt_b = src[1];
    } else {
      nxt_a = nxt_b = make_uint4(0, 0, 0, 0);
    }
  }
  // Paged cache: a thread's 16 consecutive tokens share one page; its number is
  // fetched like the distances, a pass ahead, and used when rows are emitted.
  int32_t cur_pg = 0, nxt_pg = 0;
  if constexpr (PAGED) {
    const int32_t* prow = p.page_table + (int64_t)b * p.max_pages;
    const int t_a = seg_t0 + tid * kSelTokPerThread;
    cur_pg = prow[min(t_a >> p.page_shift, p.max_pages - 1)];
    nxt_pg = prow[min((t_a + PASS) >> p.page_shift, p.max_pages - 1)];
  }
  // Tile histograms: a thread owns PP pairs of bins, pair tid + j * THREADS (one
  // 32-bit load per pair and tile); pairs past the row repeat its last pair.
  const uint16_t* hrow = p.tilehist + head * p.n_tiles * kHistStride;
  const int first_tile = seg_t0 / p.tile_tokens;
  int pair[PP];
#pragma unroll
  for (int j = 0; j < PP; ++j) pair[j] = min(tid + j * THREADS, kHistPairs - 1);
  uint32_t hv[PP][kHistBatch];
#pragma unroll
  for (int u = 0; u < kHistBatch; ++u) {  // clamped, branch-free: all loads in flight together
    const uint32_t* trow =
        reinterpret_cast<const uint32_t*>(hrow + (int64_t)min(u, p.n_tiles - 1) * kHistStride);
#pragma unroll
    for (int j = 0; j < PP; ++j) hv[j][u] = trow[pair[j]];
  }

  const int L = PAGED ? safe_paged_len(p.seq_len, b, p.max_seq_len, (int64_t)p.max_pages << p.page_shift)
                      : safe_seq_len(p.seq_len, p.seq_start, b, p.max_seq_len, p.pool_tokens);
  const int kk = min(p.k, L);
  const int n_active = max(1, (L + p.seg_len - 1) / p.seg_len);  // segments that hold tokens
  if (seg >= n_active) return;
  trace.stamp(kSelLoaded);
  const int seg_t1 = min(L, seg_t0 + p.seg_len);
  const int tiles_active = (L + p.tile_tokens - 1) / p.tile_tokens;

  // Head histogram (all tiles with tokens) and the part of it before this segment.
  uint32_t tot0[PP], tot1[PP], pre0[PP], pre1[PP];
#pragma unroll
  for (int j = 0; j < PP; ++j) tot0[j] = tot1[j] = pre0[j] = pre1[j] = 0;
  for (int tb = 0; tb < tiles_active; tb += kHistBatch) {
    if (tb > 0) {
#pragma unroll
      for (int u = 0; u < kHistBatch; ++u) {
        const uint32_t* trow = reinterpret_cast<const uint32_t*>(
            hrow + (int64_t)min(tb + u, p.n_tiles - 1) * kHistStride);
#pragma unroll
        for (int j = 0; j < PP; ++j) hv[j][u] = trow[pair[j]];
      }
    }
#pragma unroll
    for (int u = 0; u < kHistBatch; ++u) {
#pragma unroll
      for (int j = 0; j < PP; ++j) {
        const uint32_t v = tb + u < tiles_active ? hv[j][u] : 0u;
        tot0[j] += v & 0xffffu;
        tot1[j] += v >> 16;
        if (tb + u < first_tile) {
          pre0[j] += v & 0xffffu;
          pre1[j] += v >> 16;
        }
      }
    }
  }
  // Head histogram into LDS: a thread writes the bins of its pairs (bins past
  // kNumBins hold nothing and count as zero), the tail up to kTot is cleared.
#pragma unroll
  for (int j = 0; j < PP; ++j) {
    const int pr = tid + j * THREADS;
    if (pr < kHistPairs) {
      s_tot[2 * pr] = 2 * pr < kNumBins ? tot0[j] : 0u;
      s_tot[2 * pr + 1] = 2 * pr + 1 < kNumBins ? tot1[j] : 0u;
    }
  }
  for (int i = kHistStride + tid; i < kTot; i += THREADS) s_tot[i] = 0u;
  if (tid == 0) {
    s_ltb = 0u;
    s_eqb = 0u;
    s_T = 0;
    s_cntlt = 0;
  }
  __syncthreads();

  // Threshold distance T and #{D < T}, by one wave: BPL bins per lane.
  if (tid < kWave) {
    uint32_t c[BPL], sum = 0;
#pragma unroll
    for (int j = 0; j < BPL; ++j) {
      c[j] = s_tot[lane * BPL + j];
      sum += c[j];
    }
    const uint32_t incl = wave_incl_scan_u32(sum);
    uint32_t run = incl - sum;
    if (kk > 0 && run < (uint32_t)kk && incl >= (uint32_t)kk) {
#pragma unroll
      for (int j = 0; j < BPL; ++j) {
        if (run < (uint32_t)kk && run + c[j] >= (uint32_t)kk) {
          s_T = lane * BPL + j;
          s_cntlt = (int32_t)run;
        }
        run += c[j];
      }
    }
  }
  __syncthreads();
  const int T = s_T;
  const int r = kk - s_cntlt;  // ties at distance T to take, lowest positions first
  trace.stamp(kSelThreshold);

  if (gridDim.x > 1) {  // tokens of earlier segments: #{D < T} and #{D == T}
    uint32_t ltb = 0, eqb = 0;
#pragma unroll
    for (int j = 0; j < PP; ++j) {
      const int pr = tid + j * THREADS, bin0 = 2 * pr, bin1 = 2 * pr + 1;
      if (pr < kHistPairs) {
        ltb += (bin0 < T ? pre0[j] : 0u) + (bin1 < T ? pre1[j] : 0u);
        eqb += (bin0 == T ? pre0[j] : 0u) + (bin1 == T ? pre1[j] : 0u);
      }
    }
    ltb = wave_sum_u32(ltb);
    eqb = wave_sum_u32(eqb);
    if (lane == 0) {
      atomicAdd(&s_ltb, ltb);
      atomicAdd(&s_eqb, eqb);
    }
    __syncthreads();
  }
  uint32_t run_lt = s_ltb, run_eq = s_eqb;
  const uint32_t seg_pos0 = run_lt + min(run_eq, (uint32_t)r);
  int32_t* idx_row = p.idx_out != nullptr ? p.idx_out + head * p.k : nullptr;

  for (int pass_t0 = seg_t0; pass_t0 < seg_t1; pass_t0 += PASS) {
    const int t = pass_t0 + tid * kSelTokPerThread;
    const uint4 da = cur_a, db = cur_b;
    cur_a = nxt_a;
    cur_b = nxt_b;
    if (t + 2 * PASS < seg_t1) {  // fetch the pass after next while this one is processed
      const uint4* src = reinterpret_cast<const uint4*>(drow + t + 2 * PASS);
      nxt_a = src[0];
      nxt_b = src[1];
    }
    int64_t page_row0 = 0;  // pool row of token t's page, minus the page offset of t itself
    if constexpr (PAGED) {
      const int64_t pg = min(max((int64_t)cur_pg, (int64_t)0), (p.pool_tokens >> p.page_shift) - 1);
      page_row0 = (pg << p.page_shift) + (t & ((1 << p.page_shift) - 1));
      cur_pg = nxt_pg;
      if (t + 2 * PASS < seg_t1)
        nxt_pg = p.page_table[(int64_t)b * p.max_pages +
                              min((t + 2 * PASS) >> p.page_shift, p.max_pages - 1)];
    }
    // Two distances per 32-bit word.  Per half-word, without unpacking:
    //   d < T  <=> bit 15 of (d - T) mod 2^16   (both below 2^15)
    //   d == T <=> (z - 1) & ~z has bit 15 set, z = d ^ T
    // Bit j of m_lt / m_eq stands for token t + j.
    const uint32_t words[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
    const uint32_t TT = (uint32_t)T * 0x00010001u;
    uint32_t m_lt = 0, m_eq = 0;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      const uint32_t y = pk_sub_u16(words[w], TT) & 0x80008000u;
      const uint32_t z = words[w] ^ TT;
      const uint32_t e = pk_sub_u16(z, 0x00010001u) & ~z & 0x80008000u;
      m_lt |= (((y >> 15) & 1u) | (y >> 30)) << (2 * w);
      m_eq |= (((e >> 15) & 1u) | (e >> 30)) << (2 * w);
    }
    const int n_valid = min(max(seg_t1 - t, 0), kSelTokPerThread);
    const uint32_t vmask = (1u << n_valid) - 1u;
    m_lt &= vmask;
    m_eq &= vmask;
    uint32_t total;
    const uint32_t ex =
        block_excl_scan<THREADS>((uint32_t)__popc(m_lt) | ((uint32_t)__popc(m_eq) << 16), s_scan, total);
    uint32_t lt = run_lt + (ex & 0xffffu), eq = run_eq + (ex >> 16);
    // Visit only the candidate tokens (set bits), in position order.
    uint32_t cand = m_lt | m_eq;
    while (cand != 0u) {
      const int j = __builtin_ctz(cand);
      cand &= cand - 1u;
      const bool is_eq = (m_eq >> j) & 1u;
      if (!is_eq || eq < (uint32_t)r) {
        const uint32_t pos = lt + min(eq, (uint32_t)r);
        // pos < kk always holds for consistent histograms; the checks keep a
        // corrupted workspace from turning into an out-of-bounds store.
        if (pos < (uint32_t)kk) {
          if (idx_row != nullptr) idx_row[pos] = t + j;
          // the gather list holds token positions, or pool rows for a paged cache
          if (ATTN && pos - seg_pos0 < (uint32_t)kMaxK)
            s_sel[pos - seg_pos0] = PAGED ? (int32_t)(page_row0 + j) : t + j;
        }
      }
      lt += is_eq ? 0u : 1u;
      eq += is_eq ? 1u : 0u;
    }
    run_lt += total & 0xffffu;
    run_eq += total >> 16;
  }
  if (seg == 0 && idx_row != nullptr)
    for (int i = kk + tid; i < p.k; i += THREADS) idx_row[i] = -1;

  if constexpr (ATTN) {
    const int n_sel = min((int)(run_lt + min(run_eq, (uint32_t)r) - seg_pos0), kk);
    __syncthreads();  // s_sel complete
    trace.stamp(kSelCompacted);
    const int kvh = hq / (p.Hq / p.Hkv);
    const int64_t row0 = ((int64_t)kvh * p.pool_tokens + (PAGED ? 0 : p.seq_start[b])) * D;
    float M, lsum, o;
    attention_rows<THREADS, D>(s_sel, n_sel, PAGED ? (int)p.pool_tokens : L, p.q + head * D,
                            p.K + row0, p.V + row0, p.scale_log2e, s_attn, M, lsum, o, trace);
    trace.stamp(kSelCombined);
    if (gridDim.x == 1 || (p.arrivals != nullptr && n_active == 1)) {
      if (tid < D) p.out[head * D + tid] = lsum > 0.f ? o / lsum : 0.f;
      trace.stamp(kSelEnd);
      trace.flush(p.trace, p.trace_records);
      return;
    }
    float* mine = p.partial + (head * kMaxParts + seg) * kPartial;
    if (p.arrivals == nullptr) {
      if (tid < D) {
        if (tid == 0) {
          mine[0] = M;
          mine[1] = lsum;
        }
        mine[4 + tid] = o;
      }
      trace.stamp(kSelEnd);
      trace.flush(p.trace, p.trace_records);
      return;
    }
    // Merge by the last segment to finish.  Everything exchanged between
    // workgroups goes through device-scope atomic accesses, which are coherent
    // by themselves: no cache write-back or invalidate is needed, only that a
    // workgroup's stores have been acknowledged before it counts itself, and
    // that the merging workgroup loads after its fetch-add has returned.  The
    // arithmetic and its order are merge_kernel's: both give the same bits.
    if (tid < D) {
      if (tid == 0) {
        __hip_atomic_store(mine + 0, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + 1, lsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __hip_atomic_store(mine + 4 + tid, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);  // this wave's stores are acknowledged
    __syncthreads();
    trace.stamp(kSelPartialAcked);
    if (tid == 0) {
      const uint32_t before = __hip_atomic_fetch_add(p.arrivals + head * p.arrivals_stride, 1u,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_T = before + 1u == (uint32_t)n_active ? 1 : 0;
    }
    __syncthreads();
    trace.stamp(kSelCounted);
    if (s_T == 0) {
      trace.stamp(kSelEnd);
      trace.flush(p.trace, p.trace_records);
      return;
    }
    if (tid >= D) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const float* ph = p.partial + head * kMaxParts * kPartial;
    float pm[kMaxParts], pl[kMaxParts], po[kMaxParts];
#pragma unroll
    for (int s = 0; s < kMaxParts; ++s) {
      const float* ps = ph + (int64_t)min(s, n_active - 1) * kPartial;
      pm[s] = __hip_atomic_load(ps + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      pl[s] = __hip_atomic_load(ps + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      po[s] = __hip_atomic_load(ps + 4 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    float Mh = kNegBig;
#pragma unroll
    for (int s = 0; s < kMaxParts; ++s) Mh = fmaxf(Mh, s < n_active ? pm[s] : kNegBig);
    float lh = 0.f, oh = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxParts; ++s) {
      const bool use = s < n_active;
      const float w = use ? exp2f(pm[s] - Mh) : 0.f;
      lh = fmaf(use ? pl[s] : 0.f, w, lh);
      oh = fmaf(use ? po[s] : 0.f, w, oh);
    }
    p.out[head * D + tid] = lh > 0.f ? oh / lh : 0.f;
    trace.stamp(kSelMerged);
    trace.stamp(kSelEnd);
    trace.flush(p.trace, p.trace_records);
  }
}

// ---------------------------------------------------------------- stand-alone attention

constexpr int kAttnThreads = 256;

struct AttnParams {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  const int64_t* seq_start;
  const int32_t* idx;  // [B*Hq][k]
  float* out;
  float* partial;      // [B*Hq][kMaxParts][partial_stride(D)]
  int64_t pool_tokens;
  int32_t Hq, Hkv, k, n_parts, chunk;  // chunk = idx entries per workgroup
  double scale_log2e;
};

// Grid (n_parts, Hq, B): workgroup `part` attends over idx entries
// [part*chunk, (part+1)*chunk) of its head.  n_parts == 1 writes out directly.
template <int D>
__global__ __launch_bounds__(kAttnThreads) void sparse_attn_kernel(const AttnParams p) {
  constexpr int kPartial = partial_stride(D);
  __shared__ int32_t s_sel[kMaxK];
  __shared__ uint32_t s_scan[kAttnThreads / kWave];
  __shared__ AttnShared<kAttnThreads, D> s_attn;
  const int part = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const int i0 = part * p.chunk, i1 = min(p.k, i0 + p.chunk);
  const int32_t* idx_row = p.idx + head * p.k;
  const int64_t start = p.seq_start[b];
  // Order-preserving compaction of the usable entries of this chunk: negative
  // entries are padding; an entry that would leave the pool is dropped too.
  uint32_t n = 0;
  for (int base = i0; base < i1; base += kAttnThreads) {
    const int i = base + tid;
    const int32_t tok = i < i1 ? idx_row[i] : -1;
    const bool use = tok >= 0 && start >= 0 && start + tok < p.pool_tokens;
    uint32_t total;
    const uint32_t ex = block_excl_scan<kAttnThreads>(use ? 1u : 0u, s_scan, total);
    if (use) s_sel[n + ex] = tok;
    n += total;
  }
  __syncthreads();
  const int kvh = hq / (p.Hq / p.Hkv);
  const int64_t row0 = ((int64_t)kvh * p.pool_tokens + start) * D;
  float M, lsum, o;
  PhaseTrace trace;  // not recorded for the stand-alone kernel
  attention_rows<kAttnThreads, D>(s_sel, (int)n, (int)min((int64_t)0x7fffffff, p.pool_tokens - start),
                               p.q + head * D, p.K + row0, p.V + row0,
                               p.scale_log2e, s_attn, M, lsum, o, trace);
  if (tid < D) {
    if (gridDim.x == 1) {
      p.out[head * D + tid] = lsum > 0.f ? o / lsum : 0.f;
    } else {
      float* mine = p.partial + (head * kMaxParts + part) * kPartial;
      if (tid == 0) {
        mine[0] = M;
        mine[1] = lsum;
      }
      mine[4 + tid] = o;
    }
  }
}

// Merges the attention partials of one head, in part order, into out.
// seg_len > 0: the number of partials is the number of segments that hold
// tokens of the head's sequence (as select_kernel wrote them); seg_len == 0:
// n_parts partials (as sparse_attn_kernel wrote them).
struct MergeParams {
  const float* partial;      // [B*Hq][kMaxParts][partial_stride(D)]
  float* out;                // [B*Hq][128]
  const int64_t* seq_start;
  const int32_t* seq_len;
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, n_parts, seg_len;
};

template <int D>
__global__ __launch_bounds__(D) void merge_kernel(const MergeParams p) {
  constexpr int kPartial = partial_stride(D);
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const float* ph = p.partial + head * kMaxParts * kPartial;
  // All kMaxParts slots exist in the workspace whatever n_parts is: load them
  // unconditionally (no branches, so every load is in flight at once) and mask
  // the unused ones afterwards.
  float pm[kMaxParts], pl[kMaxParts], po[kMaxParts];
#pragma unroll
  for (int s = 0; s < kMaxParts; ++s) {
    const float* ps = ph + (int64_t)s * kPartial;
    pm[s] = ps[0];
    pl[s] = ps[1];
    po[s] = ps[4 + tid];
  }
  int n = p.n_parts;
  if (p.seg_len > 0) {
    const int L = safe_seq_len(p.seq_len, p.seq_start, b, p.max_seq_len, p.pool_tokens);
    n = max(1, (L + p.seg_len - 1) / p.seg_len);
  }
  float M = kNegBig;
  n = min(n, min(p.n_parts, kMaxParts));
#pragma unroll
  for (int s = 0; s < kMaxParts; ++s) M = fmaxf(M, s < n ? pm[s] : kNegBig);
  float lsum = 0.f, o = 0.f;
#pragma unroll
  for (int s = 0; s < kMaxParts; ++s) {
    const bool use = s < n;  // slots past n hold whatever the workspace held
    const float w = use ? exp2f(pm[s] - M) : 0.f;
    lsum = fmaf(use ? pl[s] : 0.f, w, lsum);
    o = fmaf(use ? po[s] : 0.f, w, o);
  }
  p.out[head * D + tid] = lsum > 0.f ? o / lsum : 0.f;
}

}  // namespace adamas
