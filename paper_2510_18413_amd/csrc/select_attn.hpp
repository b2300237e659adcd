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
  const void* dist;           // [B*Hq][dist_stride] bytes or uint16 (Dist<>::kDistBytes)
  const uint64_t* dist_high;  // ninth bits, [B*Hq][dist_stride / 64] (Dist<>::kHighPlane only)
  int64_t dist_stride;        // tokens per row, a multiple of 128
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

// Candidate masks of one 32-bit word of the distance plane against the threshold
// distance T: bit (8 or 16) * j + (7 or 15) of lt / eq is set when token j of the
// word has distance < T / == T.  Byte planes hold four tokens per word, their
// ninth bits come separately (high4: bit j = ninth bit of token j).
template <bool BYTES>
__device__ __forceinline__ void word_masks(uint32_t w, uint32_t high4, int T, uint32_t& lt, uint32_t& eq) {
  if constexpr (BYTES) {
    constexpr uint32_t H = 0x80808080u, L7 = 0x7f7f7f7fu;
    const uint32_t y = (uint32_t)(T & 255) * 0x01010101u;
    // per byte, no borrow between bytes: bit 7 of t = (low 7 bits of w >= low 7 bits of y)
    const uint32_t t = (w | H) - (y & L7);
    const uint32_t lt8 = ((~w & y) | (~(w ^ y) & ~t)) & H;       // unsigned byte compare
    const uint32_t z = w ^ y;
    const uint32_t eq8 = ~(((z & L7) + L7) | z) & H;             // byte of z is zero
    // ninth bits spread to bit 7 of their bytes
    const uint32_t e = (high4 * 0x10204080u) & H;
    if (T < 256) {
      lt = lt8 & ~e;
      eq = eq8 & ~e;
    } else {
      lt = (~e & H) | lt8;
      eq = eq8 & e;
    }
  } else {
    // two uint16 per word, both operands below 2^15
    const uint32_t TT = (uint32_t)T * 0x00010001u;
    lt = pk_sub_u16(w, TT) & 0x80008000u;
    const uint32_t z = w ^ TT;
    eq = pk_sub_u16(z, 0x00010001u) & ~z & 0x80008000u;
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
  using Fmt = Dist<METRIC, D>;
  constexpr int kNumBins = Fmt::kBins, kHistStride = Fmt::kStride;
  constexpr bool BYTES = Fmt::kByteDist, HIGH = Fmt::kHighPlane;
  constexpr int kPartial = partial_stride(D);
  constexpr int kHistPairs = kHistStride / 2;                      // pairs of uint16 bins per stored row
  constexpr int PP = (kHistPairs + THREADS - 1) / THREADS;         // consecutive pairs owned by one thread
  constexpr int NW = THREADS / kWave;
  constexpr int PASS = THREADS * kSelTokPerThread;                 // tokens per pass
  constexpr int DW = BYTES ? 4 : 8;                                // 32-bit words of 16 distances
  constexpr int TPW = 16 / DW;                                     // tokens per word
  __shared__ uint32_t s_wtot[2][NW], s_wpre[NW];
  __shared__ int32_t s_T, s_cntlt;
  __shared__ uint32_t s_ltb, s_eqb;
  __shared__ int32_t s_sel[ATTN ? kMaxK : 1];
  __shared__ AttnShared<ATTN ? THREADS : D / 8, D> s_attn;

  PhaseTrace trace;
  trace.stamp(kSelStart);
  const int seg = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const int seg_t0 = seg * p.seg_len;

  // Nothing below depends on the sequence length until the loads are issued:
  // the workspace rows exist up to dist_stride / n_tiles whatever L is, and
  // what lies beyond L is masked once L has arrived.
  const uint8_t* drow = static_cast<const uint8_t*>(p.dist) + head * p.dist_stride * Fmt::kDistBytes;
  const uint16_t* hrow_high = reinterpret_cast<const uint16_t*>(p.dist_high) + head * (p.dist_stride >> 4);
  // distances (and ninth bits) of this thread for the current pass and the next one (rolling prefetch)
  uint32_t cur[DW], nxt[DW], cur_high = 0, nxt_high = 0;
  {
    const int o0 = tid * kSelTokPerThread, o1 = PASS + tid * kSelTokPerThread;
#pragma unroll
    for (int w = 0; w < DW; ++w) cur[w] = nxt[w] = 0;
    if (o0 < p.seg_len && seg_t0 + o0 < p.dist_stride) {
#pragma unroll
      for (int c = 0; c < DW / 4; ++c) load_piece<16>(drow + (int64_t)(seg_t0 + o0) * Fmt::kDistBytes + 16 * c, &cur[4 * c]);
      if constexpr (HIGH) cur_high = hrow_high[(seg_t0 + o0) >> 4];
    }
    if (o1 < p.seg_len && seg_t0 + o1 < p.dist_stride) {
#pragma unroll
      for (int c = 0; c < DW / 4; ++c) load_piece<16>(drow + (int64_t)(seg_t0 + o1) * Fmt::kDistBytes + 16 * c, &nxt[4 * c]);
      if constexpr (HIGH) nxt_high = hrow_high[(seg_t0 + o1) >> 4];
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
  // Tile histograms: a thread owns PP consecutive pairs of bins (one 32-bit load
  // per pair and tile); pairs past the row repeat its last pair and count as zero.
  const uint16_t* hrow = p.tilehist + head * p.n_tiles * kHistStride;
  const int first_tile = seg_t0 / p.tile_tokens;
  int pair[PP];
#pragma unroll
  for (int j = 0; j < PP; ++j) pair[j] = min(tid * PP + j, kHistPairs - 1);
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

  // Head histogram (all tiles with tokens) and the part of it before this
  // segment, two 16-bit bins per word.  A bin of the head total stays below
  // 2^16 for sequences of up to 65535 tokens, so that the packed words can be
  // added as they are; longer sequences add the halves separately.
  uint32_t tot0[PP], tot1[PP], pre0[PP], pre1[PP];
#pragma unroll
  for (int j = 0; j < PP; ++j) tot0[j] = tot1[j] = pre0[j] = pre1[j] = 0;
  const bool packed_sums = p.max_seq_len < 65536;
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
    if (packed_sums) {
#pragma unroll
      for (int u = 0; u < kHistBatch; ++u) {
#pragma unroll
        for (int j = 0; j < PP; ++j) {
          tot0[j] += tb + u < tiles_active ? hv[j][u] : 0u;
          pre0[j] += tb + u < first_tile ? hv[j][u] : 0u;   // first_tile <= tiles_active here
        }
      }
    } else {
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
  }
  uint32_t sum_tot = 0, sum_pre = 0;
#pragma unroll
  for (int j = 0; j < PP; ++j) {
    if (packed_sums) {
      tot1[j] = tot0[j] >> 16;
      tot0[j] &= 0xffffu;
      pre1[j] = pre0[j] >> 16;
      pre0[j] &= 0xffffu;
    }
    // bins past the last one were never written (and pairs past the row repeat its last pair)
    if (2 * (tid * PP + j) >= kNumBins) tot0[j] = pre0[j] = 0u;
    if (2 * (tid * PP + j) + 1 >= kNumBins) tot1[j] = pre1[j] = 0u;
    sum_tot += tot0[j] + tot1[j];
    sum_pre += pre0[j] + pre1[j];
  }
  // Threshold distance T = the bin in which the cumulative count reaches kk,
  // #{D < T} over the head, and (for the output offset of this segment) #{D < T}
  // and #{D == T} over the tokens of earlier segments: two prefix sums over the
  // bins in thread order, then the one thread whose bins contain the kk-th token
  // publishes all four.
  const uint32_t incl_tot = wave_incl_scan_u32(sum_tot), incl_pre = wave_incl_scan_u32(sum_pre);
  if (lane == 63) {
    s_wtot[0][wave] = incl_tot;
    s_wpre[wave] = incl_pre;
  }
  if (tid == 0) {
    s_ltb = 0u;
    s_eqb = 0u;
    s_T = 0;
    s_cntlt = 0;
  }
  __syncthreads();
  {
    uint32_t run = incl_tot - sum_tot, run_pre = incl_pre - sum_pre;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      run += w < wave ? s_wtot[0][w] : 0u;
      run_pre += w < wave ? s_wpre[w] : 0u;
    }
    if (kk > 0 && run < (uint32_t)kk && run + sum_tot >= (uint32_t)kk) {
#pragma unroll
      for (int j = 0; j < PP; ++j) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const uint32_t c = h ? tot1[j] : tot0[j], cp = h ? pre1[j] : pre0[j];
          if (run < (uint32_t)kk && run + c >= (uint32_t)kk) {
            s_T = 2 * (tid * PP + j) + h;
            s_cntlt = (int32_t)run;
            s_ltb = run_pre;
            s_eqb = cp;
          }
          run += c;
          run_pre += cp;
        }
      }
    }
  }
  __syncthreads();
  const int T = s_T;
  const int r = kk - s_cntlt;  // ties at distance T to take, lowest positions first
  uint32_t run_lt = s_ltb, run_eq = s_eqb;
  trace.stamp(kSelThreshold);
  const uint32_t seg_pos0 = run_lt + min(run_eq, (uint32_t)r);
  int32_t* idx_row = p.idx_out != nullptr ? p.idx_out + head * p.k : nullptr;

  int pass_no = 0;
  for (int pass_t0 = seg_t0; pass_t0 < seg_t1; pass_t0 += PASS, ++pass_no) {
    const int t = pass_t0 + tid * kSelTokPerThread;
    uint32_t dw[DW];
#pragma unroll
    for (int w = 0; w < DW; ++w) {
      dw[w] = cur[w];
      cur[w] = nxt[w];
    }
    const uint32_t high = cur_high;
    cur_high = nxt_high;
    if (t + 2 * PASS < seg_t1) {  // fetch the pass after next while this one is processed
#pragma unroll
      for (int c = 0; c < DW / 4; ++c)
        load_piece<16>(drow + (int64_t)(t + 2 * PASS) * Fmt::kDistBytes + 16 * c, &nxt[4 * c]);
      if constexpr (HIGH) nxt_high = hrow_high[(t + 2 * PASS) >> 4];
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
    // Per word: which of its tokens lie below / at the threshold (word_masks),
    // restricted to the tokens of this thread that exist.
    const int n_valid = min(max(seg_t1 - t, 0), kSelTokPerThread);
    uint32_t m_lt[DW], m_eq[DW], n_lt = 0, n_eq = 0;
#pragma unroll
    for (int w = 0; w < DW; ++w) {
      word_masks<BYTES>(dw[w], HIGH ? (high >> (4 * w)) & 0xfu : 0u, T, m_lt[w], m_eq[w]);
      // tokens TPW * w .. of the thread: keep the first n_valid - TPW * w of the word
      const int keep = min(max(n_valid - TPW * w, 0), TPW);
      const uint32_t vm = keep == TPW ? 0xffffffffu : (1u << ((32 / TPW) * keep)) - 1u;
      m_lt[w] &= vm;
      m_eq[w] &= vm;
      n_lt += (uint32_t)__popc(m_lt[w]);
      n_eq += (uint32_t)__popc(m_eq[w]);
    }
    // exclusive prefix over the workgroup (one barrier per pass: the wave totals alternate buffers)
    const uint32_t cnt = n_lt | (n_eq << 16);
    const uint32_t incl = wave_incl_scan_u32(cnt);
    uint32_t* wt = s_wtot[pass_no & 1];
    if (lane == 63) wt[wave] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const uint32_t x = wt[w];
      before += w < wave ? x : 0u;
      total += x;
    }
    const uint32_t ex = before + incl - cnt;
    uint32_t lt = run_lt + (ex & 0xffffu), eq = run_eq + (ex >> 16);
    // Visit only the candidate tokens (set bits), in position order.
#pragma unroll
    for (int w = 0; w < DW; ++w) {
      uint32_t cand = m_lt[w] | m_eq[w];
      while (cand != 0u) {
        const int bit = __builtin_ctz(cand);
        cand &= cand - 1u;
        const bool is_eq = (m_eq[w] >> bit) & 1u;
        const int j = TPW * w + bit / (32 / TPW);
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
