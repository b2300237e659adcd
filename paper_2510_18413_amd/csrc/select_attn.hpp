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

#include <type_traits>

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
  const uint32_t* tilehist;   // [B*Hq][n_tiles][Dist<>::kPairs] words of two 16-bit bins
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
  uint32_t group_magic;       // see kv_head_of
  int32_t n_tiles, tile_tokens, seg_len;  // tile_tokens and seg_len are powers of two
  int32_t tile_shift, seg_shift;          // their logarithms
  // Request the K / V lines of each thread's first selected token ahead of the
  // gather (see the kernel).  Pays when the kernel is bound by its chain of
  // memory round trips (few workgroups, few passes each); costs when it is bound
  // by throughput: the requests are one line per lane and double the gather's
  // traffic between the caches.
  int32_t early_rows;
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
  kSelMasked,         // (first pass) candidate masks and counts of the thread's 16 tokens
  kSelPrefix,         // (first pass) candidates before this thread known (past the pass's barrier)
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
  static constexpr int kWaves = THREADS / kWave;  // one combined state per wave
  float m[kWaves];
  float l[kWaves];
  float acc[kWaves][D];
};

// One step of combining the online-softmax states (m, l, acc[8]) of the lane
// groups of a wave: afterwards lanes i and i ^ STEP hold the combination of
// their two states (the same bits in both: each side is weighted and the two
// products are added, which commutes).  STEP 16 and 32 exchange with the
// swap instructions of the vector ALU (a: the state of the lane whose STEP bit
// is clear, b: of the lane whose bit is set, both in every lane), STEP 8 with
// a rotation inside the row of 16 lanes.
template <int STEP>
__device__ __forceinline__ void exchange_pair(float v, float& a, float& b) {
  static_assert(STEP == 8 || STEP == 16 || STEP == 32, "lane groups of 8, 16 or 32");
  const uint32_t u = __float_as_uint(v);
  if constexpr (STEP == 32) {
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
  } else if constexpr (STEP == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
  } else {
    const float o = __int_as_float(__builtin_amdgcn_update_dpp(0, (int)u, 0x128 /* row_ror:8 */, 0xf, 0xf, false));
    const bool upper = (threadIdx.x & 8) != 0;
    a = upper ? o : v;
    b = upper ? v : o;
  }
}
template <int STEP>
__device__ __forceinline__ void combine_lane_groups(float& m, float& l, float (&acc)[8]) {
#pragma clang fp contract(off)
  float ma, mb, la, lb;
  exchange_pair<STEP>(m, ma, mb);
  exchange_pair<STEP>(l, la, lb);
  const float mn = fmaxf(ma, mb);
  const float wa = exp2_neg(ma - mn), wb = exp2_neg(mb - mn);
  m = mn;
  l = la * wa + lb * wb;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float xa, xb;
    exchange_pair<STEP>(acc[j], xa, xb);
    acc[j] = xa * wa + xb * wb;
  }
}

// Softmax attention (Eq. 1) of one query over the n rows listed in s_sel (token
// positions; Kp, Vp point at the sequence's first row of the right KV head),
// by the whole workgroup: D / 8 lanes per row, 8 dims per lane, one-pass online
// softmax per lane group in fp32 (exp2 domain); the groups of a wave are then
// combined with cross-lane moves and the waves, in fixed order, through LDS.
// Threads 0..D-1 receive, for output dim tid: M (running maximum), lsum (sum of
// weights) and o (unnormalised weighted sum of V).
// Entries of s_sel are clamped to [0, n_tokens) before use (n_tokens >= 1 when n > 0).
// qv is the lane's piece of the query, from load_query_piece: the caller
// requests it as early as it can, so that it does not arrive after the rows.
// All threads must call it.
template <int D>
__device__ __forceinline__ uint4 load_query_piece(const uint16_t* __restrict__ q) {
  constexpr int LPR = HeadDim<D>::kRowGroup;
  const int gl = threadIdx.x % LPR;
  return gl < HeadDim<D>::kRowLanes ? *reinterpret_cast<const uint4*>(q + gl * 8) : make_uint4(0, 0, 0, 0);
}

template <int THREADS, int D>
__device__ __forceinline__ void attention_rows(const int32_t* s_sel, int n, int n_tokens, const uint4 qv,
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
  // A row takes D / 8 lanes of 8 dims inside an aligned group of LPR lanes (the
  // next power of two: the same for the paper's head dimensions; with D = 96,
  // 160 or 192 the last lanes of a group hold zeros and load nothing).
  constexpr int LPR = HeadDim<D>::kRowGroup, kRowLanes = HeadDim<D>::kRowLanes;
  constexpr int kGroups = THREADS / LPR;
  constexpr int NW = THREADS / kWave;
  const int tid = threadIdx.x, grp = tid / LPR, gl = tid % LPR;
  const int wave = tid >> 6, lane = tid & 63;
  const bool lane_on = gl < kRowLanes;

  double qf[8];
  {
    qf[0] = bf16_lo(qv.x); qf[1] = bf16_hi(qv.x); qf[2] = bf16_lo(qv.y); qf[3] = bf16_hi(qv.y);
    qf[4] = bf16_lo(qv.z); qf[5] = bf16_hi(qv.z); qf[6] = bf16_lo(qv.w); qf[7] = bf16_hi(qv.w);
  }
  float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;

  constexpr int U = 4;  // rows in flight per lane group
  for (int i0 = grp; i0 < n; i0 += kGroups * U) {
    uint4 kv[U], vv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * kGroups;
      ok[u] = i < n;
      kv[u] = make_uint4(0, 0, 0, 0);
      vv[u] = make_uint4(0, 0, 0, 0);
      if (ok[u] && lane_on) {
        // clamped: whatever the list holds, the gather stays inside the sequence
        const int tok = min(max(s_sel[i], 0), n_tokens - 1);
        const int64_t off = (int64_t)tok * D + gl * 8;
        kv[u] = *reinterpret_cast<const uint4*>(Kp + off);
        vv[u] = *reinterpret_cast<const uint4*>(Vp + off);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // Row slots are filled in order, so a slot that no group of this wave uses
      // ends the batch (a wave-uniform test: the rows of a small selection take
      // one or two slots, and the unused ones cost nothing).
      if (__ballot(ok[u]) == 0) break;
      if (u == 0 && i0 == grp) trace.stamp(kSelRowsFirst);
      // two chains of four: the additions of a chain wait for each other
      double s1 = qf[0] * (double)bf16_lo(kv[u].x), s2 = qf[1] * (double)bf16_hi(kv[u].x);
      s1 = fma(qf[2], (double)bf16_lo(kv[u].y), s1);
      s2 = fma(qf[3], (double)bf16_hi(kv[u].y), s2);
      s1 = fma(qf[4], (double)bf16_lo(kv[u].z), s1);
      s2 = fma(qf[5], (double)bf16_hi(kv[u].z), s2);
      s1 = fma(qf[6], (double)bf16_lo(kv[u].w), s1);
      s2 = fma(qf[7], (double)bf16_hi(kv[u].w), s2);
      // summed over the row's aligned group of 8, 16 or 32 lanes
      const double sc = ok[u] ? lanes_sum_f64<LPR>(s1 + s2) * scale_log2e : (double)kNegBig;
      const float mn = fmaxf(m, (float)sc);
      const float corr = exp2_neg(m - mn);
      const float pw = ok[u] ? exp2_neg((float)(sc - (double)mn)) : 0.f;
      m = mn;
      l = l * corr + pw;
      acc[0] = fmaf(pw, bf16_lo(vv[u].x), acc[0] * corr);
      acc[1] = fmaf(pw, bf16_hi(vv[u].x), acc[1] * corr);
      acc[2] = fmaf(pw, bf16_lo(vv[u].y), acc[2] * corr);
      acc[3] = fmaf(pw, bf16_hi(vv[u].y), acc[3] * corr);
      acc[4] = fmaf(pw, bf16_lo(vv[u].z), acc[4] * corr);
      acc[5] = fmaf(pw, bf16_hi(vv[u].z), acc[5] * corr);
      acc[6] = fmaf(pw, bf16_lo(vv[u].w), acc[6] * corr);
      acc[7] = fmaf(pw, bf16_hi(vv[u].w), acc[7] * corr);
    }
  }
  trace.stamp(kSelAttended);

  // The lane groups of a wave hold the same dims in the same lanes of their
  // group: combine them pairwise with cross-lane moves (both partners compute
  // the same values), then the waves through LDS.  A group without rows has
  // l = 0 and m = kNegBig and drops out with weight exp2(kNegBig - M) = 0.
  if constexpr (LPR <= 8) combine_lane_groups<8>(m, l, acc);
  if constexpr (LPR <= 16) combine_lane_groups<16>(m, l, acc);
  combine_lane_groups<32>(m, l, acc);
  if (lane < kRowLanes) {
    if (lane == 0) {
      sh.m[wave] = m;
      sh.l[wave] = l;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) sh.acc[wave][lane * 8 + j] = acc[j];
  }
  __syncthreads();

  M = kNegBig;
  lsum = 0.f;
  o = 0.f;
  if (tid < D) {
#pragma unroll
    for (int w = 0; w < NW; ++w) M = fmaxf(M, sh.m[w]);
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float wt = exp2_neg(sh.m[w] - M);
      lsum = fmaf(sh.l[w], wt, lsum);
      o = fmaf(sh.acc[w][tid], wt, o);
    }
  }
}

// Candidate masks of one 32-bit word of the distance plane against the threshold
// distance T: bit (8 or 16) * j + (7 or 15) of lt / eq is set when token j of the
// word has distance < T / == T.  Byte planes hold four tokens per word and carry
// the low eight bits of the distance; y = (T & 255) * 0x01010101.
template <bool BYTES>
__device__ __forceinline__ void word_masks(uint32_t w, uint32_t y, uint32_t& lt, uint32_t& eq) {
  if constexpr (BYTES) {
    constexpr uint32_t H = 0x80808080u, L7 = 0x7f7f7f7fu;
    // per byte, no borrow between bytes: bit 7 of t = (low 7 bits of w >= low 7 bits of y)
    const uint32_t t = (w | H) - (y & L7);
    lt = ((~w & y) | (~(w ^ y) & ~t)) & H;       // unsigned byte compare
    const uint32_t z = w ^ y;
    eq = ~(((z & L7) + L7) | z) & H;             // byte of z is zero
  } else {
    // two uint16 per word, both operands below 2^15; y = T * 0x00010001
    lt = pk_sub_u16(w, y) & 0x80008000u;
    const uint32_t z = w ^ y;
    eq = pk_sub_u16(z, 0x00010001u) & ~z & 0x80008000u;
  }
}

// Byte planes: the flags of four words (bit 7 of byte b of word w = token 4 w + b)
// gathered into 16 bits, bit j = token j.  A dot product of the flag bytes
// (0x80 or 0) with the weights 1, 2, 4, 8 (and 16 .. 128 for the next word)
// leaves 128 times the eight flags.
__device__ __forceinline__ uint32_t flags16(const uint32_t (&m)[4]) {
  uint32_t lo = __builtin_amdgcn_udot4(m[0], 0x08040201u, 0u, false);
  lo = __builtin_amdgcn_udot4(m[1], 0x80402010u, lo, false);
  uint32_t hi = __builtin_amdgcn_udot4(m[2], 0x08040201u, 0u, false);
  hi = __builtin_amdgcn_udot4(m[3], 0x80402010u, hi, false);
  return (lo | (hi << 8)) >> 7;
}
__device__ __forceinline__ uint32_t flags16(const uint32_t (&)[8]) { return 0u; }  // uint16 planes: not used

// The last step of the in-kernel merge: slots 0..n_active-1 (n_active <= N) of a
// head's partials, read with device-scope loads, combined in slot order with
// merge_kernel's arithmetic.
template <int N, int D>
__device__ __forceinline__ float merge_slots(const float* ph, int n_active, int tid) {
  constexpr int kPartial = partial_stride(D);
  float pm[N], pl[N], po[N];
#pragma unroll
  for (int s = 0; s < N; ++s) {
    const float* ps = ph + (int64_t)min(s, n_active - 1) * kPartial;
    pm[s] = __hip_atomic_load(ps + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    pl[s] = __hip_atomic_load(ps + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    po[s] = __hip_atomic_load(ps + 4 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  float Mh = kNegBig;
#pragma unroll
  for (int s = 0; s < N; ++s) Mh = fmaxf(Mh, s < n_active ? pm[s] : kNegBig);
  float lh = 0.f, oh = 0.f;
#pragma unroll
  for (int s = 0; s < N; ++s) {
    const bool use = s < n_active;
    const float w = use ? exp2_neg(pm[s] - Mh) : 0.f;
    lh = fmaf(use ? pl[s] : 0.f, w, lh);
    oh = fmaf(use ? po[s] : 0.f, w, oh);
  }
  return lh > 0.f ? oh / lh : 0.f;
}

// Grid (n_segs, Hq, B).  With ATTN a head that has a single segment with
// tokens is finished by that workgroup; otherwise each workgroup leaves an
// (M, lsum, o[128]) partial, merged by the last one to arrive (p.arrivals set)
// or by merge_kernel (p.arrivals null).
//
// A workgroup is one wave per SIMD and runs alone on its compute unit, so its
// time is the number of instructions a wave issues (about 2 ns each) plus the
// memory round trips: the code below is written to issue few.
template <int THREADS, bool ATTN, int METRIC, bool PAGED, int D, int CHUNK>
__global__ __launch_bounds__(THREADS) void select_kernel(const SelectParams p) {
  static_assert(CHUNK == 1 || CHUNK == 8, "passes per workgroup barrier");
  static_assert(ATTN || !PAGED, "only the gather needs the page table");
  static_assert(THREADS >= D, "one thread per output dimension in the merge");
  using Fmt = Dist<METRIC, D>;
  constexpr int kNumBins = Fmt::kBins;
  constexpr bool BYTES = Fmt::kByteDist, HIGH = Fmt::kHighPlane;
  static_assert(!BYTES || HIGH || Fmt::kMaxDist < 255, "0xff marks a token that does not exist");
  static_assert(!HIGH || Fmt::kMaxDist < 511, "0x1ff marks a token that does not exist");
  constexpr int kPartial = partial_stride(D);
  constexpr int kHistPairs = Fmt::kPairs;                          // words (pairs of bins) of a histogram
  constexpr int PP = (kHistPairs + THREADS - 1) / THREADS;         // consecutive pairs owned by one thread
  constexpr int NW = THREADS / kWave;
  constexpr int PASS = THREADS * kSelTokPerThread;                 // tokens per pass
  constexpr int DW = BYTES ? 4 : 8;                                // 32-bit words of 16 distances
  constexpr int TPW = 16 / DW;                                     // tokens per word
  constexpr int TB = 32 / TPW;                                     // bits per token in a word
  __shared__ __align__(16) uint32_t s_wave[1][NW][2];   // per-wave prefix totals of the threshold search
  __shared__ uint32_t s_pass[BYTES ? CHUNK : 1][NW];    // per-wave totals of the passes of a chunk
  __shared__ __align__(16) int32_t s_found[4];          // T, #{D<T}, and #{D<T}, #{D==T} before the segment
  __shared__ int32_t s_last;
  __shared__ int32_t s_sel[ATTN ? kMaxK : 1];
  __shared__ AttnShared<ATTN ? THREADS : kWave, D> s_attn;

  PhaseTrace trace;
  trace.stamp(kSelStart);
  // first of all, ahead of everything else the compiler may want to load
  SeqInfo seq = SeqInfo::request<PAGED, false>(p.seq_len, p.seq_start, (int)blockIdx.z);
  __builtin_amdgcn_sched_barrier(0);
  const int seg = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const int seg_t0 = seg * p.seg_len;
  uint4 qv = make_uint4(0, 0, 0, 0);  // this lane's piece of the query, for the attention at the end
  if constexpr (ATTN) qv = load_query_piece<D>(p.q + head * D);

  // Nothing below depends on the sequence length until the loads are issued:
  // the workspace rows exist up to dist_stride / n_tiles (+ kHistBatch rows of
  // slack behind the last histogram) whatever L is, and what lies beyond L is
  // masked once L has arrived.
  const uint8_t* drow = static_cast<const uint8_t*>(p.dist) +
                        (head * p.dist_stride + seg_t0 + tid * kSelTokPerThread) * Fmt::kDistBytes;
  const uint16_t* hrow_high = reinterpret_cast<const uint16_t*>(p.dist_high) +
                              ((head * p.dist_stride + seg_t0) >> 4) + tid;
  // distances (and ninth bits) of this thread for the current pass and the next one (rolling prefetch)
  uint32_t cur[DW], nxt[DW], cur_high = 0, nxt_high = 0;
#pragma unroll
  for (int w = 0; w < DW; ++w) cur[w] = nxt[w] = 0;
  // (the last segment may reach past the row of the plane: nothing is read there)
  if (tid * kSelTokPerThread < p.seg_len && seg_t0 + tid * kSelTokPerThread < p.dist_stride) {
#pragma unroll
    for (int c = 0; c < DW / 4; ++c) load_piece<16>(drow + 16 * c, &cur[4 * c]);
    if constexpr (HIGH) cur_high = hrow_high[0];
  }
  if (PASS + tid * kSelTokPerThread < p.seg_len && seg_t0 + PASS + tid * kSelTokPerThread < p.dist_stride) {
#pragma unroll
    for (int c = 0; c < DW / 4; ++c) load_piece<16>(drow + PASS * Fmt::kDistBytes + 16 * c, &nxt[4 * c]);
    if constexpr (HIGH) nxt_high = hrow_high[PASS >> 4];
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
  // per pair and tile); pairs past the histogram repeat its last pair and count as
  // zero.  Rows past the head's last tile are read as well (they exist: the next
  // head's, or the slack behind the last head) and left out of the sums.
  const uint32_t* hbase = p.tilehist + head * p.n_tiles * kHistPairs;
  int pair_off[PP];
#pragma unroll
  for (int j = 0; j < PP; ++j) pair_off[j] = min(tid * PP + j, kHistPairs - 1);
  uint32_t hv[PP][kHistBatch];
#pragma unroll
  for (int u = 0; u < kHistBatch; ++u) {
#pragma unroll
    for (int j = 0; j < PP; ++j) hv[j][u] = hbase[u * kHistPairs + pair_off[j]];
  }

  loads_issued_before_here();
  seq.make_uniform();
  const int L = PAGED ? seq.paged_length(p.max_seq_len, (int64_t)p.max_pages << p.page_shift)
                      : seq.length(p.max_seq_len, p.pool_tokens);
  const int kk = min(p.k, L);
  // segments and tiles are powers of two: no division
  const int n_active = max(1, (L + p.seg_len - 1) >> p.seg_shift);  // segments that hold tokens
  if (seg >= n_active) return;
  trace.stamp(kSelLoaded);
  const int seg_t1 = min(L, seg_t0 + p.seg_len);
  const int tiles_active = (L + p.tile_tokens - 1) >> p.tile_shift;
  const int first_tile = seg_t0 >> p.tile_shift;  // < tiles_active

  // Head histogram (all tiles with tokens) and the part of it before this
  // segment, two 16-bit bins per word.  A bin of the head total stays below
  // 2^16 for sequences of up to 65535 tokens, so that the packed words can be
  // added as they are; longer sequences add the halves separately.  Which tiles
  // count is wave-uniform; a full batch of tiles needs no masks at all.
  uint32_t tot0[PP], tot1[PP], pre0[PP], pre1[PP];
#pragma unroll
  for (int j = 0; j < PP; ++j) tot0[j] = tot1[j] = pre0[j] = pre1[j] = 0;
  const bool packed_sums = p.max_seq_len < 65536;
  for (int tb = 0; tb < tiles_active; tb += kHistBatch) {
    if (tb > 0) {
#pragma unroll
      for (int u = 0; u < kHistBatch; ++u) {
#pragma unroll
        for (int j = 0; j < PP; ++j) hv[j][u] = hbase[(tb + u) * kHistPairs + pair_off[j]];
      }
    }
    const int n_tot = tiles_active - tb, n_pre = first_tile - tb;  // tiles of this batch that count
    if (packed_sums) {
      if (n_tot >= kHistBatch) {
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) {
#pragma unroll
          for (int j = 0; j < PP; ++j) tot0[j] += hv[j][u];
        }
      } else {
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) {
          const uint32_t on = u < n_tot ? 0xffffffffu : 0u;
#pragma unroll
          for (int j = 0; j < PP; ++j) tot0[j] += hv[j][u] & on;
        }
      }
      if (n_pre >= kHistBatch) {
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) {
#pragma unroll
          for (int j = 0; j < PP; ++j) pre0[j] += hv[j][u];
        }
      } else if (n_pre > 0) {
#pragma unroll
        for (int u = 0; u < kHistBatch; ++u) {
          const uint32_t on = u < n_pre ? 0xffffffffu : 0u;
#pragma unroll
          for (int j = 0; j < PP; ++j) pre0[j] += hv[j][u] & on;
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < kHistBatch; ++u) {
        const uint32_t on = u < n_tot ? 0xffffffffu : 0u, before = u < n_pre ? 0xffffffffu : 0u;
#pragma unroll
        for (int j = 0; j < PP; ++j) {
          const uint32_t v = hv[j][u] & on;
          tot0[j] += v & 0xffffu;
          tot1[j] += v >> 16;
          pre0[j] += v & before & 0xffffu;
          pre1[j] += (v & before) >> 16;
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
    s_wave[0][wave][0] = incl_tot;
    s_wave[0][wave][1] = incl_pre;
  }
  if (tid == 0) {
    s_found[0] = 0;
    s_found[1] = 0;
    s_found[2] = 0;
    s_found[3] = 0;
  }
  __syncthreads();
  {
    uint32_t run = incl_tot - sum_tot, run_pre = incl_pre - sum_pre;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w) {  // the last wave's total is nobody's prefix
      run += w < wave ? s_wave[0][w][0] : 0u;
      run_pre += w < wave ? s_wave[0][w][1] : 0u;
    }
    if (kk > 0 && run < (uint32_t)kk && run + sum_tot >= (uint32_t)kk) {
#pragma unroll
      for (int j = 0; j < PP; ++j) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const uint32_t c = h ? tot1[j] : tot0[j], cp = h ? pre1[j] : pre0[j];
          if (run < (uint32_t)kk && run + c >= (uint32_t)kk) {
            s_found[0] = 2 * (tid * PP + j) + h;
            s_found[1] = (int32_t)run;
            s_found[2] = (int32_t)run_pre;
            s_found[3] = (int32_t)cp;
          }
          run += c;
          run_pre += cp;
        }
      }
    }
  }
  __syncthreads();
  const int4 found = *reinterpret_cast<const int4*>(s_found);
  const int T = found.x;
  const int r = kk - found.y;  // ties at distance T to take, lowest positions first
  uint32_t run_lt = (uint32_t)found.z, run_eq = (uint32_t)found.w;
  trace.stamp(kSelThreshold, false);
  const uint32_t seg_pos0 = run_lt + min(run_eq, (uint32_t)r);
  int32_t* idx_row = p.idx_out != nullptr ? p.idx_out + head * p.k : nullptr;
  // what the low bits of a stored distance are compared with
  const uint32_t y = BYTES ? (uint32_t)(T & 255) * 0x01010101u : (uint32_t)T * 0x00010001u;

  // gather: rows of the sequence's KV head (pool rows for a paged cache)
  constexpr int kRowLines = (D + 63) / 64;  // 128-byte lines that a row of D bf16 values touches
  const int64_t row0 = ((int64_t)kv_head_of(hq, p.group_magic) * p.pool_tokens + seq.start) * D;
  const int64_t gather_rows = PAGED ? p.pool_tokens : (int64_t)L;
  uint32_t early[2 * kRowLines];
#pragma unroll
  for (int i = 0; i < 2 * kRowLines; ++i) early[i] = 0u;

  // The passes of a segment (4096 tokens each, 16 per thread) are taken in chunks of up to kChunk:
  // first the candidate flags and counts of every pass of the chunk (the distances are needed
  // for nothing else), then ONE workgroup barrier for the prefix sums of all of them, then the
  // emission from the stored flags.  (A barrier per pass cost a segment of eight passes about
  // 0.15 us each.)  uint16 planes keep their flags in eight words per pass and take a pass at a time.
  // CHUNK = 1 (a pass at a time) is its own instantiation of the kernel, launched for segments of
  // one or two passes: with both forms in one kernel those lose 0.3-0.8 us.
  auto run_passes = [&](auto chunk_) {
  constexpr int kChunk = decltype(chunk_)::value;
  bool first_chunk = true;
  for (int chunk_t0 = seg_t0; chunk_t0 < seg_t1; chunk_t0 += kChunk * PASS) {
    const int n_pass = min(kChunk, (seg_t1 - chunk_t0 + PASS - 1) / PASS);  // wave-uniform, >= 1
    uint32_t flags[kChunk], cnt[kChunk];   // byte planes: lt flags | eq flags << 16; counts packed alike
    int64_t prow[kChunk];                  // paged cache: pool row of the thread's first token of the pass
    uint32_t m_lt[DW], m_eq[DW];           // uint16 planes (one pass per chunk)
#pragma unroll
    for (int w = 0; w < DW; ++w) m_lt[w] = m_eq[w] = 0u;
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      flags[c] = cnt[c] = 0u;
      prow[c] = 0;
      if (c < n_pass) {
        const int pass_t0 = chunk_t0 + c * PASS;
        const int t = pass_t0 + tid * kSelTokPerThread;
        uint32_t dw[DW];
#pragma unroll
        for (int w = 0; w < DW; ++w) {
          dw[w] = cur[w];
          cur[w] = nxt[w];
        }
        uint32_t high = cur_high;
        cur_high = nxt_high;
        if (t + 2 * PASS < seg_t1) {  // fetch the pass after next while this one is processed
          const uint8_t* src = drow + (int64_t)(pass_t0 - seg_t0 + 2 * PASS) * Fmt::kDistBytes;
#pragma unroll
          for (int q4 = 0; q4 < DW / 4; ++q4) load_piece<16>(src + 16 * q4, &nxt[4 * q4]);
          if constexpr (HIGH) nxt_high = hrow_high[(pass_t0 - seg_t0 + 2 * PASS) >> 4];
        }
        if constexpr (PAGED) {
          // pool row of token t's page, minus the page offset of t itself
          const int64_t pg = min(max((int64_t)cur_pg, (int64_t)0), (p.pool_tokens >> p.page_shift) - 1);
          prow[c] = (pg << p.page_shift) + (t & ((1 << p.page_shift) - 1));
          cur_pg = nxt_pg;
          if (t + 2 * PASS < seg_t1)
            nxt_pg = p.page_table[(int64_t)b * p.max_pages +
                                  min((t + 2 * PASS) >> p.page_shift, p.max_pages - 1)];
        }
        // Tokens of this thread past the end of the segment (only in its last
        // 16-token group) get the largest stored value, which no threshold reaches.
        if (t + kSelTokPerThread > seg_t1) {
          const int n_valid = max(seg_t1 - t, 0);
#pragma unroll
          for (int w = 0; w < DW; ++w) {
            const int keep = min(max(n_valid - TPW * w, 0), TPW);
            const uint32_t gone = keep == TPW ? 0u : ~((1u << (TB * keep)) - 1u);
            // bytes: 0xff (with the ninth bit below: 0x1ff); uint16: exactly 0x7fff, whatever was loaded
            dw[w] = BYTES ? (dw[w] | gone) : ((dw[w] & ~gone) | (gone & 0x7fff7fffu));
          }
          if (HIGH) high |= ~((1u << n_valid) - 1u);
        }
        // Per word: which of its tokens lie below / at the threshold.
        uint32_t n_lt = 0, n_eq = 0;
#pragma unroll
        for (int w = 0; w < DW; ++w) word_masks<BYTES>(dw[w], y, m_lt[w], m_eq[w]);
        if constexpr (BYTES) {
          // the flags of the thread's 16 tokens gathered into 16 bits (bit j = token j)
          uint32_t lt16 = flags16(m_lt), eq16 = flags16(m_eq);
          if constexpr (HIGH) {
            // The bytes were compared on their low eight bits; `high` holds the ninth bits.
            const uint32_t h16 = high & 0xffffu;
            if (T < 256) {
              lt16 &= ~h16;
              eq16 &= ~h16;
            } else {
              lt16 |= ~h16 & 0xffffu;
              eq16 &= h16;
            }
          }
          n_lt = (uint32_t)__popc(lt16);
          n_eq = (uint32_t)__popc(eq16);
          flags[c] = lt16 | (eq16 << 16);
        } else {
#pragma unroll
          for (int w = 0; w < DW; ++w) {
            n_lt += (uint32_t)__popc(m_lt[w]);
            n_eq += (uint32_t)__popc(m_eq[w]);
          }
        }
        cnt[c] = n_lt | (n_eq << 16);
      }
    }
    if (first_chunk) trace.stamp(kSelMasked, false);
    // exclusive prefixes over the workgroup, all passes of the chunk behind one barrier
    uint32_t incl[kChunk];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      incl[c] = 0u;
      if (c < n_pass) {
        incl[c] = wave_incl_scan_u32(cnt[c]);
        if (lane == 63) s_pass[c][wave] = incl[c];
      }
    }
    __syncthreads();
    uint32_t lt0[kChunk], eq0[kChunk];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      lt0[c] = eq0[c] = 0u;
      if (c < n_pass) {
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const uint32_t x = s_pass[c][w];
          before += w < wave ? x : 0u;
          total += x;
        }
        const uint32_t ex = before + incl[c] - cnt[c];
        lt0[c] = run_lt + (ex & 0xffffu);
        eq0[c] = run_eq + (ex >> 16);
        run_lt += total & 0xffffu;
        run_eq += total >> 16;
      }
    }
    if (first_chunk) trace.stamp(kSelPrefix, false);
    if constexpr (ATTN) {
      // The gather below starts only after the compaction; the K and V rows of
      // this thread's first selected token are requested here already (one word
      // per 128-byte line, never used), so that the gather finds them in the
      // cache.  First pass only: the registers are not reused while in flight.
      // The host switches this on for launches that are bound by latency.
      if (first_chunk && p.early_rows != 0) {
        const int t = chunk_t0 + tid * kSelTokPerThread;
        int j = 0;
        bool some = false, first_eq = false;
        if constexpr (BYTES) {
          const uint32_t lt16 = flags[0] & 0xffffu, eq16 = flags[0] >> 16;
          const uint32_t c16 = lt16 | eq16;
          j = __builtin_ctz(c16 | 0x10000u);
          some = c16 != 0u;
          first_eq = (eq16 >> j) & 1u;
        } else {
#pragma unroll
          for (int w = DW - 1; w >= 0; --w) {
            const uint32_t cw = m_lt[w] | m_eq[w];
            if (cw != 0u) {
              const int bit = __builtin_ctz(cw);
              some = true;
              first_eq = (m_eq[w] >> bit) & 1u;
              j = TPW * w + bit / TB;
            }
          }
        }
        if (some && (!first_eq || eq0[0] < (uint32_t)r)) {
          const int64_t row = min(PAGED ? prow[0] + j : (int64_t)(t + j), gather_rows - 1);
          const uint32_t* kr = reinterpret_cast<const uint32_t*>(p.K + row0 + row * D);
          const uint32_t* vr = reinterpret_cast<const uint32_t*>(p.V + row0 + row * D);
#pragma unroll
          for (int c128 = 0; c128 < kRowLines; ++c128) {
            early[2 * c128] = kr[32 * c128];
            early[2 * c128 + 1] = vr[32 * c128];
          }
        }
      }
    }
    // Visit only the candidate tokens (set bits), in position order.
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      if (c < n_pass) {
        const int t = chunk_t0 + c * PASS + tid * kSelTokPerThread;
        const int64_t page_row0 = prow[c];
        uint32_t lt = lt0[c], eq = eq0[c];
        auto emit = [&](int j, bool is_eq) {
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
        };
        if constexpr (BYTES) {
          const uint32_t eq16 = flags[c] >> 16;
          uint32_t cand = (flags[c] & 0xffffu) | eq16;
          while (cand != 0u) {
            const int j = __builtin_ctz(cand);
            cand &= cand - 1u;
            emit(j, (eq16 >> j) & 1u);
          }
        } else {
#pragma unroll
          for (int w = 0; w < DW; ++w) {
            uint32_t cand = m_lt[w] | m_eq[w];
            while (cand != 0u) {
              const int bit = __builtin_ctz(cand);
              cand &= cand - 1u;
              emit(TPW * w + bit / TB, (m_eq[w] >> bit) & 1u);
            }
          }
        }
      }
    }
    first_chunk = false;
    // the next chunk rewrites the wave totals that slower waves may still be reading
    if (chunk_t0 + kChunk * PASS < seg_t1) __syncthreads();
  }
  };
  run_passes(std::integral_constant<int, BYTES ? CHUNK : 1>{});
  if (seg == 0 && idx_row != nullptr)
    for (int i = kk + tid; i < p.k; i += THREADS) idx_row[i] = -1;

  if constexpr (ATTN) {
    const int n_sel = min((int)(run_lt + min(run_eq, (uint32_t)r) - seg_pos0), kk);
    __syncthreads();  // s_sel complete
    trace.stamp(kSelCompacted, false);  // (not waiting for the index stores)
    float M, lsum, o;
    attention_rows<THREADS, D>(s_sel, n_sel, (int)gather_rows, qv,
                            p.K + row0, p.V + row0, p.scale_log2e, s_attn, M, lsum, o, trace);
    // the early requests have long returned; this only keeps them alive until here
#pragma unroll
    for (int i = 0; i < 2 * kRowLines; ++i) asm volatile("" : : "v"(early[i]));
    trace.stamp(kSelCombined, false);
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
      s_last = before + 1u == (uint32_t)n_active ? 1 : 0;
    }
    __syncthreads();
    trace.stamp(kSelCounted);
    if (s_last == 0) {
      trace.stamp(kSelEnd);
      trace.flush(p.trace, p.trace_records);
      return;
    }
    if (tid >= D) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const float* ph = p.partial + head * kMaxParts * kPartial;
    static_assert(kMaxParts == 16, "two merge widths: up to 8 and up to 16 partials");
    p.out[head * D + tid] = n_active <= 8 ? merge_slots<8, D>(ph, n_active, tid)
                                          : merge_slots<16, D>(ph, n_active, tid);
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
  uint32_t group_magic;                // see kv_head_of
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
  const uint4 qv = load_query_piece<D>(p.q + head * D);
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
  const int kvh = kv_head_of(hq, p.group_magic);
  const int64_t row0 = ((int64_t)kvh * p.pool_tokens + start) * D;
  float M, lsum, o;
  PhaseTrace trace;  // not recorded for the stand-alone kernel
  attention_rows<kAttnThreads, D>(s_sel, (int)n, (int)min((int64_t)0x7fffffff, p.pool_tokens - start),
                               qv, p.K + row0, p.V + row0, p.scale_log2e, s_attn, M, lsum, o, trace);
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
    const float w = use ? exp2_neg(pm[s] - M) : 0.f;
    lsum = fmaf(use ? pl[s] : 0.f, w, lsum);
    o = fmaf(use ? po[s] : 0.f, w, o);
  }
  p.out[head * D + tid] = lsum > 0.f ? o / lsum : 0.f;
}

}  // namespace adamas
