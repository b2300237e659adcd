// Manhattan-distance scan over the packed code plane (Algorithm 1, distance
// step, Eq. 6), with the query encode and the cache append of the same
// algorithm fused into its prologue for the decode step.
//
// One workgroup owns one tile of blockDim.x * 4 consecutive tokens of one
// (sequence, KV head) and evaluates all G query heads of that KV head's
// group on it, so every code row is fetched once.  It writes
//   - one distance per (query head, token), staged through LDS so that a lane
//     stores four consecutive tokens: a byte each (plus one bit per token in a
//     plane of ninth bits, written straight from wave ballots) when the metric's
//     distances stay below 512, as Eq. 6 does (0..384); uint16 otherwise, and
//   - one histogram of those distances (385 bins for Eq. 6) per (query head, tile),
// both with plain stores: nothing needs zero-initialised memory and the
// result does not depend on the order workgroups run in.
//
// Distance on bit planes.  A row word carries 32 low bits and 32 high bits of
// 32 codes.  With x = query ^ key per plane and g = q_hi ^ q_lo (query only):
//   |a - b| = x_lo + 2 * (x_hi & ~(x_lo & g))
// (x_hi = 0: the codes differ by x_lo; x_hi = 1, x_lo = 0: by 2; both set:
// by 3 when the query code is 0 or 3 (g = 0), by 1 when it is 1 or 2), so a
// 32-coefficient word costs two xor, one and, one and-not and two popcounts.
// The squared-difference variant (Section 4.4) needs one more and + popcount:
//   (a - b)^2 = x_lo + 4 * u + 4 * (u & x_lo),  u = x_hi & ~(x_lo & g).
#pragma once

#include <type_traits>

#include "device_utils.hpp"
#include "encode.hpp"

namespace adamas {

constexpr int kScanTokPerThread = 4;
// LDS histogram copies, picked by lane, to thin out same-address atomics: two
// unless the histograms of the group would then take more than 48 KiB.  The
// tile histogram in memory packs two 16-bit bins per word (a tile has at most
// 4096 tokens).  In LDS a group of up to two query heads keeps that format
// (the scan is then bound by memory and the smaller histogram is flushed
// sooner); larger groups are bound by their instructions and use a 32-bit word
// per bin, whose address is the distance itself and whose increment is a
// constant (measured: 0.2 us slower for a group of one, 0.1 to 0.2 us faster
// for a group of four).
constexpr bool hist_wide_bins(int group) { return group > 2; }
constexpr int hist_replicas(int group, int bins) {
  return group * bins * (hist_wide_bins(group) ? 8 : 4) > 48 * 1024 ? 1 : 2;
}

struct ScanParams {
  const uint8_t* codes;      // [Hkv][pool][32]
  uint8_t* codes_w;          // same buffer, written on append (fused only)
  const uint16_t* q;         // bf16 [B][Hq][128]      (fused)
  const uint8_t* qcodes;     // [B][Hq][32]            (not fused)
  const uint16_t* k_new;     // bf16 [B][Hkv][128] or null
  const uint16_t* v_new;
  uint16_t* K;               // pools, written on append
  uint16_t* V;
  const int64_t* seq_start;  // [B]
  const int32_t* seq_len;    // [B]
  void* dist;                // [B*Hq][dist_stride] bytes or uint16 (Dist<>::kDistBytes); may be null
  uint64_t* dist_high;       // ninth bits, [B*Hq][dist_stride / 64] (Dist<>::kHighPlane only)
  int64_t dist_stride;       // tokens per row, a multiple of 128
  uint16_t* dist_user;       // optional second copy, [B*Hq][dist_user_stride]
  int64_t dist_user_stride;
  uint32_t* tilehist;        // [B*Hq][n_tiles][Dist<>::kPairs] words of two 16-bit bins; may be null
  uint32_t* arrivals;        // per-head counter at [head * arrivals_stride], zeroed here; may be null
  int64_t arrivals_stride;
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, Hkv, n_tiles;
  int32_t g_split;           // workgroups per (tile, KV head), 1 or 2: each takes G of the group's G * g_split query heads
  // Paged cache (PAGED kernels only): token t of sequence b lives in pool row
  // page_table[b * max_pages + (t >> page_shift)] << page_shift | (t & page mask).
  const int32_t* page_table;
  int32_t max_pages, page_shift;
  Thresholds thr_q, thr_k;
  // Profiling builds only: one record of phase stamps per workgroup (see PhaseTrace).
  uint64_t* trace;
  int64_t trace_records;
};

// Phase stamps of scan_kernel, in the order they are taken.
enum ScanPhase {
  kScanStart = 0,    // first instruction
  kScanLengthKnown,  // past the early barrier: sequence length and start have arrived
  kScanQueryReady,   // the query planes are published in LDS
  kScanRowsDone,     // every row of the tile has arrived and its distances are in LDS
  kScanDistStored,   // distance stores acknowledged
  kScanEnd           // histogram flushed and acknowledged
};

// WAVES = wavefronts per workgroup (4, 8 or 16): the tile is WAVES * 256 tokens.
// D = head dimension: W = D / 32 words per code row.
template <int G, bool FUSED, int WAVES, int METRIC, bool PAGED, int D>
__global__ __launch_bounds__(WAVES * kWave) void scan_kernel(const ScanParams p) {
  static_assert(FUSED || !PAGED, "the paged layout is served by the fused step only");
  using Fmt = Dist<METRIC, D>;
  constexpr int kNumBins = Fmt::kBins;
  constexpr int BITS = Fmt::kBits, kRowBytes = Fmt::kRowBytes, W = Fmt::kWords;
  constexpr int kRowWords = W * BITS;  // 32-bit words per code row
  constexpr int kHistReplicas = hist_replicas(G, kNumBins);
  constexpr int E = HeadDim<D>::kEncElems;  // elements per lane when a wave encodes one vector
  constexpr int kPairs = Fmt::kPairs;  // 32-bit words of a histogram: two 16-bit bins each
  constexpr bool kWideBins = hist_wide_bins(G);
  constexpr int kHistWords = kWideBins ? 2 * kPairs : kPairs;  // LDS words of one histogram copy
  __shared__ uint32_t s_hist[G][kHistReplicas][kHistWords];
  // per query head: plane p of word wd at [W * p + wd]; 2-bit codes also keep lo^hi at [2W + wd]
  __shared__ uint32_t s_q[G][3 * W];
  __shared__ uint32_t s_new[kRowWords];  // code row of the appended key, as stored
  __shared__ uint32_t s_ready;      // query / new-key code rows published so far
  // per wave: its 256 distances per query head, in token order, for wide stores
  using DistT = typename std::conditional<Fmt::kByteDist, uint8_t, uint16_t>::type;
  __shared__ __align__(8) DistT s_dt[WAVES][G][kScanTokPerThread * kWave];

  // blockIdx.y = KV head * g_split + part: the G query heads of this workgroup are
  // part `gsub` of the KV head's group of G * g_split (the parts re-read the rows).
  PhaseTrace trace;
  trace.stamp(kScanStart);
  // requested first of all: the row loads cannot be addressed without them
  SeqInfo seq = SeqInfo::request<PAGED, true>(p.seq_len, p.seq_start, (int)blockIdx.z);
  __builtin_amdgcn_sched_barrier(0);
  // g_split is 1 or 2
  const int tile_id = blockIdx.x, kvh = blockIdx.y >> (p.g_split - 1), gsub = blockIdx.y & (p.g_split - 1);
  const int b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int nthreads = WAVES * kWave;
  constexpr int tile_tokens = nthreads * kScanTokPerThread;
  const int t0 = tile_id * tile_tokens;
  const int head0 = b * p.Hq + (kvh * p.g_split + gsub) * G;

  // First of all the encoding waves request their vectors (G queries and, if
  // the call appends, the new key): their addresses need nothing from memory,
  // so these loads travel together with the scalar loads of the sequence
  // length and start below.  Only the encoding waves load: inside a compute
  // unit requests are served in order across waves, so a needless load here
  // would sit in front of other waves' rows.
  constexpr int kEncRounds = (G + 1 + WAVES - 1) / WAVES;  // G queries + 1 new key over the waves
  uint32_t enc[kEncRounds][E];
#pragma unroll
  for (int r = 0; r < kEncRounds; ++r) {
    const int v = wave + r * WAVES;
#pragma unroll
    for (int e = 0; e < E; ++e) enc[r][e] = 0;
    if (FUSED && (v < G || (v == G && p.k_new != nullptr))) {
      const uint16_t* src = v < G ? p.q + (int64_t)(head0 + v) * D
                                  : p.k_new + ((int64_t)b * p.Hkv + kvh) * D;
#pragma unroll
      for (int e = 0; e < E; ++e)
        enc[r][e] = lane < HeadDim<D>::kEncLanes ? src[HeadDim<D>::enc_index(lane, e)] : 0u;
    }
  }

  // Paged cache: the page of each of the wave's four 64-token steps (a step
  // never straddles a page: pages are multiples of 64 tokens).  Scalar loads,
  // on their way together with the length.
  int32_t pte[kScanTokPerThread];
  if constexpr (PAGED) {
    const int uw = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int i = 0; i < kScanTokPerThread; ++i) {
      const int pg = min((t0 + (uw * kScanTokPerThread + i) * kWave) >> p.page_shift, p.max_pages - 1);
      pte[i] = scalar_load(p.page_table + (int64_t)b * p.max_pages + pg);
    }
  }
  loads_issued_before_here();
  const int L = PAGED ? seq.paged_length(p.max_seq_len, (int64_t)p.max_pages << p.page_shift)
                      : seq.length(p.max_seq_len, p.pool_tokens);
  const int64_t start = seq.start;

  // The only workgroup barrier before the scan sits here, where every wave has
  // just started (and while the loads above are still on their way).  Later on
  // the waves must not wait for each other: a compute unit serves memory
  // requests in order, so late waves get their rows late, and a barrier after
  // the row loads would hold the early waves back with them.
  for (int i = tid; i < G * kHistReplicas * kHistWords; i += nthreads)
    (&s_hist[0][0][0])[i] = 0u;
  if (tid == 0) s_ready = 0u;
  __syncthreads();

  // The select kernel counts its finished segments per head from zero (tile 0
  // exists for every sequence, empty ones included).
  if (p.arrivals != nullptr && tile_id == 0 && tid < G)
    p.arrivals[(int64_t)(head0 + tid) * p.arrivals_stride] = 0u;
  if (t0 >= L) return;  // whole workgroup
#ifdef ADAMAS_PHASE_TRACE   // (no wait here: the encode vectors are still on their way)
  if (threadIdx.x == 0) trace.t[kScanLengthKnown] = wall_clock64();
#endif

  // Order of the memory operations matters: loads return in issue order, so a
  // wave that waits for one load also waits for everything it issued before.
  // The code rows are requested next and consumed one token at a time as they
  // arrive; the encode runs while they travel.
  const bool appending = FUSED && p.k_new != nullptr && (L - 1) / tile_tokens == tile_id;
  const int n_enc = FUSED ? G + (appending ? 1 : 0) : 0;
  uint32_t qraw[BITS];  // not fused: thread (head, word) of wave 0 fetches its planes
#pragma unroll
  for (int pl = 0; pl < BITS; ++pl) qraw[pl] = 0;
  if (!FUSED && wave == 0) {
    const int i = min(tid, G * W - 1);
    const uint32_t* qc =
        reinterpret_cast<const uint32_t*>(p.qcodes + (int64_t)(head0 + i / W) * kRowBytes);
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) qraw[pl] = qc[BITS * (i % W) + pl];
  }

  const uint8_t* plane = p.codes + ((int64_t)kvh * p.pool_tokens + start) * kRowBytes;
  constexpr int kPiece = Fmt::kPiece, C = kRowBytes / kPiece;  // a row is fetched in C pieces
  uint32_t rr[kScanTokPerThread][kRowWords];
#pragma unroll
  for (int i = 0; i < kScanTokPerThread; ++i) {
    // Unconditional: a lane past the end re-reads the last row (masked at use).
    // A branch here would make the compiler wait for all loads at once.
    int64_t r;
    if constexpr (PAGED) {
      // a page number outside the pool is clamped into it; lanes past the end read row 0
      const int t = t0 + (wave * kScanTokPerThread + i) * kWave + lane;
      const int64_t pg = min(max((int64_t)pte[i], (int64_t)0), (p.pool_tokens >> p.page_shift) - 1);
      r = t < L ? (pg << p.page_shift) + (t & ((1 << p.page_shift) - 1)) : 0;
    } else {
      r = min(t0 + (wave * kScanTokPerThread + i) * kWave + lane, L - 1);
    }
    const uint8_t* row = plane + r * kRowBytes;
#pragma unroll
    for (int c = 0; c < C; ++c) load_piece<kPiece>(row + c * kPiece, &rr[i][c * (kPiece / 4)]);
  }

  // Nothing above may be consumed before the row loads have been issued.
  if (FUSED) {
#pragma unroll
    for (int r = 0; r < kEncRounds; ++r) {
#pragma unroll
      for (int e = 0; e < E; ++e) asm volatile("" : "+v"(enc[r][e]));
    }
  } else {
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) asm volatile("" : "+v"(qraw[pl]));
  }

  if (FUSED) {
#pragma unroll
    for (int r = 0; r < kEncRounds; ++r) {
      const int v = wave + r * WAVES;
      if (v < n_enc) {
        uint32_t w[BITS][W];
        encode_values_wave<BITS, D>(enc[r], v < G ? p.thr_q : p.thr_k, w);
        // lane wd publishes word wd (every lane holds the whole row)
#pragma unroll
        for (int wd = 0; wd < W; ++wd) {
          if (lane == wd) {
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl) {
              if (v < G) s_q[v][W * pl + wd] = w[pl][wd];
              else s_new[BITS * wd + pl] = w[pl][wd];  // code row of the appended key
            }
            if (BITS == 2 && v < G) s_q[v][2 * W + wd] = w[0][wd] ^ w[BITS - 1][wd];
          }
        }
        if (lane == 0)
          __hip_atomic_fetch_add(&s_ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
  } else if (wave == 0) {
    if (tid < G * W) {
      const int g = tid / W, wd = tid % W;
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl) s_q[g][W * pl + wd] = qraw[pl];
      if (BITS == 2) s_q[g][2 * W + wd] = qraw[0] ^ qraw[BITS - 1];
    }
    if (lane == 0)
      __hip_atomic_fetch_add(&s_ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  // Wait for the publishing waves only.  They never wait for anybody, so this
  // ends; the spin bound is a last resort that turns a logic error into wrong
  // distances instead of a hung GPU.
  {
    const uint32_t n_ready = FUSED ? (uint32_t)n_enc : 1u;
    for (int spin = 0; spin < (1 << 22); ++spin) {
      if (__hip_atomic_load(&s_ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= n_ready)
        break;
      __builtin_amdgcn_s_sleep(2);
    }
  }

  trace.stamp(kScanQueryReady);
  // The query planes are wave-uniform.  Up to 24 words (the method's group of
  // one or two) live in vector registers.  Larger groups keep them in scalar
  // registers (every instruction of the distance needs only one of them, and the
  // kernel then fits 64 vector registers), at most 24 words at a time: the heads
  // of the group are served in passes of kPassHeads over the rows, which stay
  // in registers.  All planes of a group of four at once take about 100 scalar
  // registers, and it is then the scalar register file that limits how many
  // waves a compute unit holds (measured: the only resource the dispatcher
  // reports as full, with about four waves per SIMD resident).
  // qp[g][j][wd]: plane j of word wd; for 2-bit codes j = 2 is lo ^ hi.
  constexpr int QP = BITS == 2 ? 3 : BITS;
  constexpr bool kPlanesInVgprs = G * QP * W <= 24;
  constexpr int kPassHeads = kPlanesInVgprs ? G : (24 / (QP * W) > 0 ? 24 / (QP * W) : 1);
  uint32_t* hist_lane = &s_hist[0][lane & (kHistReplicas - 1)][0];

  // Ninth bits (byte planes of distances up to 511): the ballot of step i over the
  // wave's 64 tokens is one word of the plane; lane i keeps the word of step i.
  uint32_t high_lo[G], high_hi[G];
#pragma unroll
  for (int g = 0; g < G; ++g) high_lo[g] = high_hi[g] = 0u;
#pragma unroll
  for (int g0 = 0; g0 < G; g0 += kPassHeads) {
  uint32_t qp[kPassHeads][QP][W];
#pragma unroll
  for (int g = g0; g < g0 + kPassHeads && g < G; ++g) {
#pragma unroll
    for (int j = 0; j < QP; ++j) {
#pragma unroll
      for (int wd = 0; wd < W; ++wd) {
        if constexpr (kPlanesInVgprs) qp[g - g0][j][wd] = s_q[g][W * j + wd];
        else qp[g - g0][j][wd] = __builtin_amdgcn_readfirstlane(s_q[g][W * j + wd]);
      }
    }
  }
  auto qplane = [&](int g, int j, int wd) -> uint32_t { return qp[g - g0][j][wd]; };
#pragma unroll
  for (int i = 0; i < kScanTokPerThread; ++i) {
    // keep the tokens in load order, so that each waits only for its own rows
    if (g0 == 0) __builtin_amdgcn_sched_barrier(0);
    const int t = t0 + (wave * kScanTokPerThread + i) * kWave + lane;
    const uint64_t in_range = __builtin_amdgcn_ballot_w64(t < L);
    // kw[BITS * wd + pl]: plane pl of word wd of the key row
    uint32_t kw[kRowWords];
#pragma unroll
    for (int wq = 0; wq < kRowWords; ++wq) kw[wq] = rr[i][wq];
    if (appending && t == L - 1) {
#pragma unroll
      for (int wq = 0; wq < kRowWords; ++wq) kw[wq] = s_new[wq];
    }
#pragma unroll
    for (int g = g0; g < g0 + kPassHeads && g < G; ++g) {
      uint32_t d;
      if constexpr (BITS == 2) {
        uint32_t c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
        for (int wd = 0; wd < W; ++wd) {
          // Every instruction below takes one query plane: with two of them in one
          // instruction (the compiler's choice when it may merge them) a plane held
          // in a scalar register must first be copied.  Hence the opaque values.
          uint32_t xl = kw[2 * wd] ^ qplane(g, 0, wd);
          asm("" : "+v"(xl));
          uint32_t both = xl & qplane(g, 2, wd);
          asm("" : "+v"(both));
          const uint32_t u = (kw[2 * wd + 1] ^ qplane(g, 1, wd)) & ~both;
          c1 += __popc(xl);
          c2 += __popc(u);
          if constexpr (METRIC == kMetricL2) c3 += __popc(u & xl);
        }
        d = METRIC == kMetricL1 ? c1 + 2u * c2 : c1 + 4u * (c2 + c3);
      } else if constexpr (BITS == 1) {
        d = 0;
#pragma unroll
        for (int wd = 0; wd < W; ++wd) d += __popc(kw[wd] ^ qplane(g, 0, wd));
      } else {
        // |a - b| of 3-bit codes on bit planes (a query, b key): subtract with
        // borrow, then negate where the borrow out (a < b) is set.
        uint32_t c0 = 0, c1 = 0, c2 = 0;
#pragma unroll
        for (int wd = 0; wd < W; ++wd) {
          const uint32_t a0 = qplane(g, 0, wd), a1 = qplane(g, 1, wd), a2 = qplane(g, 2, wd);
          const uint32_t b0 = kw[3 * wd], b1 = kw[3 * wd + 1], b2 = kw[3 * wd + 2];
          const uint32_t d0 = a0 ^ b0, br1 = ~a0 & b0;
          const uint32_t x1 = a1 ^ b1, d1 = x1 ^ br1, br2 = (~a1 & b1) | (~x1 & br1);
          const uint32_t x2 = a2 ^ b2, d2 = x2 ^ br2, sg = (~a2 & b2) | (~x2 & br2);
          const uint32_t e1 = d1 ^ sg, cy1 = ~d0 & sg;
          const uint32_t r1 = e1 ^ cy1, cy2 = e1 & cy1;
          const uint32_t r2 = d2 ^ sg ^ cy2;
          c0 += __popc(d0);
          c1 += __popc(r1);
          c2 += __popc(r2);
        }
        d = c0 + 2u * c1 + 4u * c2;
      }
      s_dt[wave][g][i * kWave + lane] = (DistT)d;
      // ninth bits of 64 consecutive tokens = one word of the plane, straight from the ballot
      if constexpr (Fmt::kHighPlane) {
        const uint64_t word = __builtin_amdgcn_ballot_w64(d > 255u) & in_range;
        write_lane(high_lo[g], (uint32_t)word, i);
        write_lane(high_hi[g], (uint32_t)(word >> 32), i);
      }
      if constexpr (kWideBins) {
        if (t < L) atomicAdd(hist_lane + g * (kHistReplicas * kHistWords) + d, 1u);
      } else {
        // two 16-bit bins per word: 1 for an even distance, 0x10000 for an odd one
        // (opaque halves: otherwise the compiler turns them into a compare and a select)
        uint32_t pair = d >> 1, odd16 = (d & 1u) << 4;
        asm("" : "+v"(pair), "+v"(odd16));
        if (t < L) atomicAdd(hist_lane + g * (kHistReplicas * kHistWords) + pair, 1u << odd16);
      }
    }
  }
  }  // passes over the heads of the group

  trace.stamp(kScanRowsDone);
  // Distances leave through LDS: a lane computed tokens 64 apart, but stores
  // four consecutive tokens (8 bytes), so a wave writes 512 contiguous bytes
  // per query head with one instruction instead of four 2-byte-per-lane ones.
  // The region is private to the wave, so no barrier is needed.
  // A row of the plane holds a multiple of 128 tokens, so a lane whose first
  // token exists may store all four.
  if constexpr (Fmt::kHighPlane) {
    // The wave's kScanTokPerThread words of the ninth-bit plane are consecutive:
    // lane i stores word i (64 tokens from t64), if that word holds tokens.
    const int t64 = t0 + (wave * kScanTokPerThread + lane) * kWave;
    if (p.dist != nullptr && lane < kScanTokPerThread && t64 < L) {
#pragma unroll
      for (int g = 0; g < G; ++g)
        p.dist_high[((int64_t)(head0 + g) * p.dist_stride + t64) >> 6] =
            ((uint64_t)high_hi[g] << 32) | high_lo[g];
    }
  }
  if (p.dist_user != nullptr) {  // the caller's own array of distances (adamas_distances)
#pragma unroll
    for (int i = 0; i < kScanTokPerThread; ++i) {
      const int t = t0 + (wave * kScanTokPerThread + i) * kWave + lane;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        uint32_t d = s_dt[wave][g][i * kWave + lane];
        if constexpr (Fmt::kHighPlane) {
          const uint32_t w_lo = (uint32_t)__builtin_amdgcn_readlane((int)high_lo[g], i);
          const uint32_t w_hi = (uint32_t)__builtin_amdgcn_readlane((int)high_hi[g], i);
          d |= (((lane < 32 ? w_lo : w_hi) >> (lane & 31)) & 1u) << 8;
        }
        if (t < L) p.dist_user[(int64_t)(head0 + g) * p.dist_user_stride + t] = (uint16_t)d;
      }
    }
  }
  if (p.dist != nullptr) {
    const int tt = t0 + wave * (kScanTokPerThread * kWave) + kScanTokPerThread * lane;
    if (tt < L) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const int64_t at = (int64_t)(head0 + g) * p.dist_stride + tt;
        if constexpr (Fmt::kByteDist) {
          *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(p.dist) + at) =
              *reinterpret_cast<const uint32_t*>(&s_dt[wave][g][kScanTokPerThread * lane]);
        } else {
          *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.dist) + at) =
              *reinterpret_cast<const uint2*>(&s_dt[wave][g][kScanTokPerThread * lane]);
        }
      }
    }
  }

  trace.stamp(kScanDistStored);
  // Algorithm 1, cache update: the new token's K, V and code row enter the cache.  The
  // scan above already used the new code row (from LDS); the stores come last
  // so that no other memory operation sits between the row loads and their use.
  if (appending && wave == 0 && gsub == 0) {
    const int64_t src = ((int64_t)b * p.Hkv + kvh) * D;
    int64_t row = (int64_t)kvh * p.pool_tokens + start + (L - 1);
    if constexpr (PAGED) {
      const int64_t pg = min(max((int64_t)p.page_table[(int64_t)b * p.max_pages + ((L - 1) >> p.page_shift)],
                                 (int64_t)0), (p.pool_tokens >> p.page_shift) - 1);
      row = (int64_t)kvh * p.pool_tokens + (pg << p.page_shift) + ((L - 1) & ((1 << p.page_shift) - 1));
    }
    if (lane < kRowWords) reinterpret_cast<uint32_t*>(p.codes_w + row * kRowBytes)[lane] = s_new[lane];
#pragma unroll
    for (int c = lane; c < D / 2; c += kWave) {  // D bf16 values = D / 2 dwords per row
      reinterpret_cast<uint32_t*>(p.K + row * D)[c] = reinterpret_cast<const uint32_t*>(p.k_new + src)[c];
      reinterpret_cast<uint32_t*>(p.V + row * D)[c] = reinterpret_cast<const uint32_t*>(p.v_new + src)[c];
    }
  }
  if (p.tilehist != nullptr) {
    __syncthreads();
    for (int i = tid; i < G * kPairs; i += nthreads) {
      const int g = i / kPairs, pr = i - g * kPairs;
      uint32_t v = 0;
#pragma unroll
      for (int r = 0; r < kHistReplicas; ++r) {
        if constexpr (kWideBins) v += s_hist[g][r][2 * pr] + (s_hist[g][r][2 * pr + 1] << 16);  // (a last odd bin that no distance reaches stays zero)
        else v += s_hist[g][r][pr];
      }
      p.tilehist[((int64_t)(head0 + g) * p.n_tiles + tile_id) * kPairs + pr] = v;
    }
  }
  trace.stamp(kScanEnd);
  trace.flush(p.trace, p.trace_records);
}

}  // namespace adamas
