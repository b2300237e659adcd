// Manhattan-distance scan over the packed code plane (Algorithm 1 line 5,
// Eq. 6), with the query encode (lines 1-3) and the cache append (line 4)
// fused into its prologue for the decode step.
//
// One workgroup owns one tile of blockDim.x * 4 consecutive tokens of one
// (sequence, KV head) and evaluates all G query heads of that KV head's
// group on it, so every code row is fetched once.  It writes
//   - one uint16 distance per (query head, token), and
//   - one 385-bin histogram of those distances per (query head, tile),
// both with plain stores: nothing needs zero-initialised memory and the
// result does not depend on the order workgroups run in.
//
// Distance on bit planes.  A row word carries 32 low bits and 32 high bits of
// 32 codes.  With x = query ^ key per plane and g = q_hi ^ q_lo (query only):
//   |a - b| = x_lo + 2 * (x_hi & ~(x_lo & g))
// (x_hi = 0: the codes differ by x_lo; x_hi = 1, x_lo = 0: by 2; both set:
// by 3 when the query code is 0 or 3 (g = 0), by 1 when it is 1 or 2), so a
// 32-coefficient word costs two xor, one and, one and-not and two popcounts.
#pragma once

#include "device_utils.hpp"
#include "encode.hpp"

namespace adamas {

constexpr int kScanTokPerThread = 4;
constexpr int kHistReplicas = 4;  // LDS histogram copies, picked by lane, to thin out same-address atomics

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
  uint16_t* dist;            // [B*Hq][dist_stride]; may be null
  int64_t dist_stride;
  uint16_t* dist_user;       // optional second copy, [B*Hq][dist_user_stride]
  int64_t dist_user_stride;
  uint16_t* tilehist;        // [B*Hq][n_tiles][kHistStride]; may be null
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, Hkv, n_tiles;
  Thresholds thr_q, thr_k;
};

template <int G, bool FUSED>
__global__ __launch_bounds__(1024) void scan_kernel(const ScanParams p) {
  __shared__ uint32_t s_hist[G][kHistReplicas][kNumBins];
  __shared__ uint32_t s_q[G][12];   // per query head: lo[4], hi[4], lo^hi[4]
  __shared__ uint32_t s_new[8];     // code row of the appended key

  const int tile_id = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int tile_tokens = blockDim.x * kScanTokPerThread;
  const int L = safe_seq_len(p.seq_len, p.seq_start, b, p.max_seq_len, p.pool_tokens);
  const int64_t start = p.seq_start[b];
  const int t0 = tile_id * tile_tokens;
  const int head0 = b * p.Hq + kvh * G;

  if (t0 >= L) return;  // whole workgroup

  // Issue this thread's row loads first: they do not depend on the query.
  const uint8_t* plane = p.codes + ((int64_t)kvh * p.pool_tokens + start) * kRowBytes;
  uint4 ra[kScanTokPerThread], rb[kScanTokPerThread];
#pragma unroll
  for (int i = 0; i < kScanTokPerThread; ++i) {
    const int t = t0 + (wave * kScanTokPerThread + i) * kWave + lane;
    if (t < L) {
      const uint4* row = reinterpret_cast<const uint4*>(plane + (int64_t)t * kRowBytes);
      ra[i] = row[0];
      rb[i] = row[1];
    } else {
      ra[i] = make_uint4(0, 0, 0, 0);
      rb[i] = make_uint4(0, 0, 0, 0);
    }
  }

  for (int i = tid; i < G * kHistReplicas * kNumBins; i += blockDim.x)
    (&s_hist[0][0][0])[i] = 0u;

  const bool appending = FUSED && p.k_new != nullptr && (L - 1) / tile_tokens == tile_id;
  if (FUSED) {
    const int n_enc = G + (appending ? 1 : 0);
    for (int v = wave; v < n_enc; v += nwaves) {
      uint64_t w[4];
      if (v < G) {
#ifdef EXP_NOENC
        w[0] = w[1] = w[2] = w[3] = 0x123456789abcdefull;
#else
        encode_vector_wave(p.q + (int64_t)(head0 + v) * kHeadDim, p.thr_q, w);
#endif
        if (lane < 4) {
          const uint64_t x = lane == 0 ? w[0] : lane == 1 ? w[1] : lane == 2 ? w[2] : w[3];
          const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
          s_q[v][lane] = lo;
          s_q[v][4 + lane] = hi;
          s_q[v][8 + lane] = lo ^ hi;
        }
      } else {
        // Alg. 1 line 4: the new token's K, V and code row enter the cache
        // before the scan; this workgroup owns the tile that holds it.
        const int64_t src = ((int64_t)b * p.Hkv + kvh) * kHeadDim;
        const int64_t row = (int64_t)kvh * p.pool_tokens + start + (L - 1);
        encode_vector_wave(p.k_new + src, p.thr_k, w);
        store_row_wave(p.codes_w + row * kRowBytes, w);
        if (lane < 4) {
          const uint64_t x = lane == 0 ? w[0] : lane == 1 ? w[1] : lane == 2 ? w[2] : w[3];
          s_new[2 * lane] = (uint32_t)x;
          s_new[2 * lane + 1] = (uint32_t)(x >> 32);
        }
        reinterpret_cast<uint32_t*>(p.K + row * kHeadDim)[lane] =
            reinterpret_cast<const uint32_t*>(p.k_new + src)[lane];
        reinterpret_cast<uint32_t*>(p.V + row * kHeadDim)[lane] =
            reinterpret_cast<const uint32_t*>(p.v_new + src)[lane];
      }
    }
  } else {
    if (tid < G * 4) {
      const int g = tid >> 2, wd = tid & 3;
      const uint32_t* qc = reinterpret_cast<const uint32_t*>(p.qcodes + (int64_t)(head0 + g) * kRowBytes);
      const uint32_t lo = qc[2 * wd], hi = qc[2 * wd + 1];
      s_q[g][wd] = lo;
      s_q[g][4 + wd] = hi;
      s_q[g][8 + wd] = lo ^ hi;
    }
  }
  __syncthreads();

  // The query planes are wave-uniform: keep them in scalar registers.
  uint32_t qlo[G][4], qhi[G][4], qg[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) {
      qlo[g][wd] = __builtin_amdgcn_readfirstlane(s_q[g][wd]);
      qhi[g][wd] = __builtin_amdgcn_readfirstlane(s_q[g][4 + wd]);
      qg[g][wd] = __builtin_amdgcn_readfirstlane(s_q[g][8 + wd]);
    }
  }
  uint32_t* hist_lane = &s_hist[0][lane & (kHistReplicas - 1)][0];

#pragma unroll
  for (int i = 0; i < kScanTokPerThread; ++i) {
    const int t = t0 + (wave * kScanTokPerThread + i) * kWave + lane;
    uint32_t klo[4] = {ra[i].x, ra[i].z, rb[i].x, rb[i].z};
    uint32_t khi[4] = {ra[i].y, ra[i].w, rb[i].y, rb[i].w};
    if (appending && t == L - 1) {
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        klo[wd] = s_new[2 * wd];
        khi[wd] = s_new[2 * wd + 1];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint32_t c1 = 0, c2 = 0;
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const uint32_t xl = klo[wd] ^ qlo[g][wd], xh = khi[wd] ^ qhi[g][wd];
        c1 += __popc(xl);
        c2 += __popc(xh & ~(xl & qg[g][wd]));
      }
      const uint32_t d = c1 + 2u * c2;
      if (t < L) {
        const int64_t head = head0 + g;
#ifndef EXP_NODIST
        if (p.dist != nullptr) p.dist[head * p.dist_stride + t] = (uint16_t)d;
#endif
        if (p.dist_user != nullptr) p.dist_user[head * p.dist_user_stride + t] = (uint16_t)d;
#ifndef EXP_NOHIST
        atomicAdd(hist_lane + g * (kHistReplicas * kNumBins) + d, 1u);
#else
        if (d == 0x7fffffffu) hist_lane[0] = 1;
#endif
      }
    }
  }

  if (p.tilehist != nullptr) {
    __syncthreads();
    for (int i = tid; i < G * kNumBins; i += blockDim.x) {
      const int g = i / kNumBins, bin = i - g * kNumBins;
      uint32_t s = 0;
#pragma unroll
      for (int r = 0; r < kHistReplicas; ++r) s += s_hist[g][r][bin];
      p.tilehist[((int64_t)(head0 + g) * p.n_tiles + tile_id) * kHistStride + bin] = (uint16_t)s;
    }
  }
}

}  // namespace adamas
