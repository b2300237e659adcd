// Dense decode attention: Eq. 1 over EVERY cached row of a sequence.  This is
// not a step of the method but what it is compared with (the paper's
// "self-attention speedup" is sparse attention against full attention), so
// that both sides of that ratio can be measured on the same GPU.
//
// Split along the sequence: workgroup (split, KV head, sequence) streams the K
// and V rows of its chunk once and serves all G query heads of the group from
// them, keeping one online-softmax state (m, l, o[128]) per query head; a
// second kernel merges the splits of a head.  HBM-bound: 512 B per cached row
// per KV head, 4 * G * 128 flop on it.
#pragma once

#include "device_utils.hpp"
#include "select_attn.hpp"

namespace adamas {

constexpr int kFullThreads = 256;
constexpr int kFullMaxSplits = 256;

// One softmax state per row group of a workgroup, for the combine through LDS.
template <int D>
struct FullShared {
  static constexpr int kGroups = kFullThreads / HeadDim<D>::kRowGroup;
  float m[kGroups];
  float l[kGroups];
  float acc[kGroups][D];
};

struct FullAttnParams {
  const uint16_t* q;         // bf16 [B][Hq][128]
  const uint16_t* K;         // pools
  const uint16_t* V;
  const int64_t* seq_start;  // [B]
  const int32_t* seq_len;    // [B]
  float* partial;            // [B*Hq][n_splits][kPartial]
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, Hkv, n_splits, chunk;  // chunk = tokens per split
  float scale_log2e;
};

// Grid (n_splits, Hkv, B).  16 lanes per row (8 dims each), 16 rows per pass
// per workgroup, U passes in flight.  A split without tokens leaves an empty
// partial (l = 0), so the merge needs no knowledge of the lengths.
template <int G, int D>
__global__ __launch_bounds__(kFullThreads) void full_attn_kernel(const FullAttnParams p) {
#pragma clang fp contract(off)  // a scaled score is rounded once and feeds both max and exponent
  // lanes per row: D / 8 of them hold 8 dims each, inside an aligned group of LPR (a power of two)
  constexpr int LPR = HeadDim<D>::kRowGroup, kRowLanes = HeadDim<D>::kRowLanes;
  constexpr int kGroups = kFullThreads / LPR;
  constexpr int kPartial = partial_stride(D);
  __shared__ FullShared<D> sh;
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, grp = tid / LPR;
  // lanes of a group beyond the row's D / 8 compute on a zero query: they re-read
  // the first piece of the row and leave nothing behind
  const bool lane_on = tid % LPR < kRowLanes;
  const int gl = lane_on ? tid % LPR : 0;
  const int head0 = b * p.Hq + kvh * G;

  float qf[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    uint4 qv = *reinterpret_cast<const uint4*>(p.q + (int64_t)(head0 + g) * D + gl * 8);
    if (!lane_on) qv = make_uint4(0, 0, 0, 0);
    qf[g][0] = bf16_lo(qv.x); qf[g][1] = bf16_hi(qv.x); qf[g][2] = bf16_lo(qv.y); qf[g][3] = bf16_hi(qv.y);
    qf[g][4] = bf16_lo(qv.z); qf[g][5] = bf16_hi(qv.z); qf[g][6] = bf16_lo(qv.w); qf[g][7] = bf16_hi(qv.w);
  }
  const int L = safe_seq_len(p.seq_len, p.seq_start, b, p.max_seq_len, p.pool_tokens);
  const int t_begin = split * p.chunk, t_end = min(L, t_begin + p.chunk);
  const int64_t row0 = ((int64_t)kvh * p.pool_tokens + (L > 0 ? p.seq_start[b] : 0)) * D;
  const uint16_t* Kp = p.K + row0;
  const uint16_t* Vp = p.V + row0;

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNegBig;
    l[g] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[g][j] = 0.f;
  }

  constexpr int U = 4;
  for (int t0 = t_begin + grp; t0 < t_end; t0 += kGroups * U) {
    uint4 kv[U], vv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kGroups;
      ok[u] = t < t_end;
      // unconditional, clamped: all loads of the pass are in flight together
      const int64_t off = (int64_t)min(t, t_end - 1) * D + gl * 8;
      kv[u] = *reinterpret_cast<const uint4*>(Kp + off);
      vv[u] = *reinterpret_cast<const uint4*>(Vp + off);
    }
    float kf[U][8], vf[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      kf[u][0] = bf16_lo(kv[u].x); kf[u][1] = bf16_hi(kv[u].x); kf[u][2] = bf16_lo(kv[u].y); kf[u][3] = bf16_hi(kv[u].y);
      kf[u][4] = bf16_lo(kv[u].z); kf[u][5] = bf16_hi(kv[u].z); kf[u][6] = bf16_lo(kv[u].w); kf[u][7] = bf16_hi(kv[u].w);
      vf[u][0] = bf16_lo(vv[u].x); vf[u][1] = bf16_hi(vv[u].x); vf[u][2] = bf16_lo(vv[u].y); vf[u][3] = bf16_hi(vv[u].y);
      vf[u][4] = bf16_lo(vv[u].z); vf[u][5] = bf16_hi(vv[u].z); vf[u][6] = bf16_lo(vv[u].w); vf[u][7] = bf16_hi(vv[u].w);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float sc[U];
      float mn = m[g];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float s = qf[g][0] * kf[u][0];
#pragma unroll
        for (int j = 1; j < 8; ++j) s = fmaf(qf[g][j], kf[u][j], s);
        s = lanes_sum_f32<LPR>(s) * p.scale_log2e;
        sc[u] = ok[u] ? s : kNegBig;
        mn = fmaxf(mn, sc[u]);
      }
      const float corr = exp2f(m[g] - mn);
      m[g] = mn;
      l[g] *= corr;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[g][j] *= corr;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float pw = ok[u] ? exp2f(sc[u] - mn) : 0.f;
        l[g] += pw;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(pw, vf[u][j], acc[g][j]);
      }
    }
  }

  // Combine the 16 row groups, one query head at a time through the same LDS block.
#pragma unroll
  for (int g = 0; g < G; ++g) {
    if (tid % LPR == 0) {
      sh.m[grp] = m[g];
      sh.l[grp] = l[g];
    }
    if (lane_on) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sh.acc[grp][gl * 8 + j] = acc[g][j];
    }
    __syncthreads();
    if (tid < D) {
      float M = kNegBig, lsum = 0.f, o = 0.f;
      for (int r = 0; r < kGroups; ++r) M = fmaxf(M, sh.m[r]);
      for (int r = 0; r < kGroups; ++r) {
        const float w = exp2f(sh.m[r] - M);
        lsum = fmaf(sh.l[r], w, lsum);
        o = fmaf(sh.acc[r][tid], w, o);
      }
      float* mine = p.partial + ((int64_t)(head0 + g) * p.n_splits + split) * kPartial;
      if (tid == 0) {
        mine[0] = M;
        mine[1] = lsum;
      }
      mine[4 + tid] = o;
    }
    __syncthreads();
  }
}

// Merges the n_parts partials of one head into out.  Grid (Hq, B), kMergeThreads
// threads: the parts are cut into kMergeThreads / D contiguous slices, one
// thread per (slice, output dimension) reduces its slice with eight loads in
// flight, and the slices are combined through LDS.
constexpr int kMergeThreads = 512;

template <int D>
__global__ __launch_bounds__(kMergeThreads) void merge_parts_kernel(const float* __restrict__ partial,
                                                                    float* __restrict__ out, int Hq,
                                                                    int n_parts) {
  constexpr int kPartial = partial_stride(D);
  constexpr int S = kMergeThreads / D;  // slices
  __shared__ float s_m[S], s_l[S], s_o[S][D];
  const int64_t head = (int64_t)blockIdx.y * Hq + blockIdx.x;
  const int tid = threadIdx.x % D, slice = threadIdx.x / D;  // threads past S * D idle (D = 96, 160, 192)
  const float* ph = partial + head * n_parts * kPartial;
  const int per = (n_parts + S - 1) / S;
  const int begin = slice * per, end = min(n_parts, begin + per);  // may be empty
  float M = kNegBig;
  for (int s0 = begin; s0 < end; s0 += 8) {
    float pm[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) pm[u] = ph[(int64_t)min(s0 + u, end - 1) * kPartial];
#pragma unroll
    for (int u = 0; u < 8; ++u) M = fmaxf(M, pm[u]);
  }
  float lsum = 0.f, o = 0.f;
  for (int s0 = begin; s0 < end; s0 += 8) {
    float pm[8], pl[8], po[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float* ps = ph + (int64_t)min(s0 + u, end - 1) * kPartial;
      pm[u] = ps[0];
      pl[u] = ps[1];
      po[u] = ps[4 + tid];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool use = s0 + u < end;
      const float w = use ? exp2f(pm[u] - M) : 0.f;
      lsum = fmaf(use ? pl[u] : 0.f, w, lsum);
      o = fmaf(use ? po[u] : 0.f, w, o);
    }
  }
  if (slice < S) {
    if (tid == 0) {
      s_m[slice] = M;
      s_l[slice] = lsum;
    }
    s_o[slice][tid] = o;
  }
  __syncthreads();
  if (slice != 0) return;
  float Mh = kNegBig, lh = 0.f, oh = 0.f;
#pragma unroll
  for (int r = 0; r < S; ++r) Mh = fmaxf(Mh, s_m[r]);
#pragma unroll
  for (int r = 0; r < S; ++r) {
    const float w = exp2f(s_m[r] - Mh);  // an empty slice holds l = 0, o = 0
    lh = fmaf(s_l[r], w, lh);
    oh = fmaf(s_o[r][tid], w, oh);
  }
  out[head * D + tid] = lh > 0.f ? oh / lh : 0.f;
}

}  // namespace adamas
