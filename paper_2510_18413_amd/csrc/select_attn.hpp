// Top-k selection from the scan's distances and tile histograms (Algorithm 1
// line 6) and softmax attention over the selected rows (lines 7-8, Eq. 1).
//
// Selection without sorting.  Distances take 385 values, so the k-th smallest
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
// one-pass online softmax over them (16 lanes per row, 8 dims per lane, fp32),
// stores an (m, l, o[128]) partial; a small follow-up kernel merges the
// partials of a head in segment order into the output.  (A merge inside the
// same kernel would need device-scope fences, which on this part cost far more
// than a kernel boundary: each one walks the XCD's whole L2.)
#pragma once

#include "device_utils.hpp"

namespace adamas {

constexpr int kSelThreads = 256;
constexpr int kSelTokPerThread = 16;
constexpr int kSelPass = kSelThreads * kSelTokPerThread;  // tokens per pass
constexpr int kMaxK = 4096;
constexpr int kAttnGroups = kSelThreads / 16;
constexpr float kNegBig = -1.0e30f;

struct SelectParams {
  const uint16_t* dist;       // [B*Hq][dist_stride]
  int64_t dist_stride;
  const uint16_t* tilehist;   // [B*Hq][n_tiles][kHistStride]
  const int64_t* seq_start;   // [B]
  const int32_t* seq_len;     // [B]
  int32_t* idx_out;           // [B*Hq][k] or null
  const uint16_t* q;          // bf16 [B*Hq][128]
  const uint16_t* K;          // pools
  const uint16_t* V;
  float* out;                 // [B*Hq][128]
  float* partial;             // [B*Hq][n_parts][kPartialStride]
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, Hkv, k;
  int32_t n_tiles, tile_tokens, seg_len, n_parts;
  float scale_log2e;          // sm_scale * log2(e)
};

struct AttnShared {
  float m[kAttnGroups];
  float l[kAttnGroups];
  float acc[kAttnGroups][kHeadDim];
};

// Attention partial of this workgroup over the n rows listed in s_sel (token
// positions; Kp, Vp point at the sequence's first row of the right KV head):
// writes (m, l, o[128]) -- running maximum in the exp2 domain, sum of weights,
// unnormalised weighted sum of V -- to partial_head[part].
// All 256 threads must call it.
__device__ __forceinline__ void attention_partial(
    const int32_t* s_sel, int n, const uint16_t* __restrict__ q, const uint16_t* __restrict__ Kp,
    const uint16_t* __restrict__ Vp, float scale_log2e, float* __restrict__ partial_head,
    int part, AttnShared& sh) {
  const int tid = threadIdx.x, grp = tid >> 4, gl = tid & 15;

  float qf[8];
  {
    const uint4 qv = *reinterpret_cast<const uint4*>(q + gl * 8);
    qf[0] = bf16_lo(qv.x); qf[1] = bf16_hi(qv.x); qf[2] = bf16_lo(qv.y); qf[3] = bf16_hi(qv.y);
    qf[4] = bf16_lo(qv.z); qf[5] = bf16_hi(qv.z); qf[6] = bf16_lo(qv.w); qf[7] = bf16_hi(qv.w);
  }
  float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;

  constexpr int U = 4;  // rows in flight per 16-lane group
  for (int i0 = grp; i0 < n; i0 += kAttnGroups * U) {
    uint4 kv[U], vv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u * kAttnGroups;
      ok[u] = i < n;
      if (ok[u]) {
        const int64_t off = (int64_t)s_sel[i] * kHeadDim + gl * 8;
        kv[u] = *reinterpret_cast<const uint4*>(Kp + off);
        vv[u] = *reinterpret_cast<const uint4*>(Vp + off);
      } else {
        kv[u] = make_uint4(0, 0, 0, 0);
        vv[u] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float s = qf[0] * bf16_lo(kv[u].x);
      s = fmaf(qf[1], bf16_hi(kv[u].x), s);
      s = fmaf(qf[2], bf16_lo(kv[u].y), s);
      s = fmaf(qf[3], bf16_hi(kv[u].y), s);
      s = fmaf(qf[4], bf16_lo(kv[u].z), s);
      s = fmaf(qf[5], bf16_hi(kv[u].z), s);
      s = fmaf(qf[6], bf16_lo(kv[u].w), s);
      s = fmaf(qf[7], bf16_hi(kv[u].w), s);
      // the 16 lanes of a group sit in one wave: butterfly over lane bits 0..3
      s += __shfl_xor(s, 1, kWave);
      s += __shfl_xor(s, 2, kWave);
      s += __shfl_xor(s, 4, kWave);
      s += __shfl_xor(s, 8, kWave);
      if (ok[u]) {
        s *= scale_log2e;
        const float mn = fmaxf(m, s);
        const float corr = exp2f(m - mn), pw = exp2f(s - mn);
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
  }

  if (gl == 0) {
    sh.m[grp] = m;
    sh.l[grp] = l;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) sh.acc[grp][gl * 8 + j] = acc[j];
  __syncthreads();

  // Merge the 16 groups (fixed order), publish the workgroup's partial.
  if (tid < kHeadDim) {
    float M = kNegBig;
#pragma unroll
    for (int g = 0; g < kAttnGroups; ++g) M = fmaxf(M, sh.m[g]);
    float lsum = 0.f, o = 0.f;
#pragma unroll
    for (int g = 0; g < kAttnGroups; ++g) {
      const float w = exp2f(sh.m[g] - M);
      lsum = fmaf(sh.l[g], w, lsum);
      o = fmaf(sh.acc[g][tid], w, o);
    }
    float* mine = partial_head + (int64_t)part * kPartialStride;
    if (tid == 0) {
      mine[0] = M;
      mine[1] = lsum;
    }
    mine[4 + tid] = o;
  }
}

template <bool ATTN>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams p) {
  __shared__ uint32_t s_tot[448];
  __shared__ uint32_t s_scan[4];
  __shared__ int32_t s_T, s_cntlt;
  __shared__ uint32_t s_ltb, s_eqb;
  __shared__ int32_t s_sel[ATTN ? kMaxK : 1];
  __shared__ AttnShared s_attn;

  const int seg = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const int L = safe_seq_len(p.seq_len, p.seq_start, b, p.max_seq_len, p.pool_tokens);
  const int kk = min(p.k, L);
  const int n_active = max(1, (L + p.seg_len - 1) / p.seg_len);  // segments that hold tokens
  if (seg >= n_active) return;
  const int seg_t0 = seg * p.seg_len, seg_t1 = min(L, seg_t0 + p.seg_len);

  // Prefetch the first pass of this segment's distances.
  const uint16_t* drow = p.dist + head * p.dist_stride;
  uint4 da, db;
  {
    const int t = seg_t0 + tid * kSelTokPerThread;
    if (t < seg_t1) {
      const uint4* src = reinterpret_cast<const uint4*>(drow + t);
      da = src[0];
      db = src[1];
    } else {
      da = db = make_uint4(0, 0, 0, 0);
    }
  }

  // Head histogram (all tiles) and the part of it that lies before this segment.
  const int tiles_active = (L + p.tile_tokens - 1) / p.tile_tokens;
  const int first_tile = seg_t0 / p.tile_tokens;
  const uint16_t* hrow = p.tilehist + head * p.n_tiles * kHistStride;
  uint32_t tot0 = 0, tot1 = 0, pre0 = 0, pre1 = 0;
  const int bin0 = tid, bin1 = tid + kSelThreads;
  for (int tb = 0; tb < tiles_active; tb += 8) {
    uint32_t v0[8], v1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {  // all loads of the batch in flight together
      const int ti = tb + u;
      const bool in = ti < tiles_active;
      v0[u] = in ? hrow[(int64_t)ti * kHistStride + bin0] : 0u;
      v1[u] = (in && bin1 < kNumBins) ? hrow[(int64_t)ti * kHistStride + bin1] : 0u;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      tot0 += v0[u];
      tot1 += v1[u];
      if (tb + u < first_tile) {
        pre0 += v0[u];
        pre1 += v1[u];
      }
    }
  }
  s_tot[bin0] = tot0;
  if (bin1 < 448) s_tot[bin1] = tot1;
  if (tid == 0) {
    s_ltb = 0u;
    s_eqb = 0u;
    s_T = 0;
    s_cntlt = 0;
  }
  __syncthreads();

  // Threshold distance T and #{D < T}, by one wave: 7 bins per lane.
  if (tid < kWave) {
    uint32_t c[7], sum = 0;
#pragma unroll
    for (int j = 0; j < 7; ++j) {
      c[j] = s_tot[lane * 7 + j];
      sum += c[j];
    }
    const uint32_t incl = wave_incl_scan_u32(sum, lane);
    uint32_t run = incl - sum;
    if (kk > 0 && run < (uint32_t)kk && incl >= (uint32_t)kk) {
#pragma unroll
      for (int j = 0; j < 7; ++j) {
        if (run < (uint32_t)kk && run + c[j] >= (uint32_t)kk) {
          s_T = lane * 7 + j;
          s_cntlt = (int32_t)run;
        }
        run += c[j];
      }
    }
  }
  __syncthreads();
  const int T = s_T;
  const int r = kk - s_cntlt;  // ties at distance T to take, lowest positions first

  {
    uint32_t ltb = (bin0 < T ? pre0 : 0u) + (bin1 < T ? pre1 : 0u);
    uint32_t eqb = (bin0 == T ? pre0 : 0u) + (bin1 == T ? pre1 : 0u);
    ltb = wave_sum_u32(ltb);
    eqb = wave_sum_u32(eqb);
    if (lane == 0) {
      atomicAdd(&s_ltb, ltb);
      atomicAdd(&s_eqb, eqb);
    }
  }
  __syncthreads();
  uint32_t run_lt = s_ltb, run_eq = s_eqb;
  const uint32_t seg_pos0 = run_lt + min(run_eq, (uint32_t)r);
  int32_t* idx_row = p.idx_out != nullptr ? p.idx_out + head * p.k : nullptr;

  for (int pass_t0 = seg_t0; pass_t0 < seg_t1; pass_t0 += kSelPass) {
    const int t = pass_t0 + tid * kSelTokPerThread;
    if (pass_t0 != seg_t0) {
      if (t < seg_t1) {
        const uint4* src = reinterpret_cast<const uint4*>(drow + t);
        da = src[0];
        db = src[1];
      } else {
        da = db = make_uint4(0, 0, 0, 0);
      }
    }
    const uint32_t words[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
    uint32_t c_lt = 0, c_eq = 0;
#pragma unroll
    for (int j = 0; j < kSelTokPerThread; ++j) {
      const int d = (int)((words[j >> 1] >> ((j & 1) * 16)) & 0xffffu);
      const bool valid = t + j < seg_t1;
      c_lt += (valid && d < T) ? 1u : 0u;
      c_eq += (valid && d == T) ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t ex = block256_excl_scan(c_lt | (c_eq << 16), s_scan, total);
    uint32_t lt = run_lt + (ex & 0xffffu), eq = run_eq + (ex >> 16);
#pragma unroll
    for (int j = 0; j < kSelTokPerThread; ++j) {
      const int d = (int)((words[j >> 1] >> ((j & 1) * 16)) & 0xffffu);
      const bool valid = t + j < seg_t1;
      const bool is_lt = valid && d < T, is_eq = valid && d == T;
      if (is_lt || (is_eq && eq < (uint32_t)r)) {
        const uint32_t pos = lt + min(eq, (uint32_t)r);
        // pos < kk always holds for consistent histograms; the checks keep a
        // corrupted workspace from turning into an out-of-bounds store.
        if (pos < (uint32_t)kk) {
          if (idx_row != nullptr) idx_row[pos] = t + j;
          if (ATTN && pos - seg_pos0 < (uint32_t)kMaxK) s_sel[pos - seg_pos0] = t + j;
        }
      }
      lt += is_lt ? 1u : 0u;
      eq += is_eq ? 1u : 0u;
    }
    run_lt += total & 0xffffu;
    run_eq += total >> 16;
  }
  if (seg == 0 && idx_row != nullptr)
    for (int i = kk + tid; i < p.k; i += kSelThreads) idx_row[i] = -1;

  if (ATTN) {
    const int n_sel = min((int)(run_lt + min(run_eq, (uint32_t)r) - seg_pos0), kk);
    __syncthreads();  // s_sel complete
    const int kvh = hq / (p.Hq / p.Hkv);
    const int64_t row0 = ((int64_t)kvh * p.pool_tokens + p.seq_start[b]) * kHeadDim;
    attention_partial(s_sel, n_sel, p.q + head * kHeadDim, p.K + row0, p.V + row0, p.scale_log2e,
                      p.partial + head * p.n_parts * kPartialStride, seg, s_attn);
  }
}

// ---------------------------------------------------------------- stand-alone attention

struct AttnParams {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  const int64_t* seq_start;
  const int32_t* idx;  // [B*Hq][k]
  float* out;
  float* partial;      // [B*Hq][n_parts][kPartialStride]
  int64_t pool_tokens;
  int32_t Hq, Hkv, k, n_parts, chunk;  // chunk = idx entries per workgroup
  float scale_log2e;
};

__global__ __launch_bounds__(kSelThreads) void sparse_attn_kernel(const AttnParams p) {
  __shared__ int32_t s_sel[kMaxK];
  __shared__ uint32_t s_scan[4];
  __shared__ AttnShared s_attn;
  const int part = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int64_t head = (int64_t)b * p.Hq + hq;
  const int i0 = part * p.chunk, i1 = min(p.k, i0 + p.chunk);
  const int32_t* idx_row = p.idx + head * p.k;
  const int64_t start = p.seq_start[b];
  // Order-preserving compaction of the usable entries of this chunk: negative
  // entries are padding; an entry that would leave the pool is dropped too.
  uint32_t n = 0;
  for (int base = i0; base < i1; base += kSelThreads) {
    const int i = base + tid;
    const int32_t tok = i < i1 ? idx_row[i] : -1;
    const bool use = tok >= 0 && start >= 0 && start + tok < p.pool_tokens;
    uint32_t total;
    const uint32_t ex = block256_excl_scan(use ? 1u : 0u, s_scan, total);
    if (use) s_sel[n + ex] = tok;
    n += total;
  }
  __syncthreads();
  const int kvh = hq / (p.Hq / p.Hkv);
  const int64_t row0 = ((int64_t)kvh * p.pool_tokens + start) * kHeadDim;
  attention_partial(s_sel, (int)n, p.q + head * kHeadDim, p.K + row0, p.V + row0, p.scale_log2e,
                    p.partial + head * p.n_parts * kPartialStride, part, s_attn);
}

// Merges the attention partials of one head, in part order, into out.
// seg_len > 0: the number of partials is the number of segments that hold
// tokens of the head's sequence (as select_kernel wrote them); seg_len == 0:
// n_parts partials (as sparse_attn_kernel wrote them).
struct MergeParams {
  const float* partial;      // [B*Hq][n_parts][kPartialStride]
  float* out;                // [B*Hq][128]
  const int64_t* seq_start;
  const int32_t* seq_len;
  int64_t pool_tokens, max_seq_len;
  int32_t Hq, n_parts, seg_len;
};

__global__ __launch_bounds__(kHeadDim) void merge_kernel(const MergeParams p) {
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int64_t head = (int64_t)b * p.Hq + hq;
  int n = p.n_parts;
  if (p.seg_len > 0) {
    const int L = safe_seq_len(p.seq_len, p.seq_start, b, p.max_seq_len, p.pool_tokens);
    n = max(1, (L + p.seg_len - 1) / p.seg_len);
  }
  const float* ph = p.partial + head * p.n_parts * kPartialStride;
  float M = kNegBig;
  for (int s = 0; s < n; ++s) M = fmaxf(M, ph[(int64_t)s * kPartialStride]);
  float lsum = 0.f, o = 0.f;
  for (int s = 0; s < n; ++s) {
    const float* ps = ph + (int64_t)s * kPartialStride;
    const float w = exp2f(ps[0] - M);
    lsum = fmaf(ps[1], w, lsum);
    o = fmaf(ps[4 + tid], w, o);
  }
  p.out[head * kHeadDim + tid] = lsum > 0.f ? o / lsum : 0.f;
}

}  // namespace adamas
