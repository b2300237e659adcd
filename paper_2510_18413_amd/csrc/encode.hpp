// Hadamard transform (Eq. 4) + bucketize (Eq. 5) + 2-bit pack of one 128-d
// bf16 vector by one wavefront, and the bulk key / query encode kernels
// (Algorithm 1, transform / bucketize / compress steps).
#pragma once

#include <utility>

#include "device_utils.hpp"

namespace adamas {

// Thresholds as the kernels compare against them: multiplied by sqrt(128)
// when the vector is transformed (the kernels form the unnormalised +-1 sums),
// as given for the ablation without the transform (Section 4.4), which applies
// Eq. 5 to the raw vector (transform == 0).
struct Thresholds {
  double tau[7];  // 2^BITS - 1 used
  int transform;
  // For the bulk encode's single-precision attempt (see encode_rows_kernel):
  // tau rounded to float, an upper bound of max |tau32[i] - tau[i]|, and
  // whether that attempt may be made at all (it needs every tau32[i] to keep
  // the sign of tau[i], zero included).
  float tau32[7];
  float dtau;
  int fast;
  // Two-bit codes whose thresholds are (-t, 0, t) with t > 0, exactly: the
  // attempt then compares |y| with t and reads the sign of y.
  int symmetric;
};

// Bit planes of the bucket index c = #{i : y > tau_i} from the nested indicator
// masks m_1 >= m_2 >= ... of Eq. 5 (bit j of m_i: coefficient j exceeds tau_i):
// the lowest plane is the parity of all masks, the highest is the middle mask.
template <int BITS, typename M>
__device__ __forceinline__ void planes_from_masks(const M* m, M* plane) {
  if constexpr (BITS == 1) {
    plane[0] = m[0];
  } else if constexpr (BITS == 2) {
    plane[0] = m[0] ^ m[1] ^ m[2];
    plane[1] = m[1];
  } else {
    plane[0] = m[0] ^ m[1] ^ m[2] ^ m[3] ^ m[4] ^ m[5] ^ m[6];
    plane[1] = m[1] ^ m[3] ^ m[5];
    plane[2] = m[3];
  }
}

// One wave64 encodes one vector of D elements.  Lane l holds x[l + 64e] for
// e < D / 64; the butterflies over index bits 6 and up are lane-local, bits
// 0..5 go across lanes.  All sums are fp64 and exact for inputs within the
// documented exponent spread, so the stage order does not influence the result.
// Result: w[p][g], plane p of word g of the packed row, identical in every lane.
// All 64 lanes must be active.  The elements come already loaded (raw bf16
// bits), so that a caller can issue that load ahead of other memory traffic.
// ---- D = 2^n * m, m = 12 or 20 (Section 2: H_D = H_{2^n} (x) H_m) ------------
//
// H_m is Paley's matrix for the prime q = m - 1 (the paper names no H_12 / H_20):
//   P[0][c] = 1,  P[r][0] = -1 (r >= 1),  P[r][r] = 1,
//   P[r][c] = +1 if r - c is a non-zero square mod q, else -1   (r != c; r, c >= 1).
// Bit r of paley_neg_column(m, c) is set where P[r][c] = -1: the signs of the
// inputs in output coefficient c of y = x P.
constexpr bool paley_is_square(int q, int a) {
  for (int t = 1; t < q; ++t)
    if ((t * t) % q == a) return true;
  return false;
}
constexpr uint32_t paley_neg_column(int m, int c) {
  const int q = m - 1;
  uint32_t neg = 0;
  for (int r = 1; r < m; ++r) {
    bool minus = false;
    if (c == 0) minus = true;
    else if (r == c) minus = false;
    else minus = !paley_is_square(q, (((r - c) % q) + q) % q);
    if (minus) neg |= 1u << r;
  }
  return neg;
}

// The sign masks as compile-time constants (a call of paley_neg_column in device
// code with a loop variable as argument leaves its loops and remainders to run
// time when m = 20): kPaleyNeg<M, C>, and a loop whose index is a constant
// expression to name them with.
template <int M, int C>
inline constexpr uint32_t kPaleyNeg = paley_neg_column(M, C);
template <typename F, int... I>
__device__ __forceinline__ void static_for_each(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_each(f, std::make_integer_sequence<int, N>{});
}

template <int CTRL>
__device__ __forceinline__ double quad_bcast_f64(double v) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)b, CTRL, 0xf, 0xf, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, true);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// One wave64 encodes one vector of D = 2^n * m elements.  Lane l < 4 * 2^n holds
// the m / 4 consecutive elements from l * m / 4 on (raw bf16 bits; lanes beyond
// hold nothing), so that a quad of lanes holds one block of m: the m-point stage
// gathers the quad's values with DPP broadcasts and forms the lane's own m / 4
// outputs as signed sums; the 2^n stage is butterflies across lane bits 2 and up.
// All sums are fp64 and exact for inputs within the documented exponent spread.
// The bucket indices then move to the lanes that own their bit of the packed
// row (coefficient 64 k + l to lane l) and wave ballots give the planes.
// Result: w[p][g], plane p of word g, identical in every lane.  All 64 lanes active.
template <int BITS, int D>
__device__ __forceinline__ void encode_values_wave_kron(const uint32_t (&raw)[HeadDim<D>::kEncElems],
                                                        const Thresholds& thr,
                                                        uint32_t w[BITS][D / 32]) {
  constexpr int T = (1 << BITS) - 1, M = HeadDim<D>::kBase, E = M / 4;
  constexpr int kLanes = HeadDim<D>::kEncLanes;
  const int lane = threadIdx.x & 63, c4 = lane & 3;
  double v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) v[e] = lane < kLanes ? (double)bf16_bits_to_float(raw[e]) : 0.0;
  if (thr.transform) {
    // the quad's block of m inputs, in element order
    double xs[M];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      xs[0 * E + e] = quad_bcast_f64<0x00>(v[e]);
      xs[1 * E + e] = quad_bcast_f64<0x55>(v[e]);
      xs[2 * E + e] = quad_bcast_f64<0xAA>(v[e]);
      xs[3 * E + e] = quad_bcast_f64<0xFF>(v[e]);
    }
    double out[E];
    static_for<E>([&](auto e_) {
      constexpr int e = decltype(e_)::value;
      // signs of output coefficient c4 * E + e of the block
      const uint32_t neg = c4 == 0 ? kPaleyNeg<M, 0 * E + e>
                         : c4 == 1 ? kPaleyNeg<M, 1 * E + e>
                         : c4 == 2 ? kPaleyNeg<M, 2 * E + e>
                                   : kPaleyNeg<M, 3 * E + e>;
      double acc = 0.0;
#pragma unroll
      for (int r = 0; r < M; ++r) {
        const uint64_t flip = (uint64_t)((neg >> r) & 1u) << 63;
        acc += __builtin_bit_cast(double, __builtin_bit_cast(uint64_t, xs[r]) ^ flip);
      }
      out[e] = acc;
    });
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = out[e];
#pragma unroll
    for (int h = 4; h < kLanes; h <<= 1) {  // index bits of the 2^n factor: across lanes
      const bool upper = (lane & h) != 0;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const double partner = __shfl_xor(v[e], h, kWave);
        v[e] = upper ? partner - v[e] : v[e] + partner;
      }
    }
  }
  // bucket indices of the lane's coefficients, three bits each
  uint32_t packed = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < T; ++i) c += v[e] > thr.tau[i] ? 1u : 0u;
    packed |= c << (3 * e);
  }
#pragma unroll
  for (int k = 0; k < (D + 63) / 64; ++k) {
    const int coef = 64 * k + lane;  // lives in lane coef / E as element coef % E
    const uint32_t from = (uint32_t)__shfl((int)packed, coef / E, kWave);
    const uint32_t c = coef < D ? (from >> (3 * (coef % E))) & 7u : 0u;
#pragma unroll
    for (int p = 0; p < BITS; ++p) {
      const uint64_t plane = __ballot((c >> p) & 1u);
      w[p][2 * k] = (uint32_t)plane;
      if (2 * k + 1 < D / 32) w[p][2 * k + 1] = (uint32_t)(plane >> 32);
    }
  }
}

template <int BITS, int D>
__device__ __forceinline__ void encode_values_wave(const uint32_t (&raw)[HeadDim<D>::kEncElems],
                                                   const Thresholds& thr,
                                                   uint32_t w[BITS][D / 32]) {
  if constexpr (!HeadDim<D>::kPow2) {
    encode_values_wave_kron<BITS, D>(raw, thr, w);
    return;
  } else {
  constexpr int T = (1 << BITS) - 1, E = D / 64;
  const int lane = threadIdx.x & 63;
  double v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) v[e] = (double)bf16_bits_to_float(raw[e]);
  if (thr.transform) {
#pragma unroll
    for (int h = 1; h < E; h <<= 1) {  // index bits 6.. : inside the lane
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if ((e & h) == 0) {
          const double a = v[e], b = v[e + h];
          v[e] = a + b;
          v[e + h] = a - b;
        }
      }
    }
#pragma unroll
    for (int h = 1; h < 64; h <<= 1) {  // index bits 0..5: across the wave
      const bool upper = (lane & h) != 0;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const double partner = __shfl_xor(v[e], h, kWave);
        v[e] = upper ? partner - v[e] : v[e] + partner;
      }
    }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    uint64_t m[T], plane[BITS];
#pragma unroll
    for (int i = 0; i < T; ++i) m[i] = __ballot(v[e] > thr.tau[i]);
    planes_from_masks<BITS>(m, plane);
#pragma unroll
    for (int p = 0; p < BITS; ++p) {
      w[p][2 * e] = (uint32_t)plane[p];
      w[p][2 * e + 1] = (uint32_t)(plane[p] >> 32);
    }
  }
  }  // power of two
}

// ---- bulk encode: D / 32 lanes per vector ---------------------------------
//
// Lane j of a group holds elements 32j .. 32j+31 of one vector, so five
// butterfly stages are register-to-register and only the index bits from 5 up
// cross lanes (two stages at D = 128, by DPP quad permutes).  After the
// transform lane j holds coefficients 32j .. 32j+31, which is exactly word j of
// the packed row: every lane assembles and stores its own word.  At D = 128 a
// wave encodes 16 vectors and moves 4 KiB in, 512 B out, both contiguous.
//
// The codes are defined on the exact sums.  The four-lane routine works in
// fp32 and certifies its own result (below); the few vectors it cannot certify
// are redone in fp64 by the whole wave with encode_values_wave, one at a time.

// ---- bulk encode, single-precision attempt with a certified guard ----------
//
// The same butterflies in fp32.  An fp32 sum is rounded, so its comparison with
// a threshold can come out wrong -- but only when the sum is close to the
// threshold: every coefficient goes through log2(D) additions, hence
//   |y_fp32 - y_exact| <= gamma * sum_i |x_i|,  gamma = n u / (1 - n u),
//   n = log2(D), u = 2^-24
// (additions in fp32 never lose anything to underflow, and no partial sum
// exceeds sum |x_i|, which is checked to be far from overflow).  If every
// coefficient of a vector is further than that bound (plus the rounding of
// the threshold itself to fp32) from every threshold, all its comparisons are
// those of the exact sums and the fp32 masks are returned as certified;
// otherwise the caller has the vector redone exactly.  A vector of zeros has
// exact sums by itself.  Returns the same verdict in all lanes of the group.
__device__ __forceinline__ float dpp_quad_xor_f32(float v, bool xor2) {
  const int b = __float_as_int(v);
  return __int_as_float(xor2 ? __builtin_amdgcn_mov_dpp(b, kDppQuadXor2, 0xf, 0xf, true)
                             : __builtin_amdgcn_mov_dpp(b, kDppQuadXor1, 0xf, 0xf, true));
}

// Exchange with the lane whose index inside the vector's lane group differs in bit s.
__device__ __forceinline__ float group_xor_f32(float v, int s) {
  return s < 2 ? dpp_quad_xor_f32(v, s == 1) : __shfl_xor(v, 1 << s, kWave);
}

// The comparisons of Eq. 5 on the lane's N single-precision coefficients x, and the
// certificate: m[i] gets bit e set where x[e] > tau_i; the return value says whether
// every coefficient of the vector (all LPV lanes of its group) is further from every
// threshold than guard_per_abs * sum |x_i| (+ the rounding of the thresholds), i.e.
// whether the masks are those of the exact sums.  sum_abs: this lane's share of sum |x_i|.
template <int BITS, int N, int LPV, bool TRANSFORM>
__device__ __forceinline__ bool certified_masks(const float (&x)[N], float sum_abs, const Thresholds& thr,
                                                float guard_per_abs, uint32_t (&m)[(1 << BITS) - 1]) {
  constexpr int T = (1 << BITS) - 1;
  constexpr uint32_t kAll = N == 32 ? 0xffffffffu : (1u << (N & 31)) - 1u;
  float nearest = 3.0e38f;  // smallest |coefficient - threshold| of the vector
  if constexpr (BITS == 2) {
    if (thr.symmetric) {
      // Thresholds (-t, 0, t): with u = |y| - t the distances to the thresholds are
      // |u| and |y|, and away from the thresholds y > 0 is the cleared sign of y,
      // y > -t is "y > 0 or u < 0", y > t is "y > 0 and not u < 0".  A coefficient
      // on a threshold (y = 0 of either sign included) has distance 0 and is never
      // certified, so the signs of the zeros do not matter; a vector of zeros has
      // code 1 everywhere.
      uint32_t neg_y = 0, neg_u = 0;
#pragma unroll
      for (int e = N - 1; e >= 0; --e) {
        const float u = fabsf(x[e]) - thr.tau32[2];
        asm("v_alignbit_b32 %0, %1, %2, 31" : "=v"(neg_y) : "v"(neg_y), "v"(x[e]));
        asm("v_alignbit_b32 %0, %1, %2, 31" : "=v"(neg_u) : "v"(neg_u), "v"(u));
        // one instruction; a NaN would be skipped here but makes sum_abs fail its test below
        asm("v_min3_f32 %0, %1, |%2|, |%3|" : "=v"(nearest) : "v"(nearest), "v"(u), "v"(x[e]));
      }
#pragma unroll
      for (int s = 0; (1 << s) < LPV; ++s) {
        sum_abs += group_xor_f32(sum_abs, s);
        nearest = fminf(nearest, group_xor_f32(nearest, s));
      }
      const bool zeros = sum_abs == 0.f;
      m[0] = zeros ? kAll : ((~neg_y | neg_u) & kAll);
      m[1] = zeros ? 0u : (~neg_y & kAll);
      m[2] = zeros ? 0u : (~neg_y & ~neg_u & kAll);
      const float guard = (TRANSFORM ? sum_abs * guard_per_abs : 0.f) + thr.dtau;
      return sum_abs < 1.0e30f && (nearest > guard || zeros);
    }
  }
#pragma unroll
  for (int i = 0; i < T; ++i) m[i] = 0;
#pragma unroll
  for (int e = N - 1; e >= 0; --e) {
#pragma unroll
    for (int i = 0; i < T; ++i) {
      const float d = thr.tau32[i] - x[e];  // the sign of a difference is exact; +0 when equal
      // (m << 1) | sign(d); as an opaque instruction, or the compiler rebuilds the
      // chain as a tree over all the differences and runs out of registers
      asm("v_alignbit_b32 %0, %1, %2, 31" : "=v"(m[i]) : "v"(m[i]), "v"(d));
      nearest = fminf(nearest, fabsf(d));
    }
  }
  // over the lanes of the group
#pragma unroll
  for (int s = 0; (1 << s) < LPV; ++s) {
    sum_abs += group_xor_f32(sum_abs, s);
    nearest = fminf(nearest, group_xor_f32(nearest, s));
  }
  // Without the transform the "sums" are the elements themselves: exact.
  const float guard = (TRANSFORM ? sum_abs * guard_per_abs : 0.f) + thr.dtau;
  return sum_abs < 1.0e30f && (nearest > guard || guard == 0.f || sum_abs == 0.f);
}

// Butterflies across the LPV lanes of a vector's group (index bits above the lane's own elements).
template <int N, int LPV>
__device__ __forceinline__ void cross_lane_stages(float (&x)[N], int j) {
#pragma unroll
  for (int s = 0; (1 << s) < LPV; ++s) {
    const uint32_t sign_flip = ((j >> s) & 1) != 0 ? 0x80000000u : 0u;
#pragma unroll
    for (int i = 0; i < N; ++i)
      x[i] = __int_as_float(__float_as_int(x[i]) ^ (int)sign_flip) + group_xor_f32(x[i], s);
  }
}

template <int BITS, int D, bool TRANSFORM>
__device__ __forceinline__ bool encode_part_fast_as(const uint4 (&raw)[4], const Thresholds& thr, int j,
                                                    uint32_t (&m)[(1 << BITS) - 1]) {
  constexpr int LPV = D / 32;
  constexpr int kStages = D == 64 ? 6 : D == 128 ? 7 : 8;
  // gamma with a margin of 1.5 u for the rounding of sum |x_i|, of the guard
  // itself and of the differences compared with it
  constexpr float kGuard = (float)((kStages + 1.5) * 5.9604644775390625e-8);
  float x[32];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[i * 8 + 2 * e] = bf16_lo(w[e]);
      x[i * 8 + 2 * e + 1] = bf16_hi(w[e]);
    }
  }
  float sum_abs = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) sum_abs += fabsf(x[i]);
  if constexpr (TRANSFORM) {
#pragma unroll
    for (int h = 1; h < 32; h <<= 1) {
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        if ((i & h) == 0) {
          const float a = x[i], b = x[i + h];
          x[i] = a + b;
          x[i + h] = a - b;
        }
      }
    }
    cross_lane_stages<32, LPV>(x, j);
  }
  return certified_masks<BITS, 32, LPV, TRANSFORM>(x, sum_abs, thr, kGuard, m);
}

// The same attempt for D = 2^n * m (m = 12, 20): lane j of a group of 2^n holds block j of the
// vector, its m consecutive elements (raw: m / 2 words of two bf16 values).  The m-point stage
// y_c = sum_r x_r P[r][c] of Paley's matrix runs in the lane:
//   y_0 = x_0 - S,  y_c = (x_0 - S) + 2 (x_c + A_c),  S = x_1 + ... + x_q,
//   A_c = sum of the x_r (r >= 1, r != c) with r - c a non-zero square mod q = m - 1,
// then the butterflies over the 2^n blocks cross the lanes.  A value passes through at most
// m + n additions (the multiplication by two is exact).
template <int BITS, int D, bool TRANSFORM>
__device__ __forceinline__ bool encode_block_fast_as(const uint32_t (&raw)[HeadDim<D>::kBase / 2],
                                                     const Thresholds& thr, int j,
                                                     uint32_t (&m)[(1 << BITS) - 1]) {
  constexpr int M = HeadDim<D>::kBase, Q = M - 1, LPV = D / M;
  constexpr int kLog = LPV == 4 ? 2 : LPV == 8 ? 3 : 4;
  constexpr float kGuard = (float)((M + kLog + 1.5) * 5.9604644775390625e-8);
  float x[M];
#pragma unroll
  for (int i = 0; i < M / 2; ++i) {
    x[2 * i] = bf16_lo(raw[i]);
    x[2 * i + 1] = bf16_hi(raw[i]);
  }
  float sum_abs = 0.f;
#pragma unroll
  for (int i = 0; i < M; ++i) sum_abs += fabsf(x[i]);
  if constexpr (TRANSFORM) {
    float S = x[1];
#pragma unroll
    for (int r = 2; r < M; ++r) S += x[r];
    const float base = x[0] - S;
    float y[M];
    y[0] = base;
    static_for<Q>([&](auto c_) {
      constexpr int c = decltype(c_)::value + 1;  // 1 .. q
      float a = x[c];
      static_for<Q - 1>([&](auto s_) {
        constexpr int sq = decltype(s_)::value + 1;  // difference r - c mod q, 1 .. q - 1
        if constexpr (paley_is_square(Q, sq)) a += x[(c - 1 + sq) % Q + 1];
      });
      y[c] = base + 2.0f * a;
    });
#pragma unroll
    for (int i = 0; i < M; ++i) x[i] = y[i];
    cross_lane_stages<M, LPV>(x, j);
  }
  return certified_masks<BITS, M, LPV, TRANSFORM>(x, sum_abs, thr, kGuard, m);
}

// Division of a 32-bit index by a divisor fixed at launch (Granlund and
// Montgomery's round-up method): with l = ceil(log2 d) and
// m = floor(2^32 (2^l - d) / d) + 1,  n / d = (t + ((n - t) >> min(l, 1))) >> max(l - 1, 0),
// t = mulhi(m, n), for every n below 2^32.
struct Divisor32 {
  uint32_t mul, sh1, sh2;
  static Divisor32 of(uint32_t d) {  // host side; d >= 1
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;
    Divisor32 r;
    r.mul = (uint32_t)(((((uint64_t)1 << l) - d) << 32) / d + 1);
    r.sh1 = l < 1 ? l : 1;
    r.sh2 = l < 1 ? 0 : l - 1;
    return r;
  }
  __device__ __forceinline__ uint32_t quotient(uint32_t n) const {
    const uint32_t t = __umulhi(mul, n);
    return (t + ((n - t) >> sh1)) >> sh2;
  }
};

// With or without the transform (Section 4.4's ablation bucketizes the raw
// vector): two copies of the routine under one wave-uniform branch, so that
// neither carries the other's register moves.
template <int BITS, int D>
__device__ __forceinline__ bool encode_part_fast(const uint4 (&raw)[4], const Thresholds& thr, int j,
                                                 uint32_t (&m)[(1 << BITS) - 1]) {
  if (thr.transform) return encode_part_fast_as<BITS, D, true>(raw, thr, j, m);
  return encode_part_fast_as<BITS, D, false>(raw, thr, j, m);
}

template <int BITS, int D>
__device__ __forceinline__ bool encode_block_fast(const uint32_t (&raw)[HeadDim<D>::kBase / 2],
                                                  const Thresholds& thr, int j,
                                                  uint32_t (&m)[(1 << BITS) - 1]) {
  if (thr.transform) return encode_block_fast_as<BITS, D, true>(raw, thr, j, m);
  return encode_block_fast_as<BITS, D, false>(raw, thr, j, m);
}

__device__ __forceinline__ uint32_t group_xor_u32(uint32_t v, int s) {
  return __float_as_uint(group_xor_f32(__uint_as_float(v), s));
}

// Vector v of n_vec = n_heads * n_rows lives at
// src + (head * head_stride_rows + row_begin + r) * D, head = v / n_rows,
// r = v % n_rows; its code row goes to the same row of dst (D / 8 * BITS byte rows).
// A vector is encoded by a group of LPV lanes: D / 32 lanes with 32 elements each for a power
// of two, 2^n lanes with one block of m elements each for D = 2^n * m (m = 12, 20).
template <int BITS, int D>
__global__ __launch_bounds__(256) void encode_rows_kernel(const uint16_t* __restrict__ src,
                                                          uint8_t* __restrict__ dst,
                                                          int64_t head_stride_rows,
                                                          int64_t row_begin, int64_t n_rows,
                                                          int64_t n_vec, Thresholds thr,
                                                          Divisor32 by_rows) {
  constexpr int W = D / 32, E = HeadDim<D>::kEncElems;
  constexpr int kRowBytes = W * 4 * BITS;
  constexpr bool kPow2 = HeadDim<D>::kPow2;
  constexpr int M = HeadDim<D>::kBase;          // 12 or 20 (unused for a power of two)
  constexpr int LPV = kPow2 ? D / 32 : D / M;   // lanes per vector: 2, 4, 8 or 16
  constexpr int T = (1 << BITS) - 1;
  const int lane = threadIdx.x & 63;
  const int j = threadIdx.x & (LPV - 1);  // which part of the vector
  const int64_t quad = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / LPV;
  const int64_t n_quads = ((int64_t)gridDim.x * blockDim.x) / LPV;
  // All 64 lanes of a wave stay in the loop as long as its first group has a
  // vector (the groups of a wave take consecutive vectors), because the exact
  // redo below needs the whole wave.
  for (int64_t v = quad; __builtin_amdgcn_readfirstlane((int)(v < n_vec)) != 0; v += n_quads) {
    const bool valid = v < n_vec;
    int64_t row = 0;
    bool certified = true;
    // Eq. 5 on the lane's coefficients: nested indicator masks (bit e: coefficient e of the lane)
    uint32_t m[T];
#pragma unroll
    for (int i = 0; i < T; ++i) m[i] = 0u;
    if (valid) {
      // by_rows divides by n_rows; built by the launcher when n_vec fits 32 bits (mul = 0 otherwise; a divisor's mul is never 0)
      const int64_t head = by_rows.mul != 0u ? (int64_t)by_rows.quotient((uint32_t)v) : v / n_rows;
      const int64_t r = v - head * n_rows;
      row = head * head_stride_rows + row_begin + r;
      if constexpr (kPow2) {
        const uint4* in = reinterpret_cast<const uint4*>(src + row * D + j * 32);
        uint4 raw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) raw[i] = in[i];
        certified = encode_part_fast<BITS, D>(raw, thr, j, m) && thr.fast != 0;
      } else {
        // m bf16 values = m / 4 pieces of 8 bytes (rows and blocks are multiples of 8 bytes)
        const uint2* in = reinterpret_cast<const uint2*>(src + row * D + j * M);
        uint32_t raw[M / 2];
#pragma unroll
        for (int i = 0; i < M / 4; ++i) {
          const uint2 piece = in[i];
          raw[2 * i] = piece.x;
          raw[2 * i + 1] = piece.y;
        }
        certified = encode_block_fast<BITS, D>(raw, thr, j, m) && thr.fast != 0;
      }
    }
    uint32_t plane[BITS];
    planes_from_masks<BITS>(m, plane);
    if constexpr (kPow2) {
      // lane j holds coefficients 32 j .. 32 j + 31 = word j of the row
      if (valid && certified) {
        uint32_t* out = reinterpret_cast<uint32_t*>(dst + row * kRowBytes + j * (4 * BITS));
        if constexpr (BITS == 2) {
          *reinterpret_cast<uint2*>(out) = make_uint2(plane[0], plane[1]);
        } else {
#pragma unroll
          for (int p = 0; p < BITS; ++p) out[p] = plane[p];
        }
      }
    } else {
      // Lane j holds the m bits of coefficients j m .. j m + m - 1 of each plane: they go to bit
      // (j m) % 32 of word (j m) / 32 and may run over into the next word.  Every lane places
      // its bits in a row of zeros; an OR across the group's lanes (all lanes of the wave take
      // part in the exchanges, groups do not mix) leaves the whole row in every lane, and lane
      // wd < W stores word wd.
      const int at = j * M, w0 = at >> 5, sh = at & 31;
      uint32_t words[BITS][W];
#pragma unroll
      for (int p = 0; p < BITS; ++p) {
        const uint32_t lo = plane[p] << sh, hi = sh != 0 ? plane[p] >> (32 - sh) : 0u;
#pragma unroll
        for (int wd = 0; wd < W; ++wd) words[p][wd] = (wd == w0 ? lo : 0u) | (wd == w0 + 1 ? hi : 0u);
      }
#pragma unroll
      for (int st = 0; (1 << st) < LPV; ++st) {
#pragma unroll
        for (int p = 0; p < BITS; ++p) {
#pragma unroll
          for (int wd = 0; wd < W; ++wd) words[p][wd] |= group_xor_u32(words[p][wd], st);
        }
      }
      if (valid && certified) {
        uint32_t* out = reinterpret_cast<uint32_t*>(dst + row * kRowBytes);
#pragma unroll
        for (int wd = 0; wd < W; ++wd) {
          if (j == wd) {
#pragma unroll
            for (int p = 0; p < BITS; ++p) out[BITS * wd + p] = words[p][wd];
          }
        }
      }
    }
    // Vectors without a certificate: the whole wave redoes them exactly, one
    // after the other (wave-uniform loop over the first lanes of their groups).
    uint64_t pending = __ballot(valid && !certified && j == 0);
    while (pending != 0) {
      const int leader = __builtin_ctzll(pending);
      pending &= pending - 1;
      const uint32_t row_lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)row, leader);
      const uint32_t row_hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)row >> 32), leader);
      const int64_t vrow = (int64_t)(((uint64_t)row_hi << 32) | row_lo);
      uint32_t rawv[E];
#pragma unroll
      for (int e = 0; e < E; ++e)
        rawv[e] = lane < HeadDim<D>::kEncLanes ? src[vrow * D + HeadDim<D>::enc_index(lane, e)] : 0u;
      uint32_t w[BITS][W];
      encode_values_wave<BITS, D>(rawv, thr, w);
      uint32_t* out = reinterpret_cast<uint32_t*>(dst + vrow * kRowBytes);
#pragma unroll
      for (int wd = 0; wd < W; ++wd) {
        if (lane == wd) {  // lane wd stores word wd (every lane holds the whole row)
#pragma unroll
          for (int p = 0; p < BITS; ++p) out[BITS * wd + p] = w[p][wd];
        }
      }
    }
  }
}

}  // namespace adamas
