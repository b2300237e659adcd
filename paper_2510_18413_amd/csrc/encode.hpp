// Hadamard transform (Eq. 4) + bucketize (Eq. 5) + 2-bit pack of one 128-d
// bf16 vector by one wavefront, and the bulk key / query encode kernels
// (Algorithm 1, transform / bucketize / compress steps).
#pragma once

#include "device_utils.hpp"

namespace adamas {

// Thresholds as the kernels compare against them: multiplied by sqrt(128)
// when the vector is transformed (the kernels form the unnormalised +-1 sums),
// as given for the ablation without the transform (Section 4.4), which applies
// Eq. 5 to the raw vector (transform == 0).
struct Thresholds {
  double tau[7];  // 2^BITS - 1 used
  int transform;
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
template <int BITS, int D>
__device__ __forceinline__ void encode_values_wave(const uint32_t (&raw)[D / 64],
                                                   const Thresholds& thr,
                                                   uint32_t w[BITS][D / 32]) {
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
}

// ---- bulk encode: D / 32 lanes per vector ---------------------------------
//
// Lane j of a group holds elements 32j .. 32j+31 of one vector as doubles, so
// five butterfly stages are register-to-register and only the index bits from 5
// up cross lanes (two stages at D = 128, by DPP quad permutes).  After the
// transform lane j holds coefficients 32j .. 32j+31, which is exactly word j of
// the packed row: every lane assembles and stores its own word.  At D = 128 a
// wave encodes 16 vectors and moves 4 KiB in, 512 B out, both contiguous.  All
// sums are fp64 and exact under the documented exponent spread, hence identical
// to the wave-per-vector routine above whatever the order.

// v of lane (l ^ 1) or (l ^ 2).  Every lane of a quad is a valid source, so the
// move needs no previous value of its destination.
__device__ __forceinline__ double dpp_quad_xor_f64(double v, bool xor2) {
  const uint64_t bits = __builtin_bit_cast(uint64_t, v);
  const int lo = (int)(uint32_t)bits, hi = (int)(uint32_t)(bits >> 32);
  int plo, phi;
  if (xor2) {
    plo = __builtin_amdgcn_mov_dpp(lo, kDppQuadXor2, 0xf, 0xf, true);
    phi = __builtin_amdgcn_mov_dpp(hi, kDppQuadXor2, 0xf, 0xf, true);
  } else {
    plo = __builtin_amdgcn_mov_dpp(lo, kDppQuadXor1, 0xf, 0xf, true);
    phi = __builtin_amdgcn_mov_dpp(hi, kDppQuadXor1, 0xf, 0xf, true);
  }
  return __builtin_bit_cast(double, ((uint64_t)(uint32_t)phi << 32) | (uint32_t)plo);
}

// v with its sign bit flipped where sign_flip is 0x80000000 (0: unchanged).
__device__ __forceinline__ double flip_sign_f64(double v, uint32_t sign_flip) {
  const uint64_t bits = __builtin_bit_cast(uint64_t, v);
  return __builtin_bit_cast(double, bits ^ ((uint64_t)sign_flip << 32));
}

// Appends the sign bit of (tau - y) -- set exactly when y > tau -- to a mask
// that is shifted left once per call: elements must be fed from 31 down to 0.
__device__ __forceinline__ uint32_t push_greater(uint32_t mask, double y, double tau) {
  const double d = tau - y;  // +0 when equal: not greater
  const uint32_t hi = (uint32_t)(__builtin_bit_cast(uint64_t, d) >> 32);
  return __builtin_amdgcn_alignbit(mask, hi, 31);  // (mask << 1) | (hi >> 31)
}

// Vector v of n_vec = n_heads * n_rows lives at
// src + (head * head_stride_rows + row_begin + r) * D, head = v / n_rows,
// r = v % n_rows; its code row goes to the same row of dst (D / 8 * BITS byte rows).
template <int BITS, int D>
__global__ __launch_bounds__(256) void encode_rows_kernel(const uint16_t* __restrict__ src,
                                                          uint8_t* __restrict__ dst,
                                                          int64_t head_stride_rows,
                                                          int64_t row_begin, int64_t n_rows,
                                                          int64_t n_vec, Thresholds thr) {
  constexpr int LPV = D / 32;        // lanes per vector: 2, 4 or 8
  const int j = threadIdx.x & (LPV - 1);  // which 32-element part of the vector
  const int64_t quad = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / LPV;
  const int64_t n_quads = ((int64_t)gridDim.x * blockDim.x) / LPV;
  for (int64_t v = quad; v < n_vec; v += n_quads) {
    const int64_t head = v / n_rows, r = v - head * n_rows;
    const int64_t row = head * head_stride_rows + row_begin + r;
    const uint4* in = reinterpret_cast<const uint4*>(src + row * D + j * 32);
    uint4 raw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) raw[i] = in[i];
    double x[32];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        x[i * 8 + 2 * e] = (double)bf16_lo(w[e]);
        x[i * 8 + 2 * e + 1] = (double)bf16_hi(w[e]);
      }
    }
    if (thr.transform) {
      // index bits 0..4: inside the lane
#pragma unroll
      for (int h = 1; h < 32; h <<= 1) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
          if ((i & h) == 0) {
            const double a = x[i], b = x[i + h];
            x[i] = a + b;
            x[i + h] = a - b;
          }
        }
      }
      // index bits 5 and up: across the lanes of the group
#pragma unroll
      for (int s = 0; (1 << s) < LPV; ++s) {
        // the upper lane of a pair takes partner - x, the lower one x + partner:
        // one addition once the upper lane's own value has changed sign
        const uint32_t sign_flip = ((j >> s) & 1) != 0 ? 0x80000000u : 0u;
#pragma unroll
        for (int i = 0; i < 32; ++i) {
          const double partner = s < 2 ? dpp_quad_xor_f64(x[i], s == 1) : __shfl_xor(x[i], 4, kWave);
          x[i] = flip_sign_f64(x[i], sign_flip) + partner;
        }
      }
    }
    // Eq. 5 on the lane's 32 coefficients: nested indicator masks, then the
    // planes of the bucket index; lane j stores word j of the row.
    constexpr int T = (1 << BITS) - 1;
    uint32_t m[T], plane[BITS];
#pragma unroll
    for (int i = 0; i < T; ++i) m[i] = 0;
#pragma unroll
    for (int e = 31; e >= 0; --e) {
#pragma unroll
      for (int i = 0; i < T; ++i) m[i] = push_greater(m[i], x[e], thr.tau[i]);
    }
    planes_from_masks<BITS>(m, plane);
    uint32_t* out = reinterpret_cast<uint32_t*>(dst + row * (LPV * 4 * BITS) + j * (4 * BITS));
    if constexpr (BITS == 2) {
      *reinterpret_cast<uint2*>(out) = make_uint2(plane[0], plane[1]);
    } else {
#pragma unroll
      for (int p = 0; p < BITS; ++p) out[p] = plane[p];
    }
  }
}

}  // namespace adamas
