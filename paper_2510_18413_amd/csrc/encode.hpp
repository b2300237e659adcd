// Hadamard transform (Eq. 4) + bucketize (Eq. 5) + 2-bit pack of one 128-d
// bf16 vector by one wavefront, and the bulk key / query encode kernels
// (Algorithm 1 lines 1-3).
#pragma once

#include "device_utils.hpp"

namespace adamas {

// Thresholds already multiplied by sqrt(128): the kernels compare the
// unnormalised +-1 sums against them.
struct Thresholds {
  double tau[3];
};

// One wave64 encodes one vector.  Lane l holds x[l] and x[l+64]; the
// butterfly over index bit 6 is lane-local, bits 0..5 go across lanes.  All
// sums are fp64 and exact for inputs within the documented exponent spread,
// so the stage order does not influence the result.
// Result: the four 64-bit words of the packed row, identical in every lane.
// src must be wave-uniform.  All 64 lanes must be active.
//
// encode_values_wave takes the two elements already loaded (raw bf16 bits), so
// that a caller can issue that load ahead of other memory traffic.
__device__ __forceinline__ void encode_values_wave(uint32_t bits_lo, uint32_t bits_hi,
                                                   const Thresholds& thr, uint64_t w[4]) {
  const int lane = threadIdx.x & 63;
  double a = (double)bf16_bits_to_float(bits_lo);
  double b = (double)bf16_bits_to_float(bits_hi);
  {
    double s = a + b, d = a - b;
    a = s;
    b = d;
  }
#pragma unroll
  for (int h = 1; h < 64; h <<= 1) {
    double pa = __shfl_xor(a, h, kWave);
    double pb = __shfl_xor(b, h, kWave);
    const bool upper = (lane & h) != 0;
    a = upper ? pa - a : a + pa;
    b = upper ? pb - b : b + pb;
  }
  // Nested indicator masks m1 >= m2 >= m3 of Eq. 5; code = m1 + m2 + m3, so
  // the high bit is m2 and the low bit is the parity m1 ^ m2 ^ m3.
  const uint64_t a1 = __ballot(a > thr.tau[0]), a2 = __ballot(a > thr.tau[1]),
                 a3 = __ballot(a > thr.tau[2]);
  const uint64_t b1 = __ballot(b > thr.tau[0]), b2 = __ballot(b > thr.tau[1]),
                 b3 = __ballot(b > thr.tau[2]);
  const uint64_t alo = a1 ^ a2 ^ a3, ahi = a2, blo = b1 ^ b2 ^ b3, bhi = b2;
  w[0] = (alo & 0xffffffffull) | (ahi << 32);
  w[1] = (alo >> 32) | (ahi & 0xffffffff00000000ull);
  w[2] = (blo & 0xffffffffull) | (bhi << 32);
  w[3] = (blo >> 32) | (bhi & 0xffffffff00000000ull);
}

__device__ __forceinline__ void encode_vector_wave(const uint16_t* __restrict__ src,
                                                   const Thresholds& thr, uint64_t w[4]) {
  const int lane = threadIdx.x & 63;
  encode_values_wave(src[lane], src[lane + 64], thr, w);
}

__device__ __forceinline__ void store_row_wave(uint8_t* __restrict__ dst, const uint64_t w[4]) {
  const int lane = threadIdx.x & 63;
  if (lane < 4) {
    uint64_t v = lane == 0 ? w[0] : lane == 1 ? w[1] : lane == 2 ? w[2] : w[3];
    reinterpret_cast<uint64_t*>(dst)[lane] = v;
  }
}

// Bulk encode: vector v of n_vec = n_heads * n_rows lives at
// src + (head * head_stride_rows + row_begin + r) * 128, head = v / n_rows,
// r = v % n_rows; its code row goes to the same row of dst (32 B rows).
// One wave per vector, grid-stride.
__global__ __launch_bounds__(256) void encode_rows_kernel(const uint16_t* __restrict__ src,
                                                          uint8_t* __restrict__ dst,
                                                          int64_t head_stride_rows,
                                                          int64_t row_begin, int64_t n_rows,
                                                          int64_t n_vec, Thresholds thr) {
  const int64_t wave_global = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t n_waves = (int64_t)gridDim.x * 4;
  for (int64_t v = wave_global; v < n_vec; v += n_waves) {
    const int64_t head = v / n_rows, r = v - head * n_rows;
    const int64_t row = head * head_stride_rows + row_begin + r;
    uint64_t w[4];
    encode_vector_wave(src + row * kHeadDim, thr, w);
    store_row_wave(dst + row * kRowBytes, w);
  }
}

}  // namespace adamas
