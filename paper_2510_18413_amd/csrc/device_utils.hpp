// Small wave64 / workgroup helpers shared by the Adamas kernels (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adamas {

constexpr int kHeadDim = 128;
constexpr int kRowBytes = 32;        // packed code row
constexpr int kNumBins = 385;        // distances 0..384 (Eq. 6 on 128 two-bit codes)
constexpr int kHistStride = 392;     // uint16 per stored tile histogram (784 B, 16-byte multiple)
constexpr int kPartialStride = 132;  // floats per attention partial: m, l, pad, pad, o[128]
constexpr int kWave = 64;

// Length of sequence b as the kernels use it: a sequence whose (device-side,
// unvalidated) start / length would reach outside the pool or beyond
// max_seq_len is treated as empty instead of being read out of bounds.
__device__ __forceinline__ int safe_seq_len(const int32_t* seq_len, const int64_t* seq_start, int b,
                                            int64_t max_seq_len, int64_t pool_tokens) {
  const int64_t L = seq_len[b], s = seq_start[b];
  const bool ok = L >= 0 && L <= max_seq_len && s >= 0 && s + L <= pool_tokens;
  return ok ? (int)L : 0;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) {
  return __uint_as_float(packed & 0xffff0000u);
}

__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    uint32_t o = __shfl_up(v, off, kWave);
    if (lane >= off) v += o;
  }
  return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Exclusive prefix sum over a 256-thread workgroup.  s_wave must hold 4 words.
// Returns the exclusive prefix of v; total receives the workgroup sum.
// Contains two barriers; every thread of the workgroup must call it.
__device__ __forceinline__ uint32_t block256_excl_scan(uint32_t v, uint32_t* s_wave,
                                                       uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = wave_incl_scan_u32(v, lane);
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  uint32_t w0 = s_wave[0], w1 = s_wave[1], w2 = s_wave[2], w3 = s_wave[3];
  uint32_t before = (wave > 0 ? w0 : 0u) + (wave > 1 ? w1 : 0u) + (wave > 2 ? w2 : 0u);
  total = w0 + w1 + w2 + w3;
  __syncthreads();
  return before + incl - v;
}

}  // namespace adamas
