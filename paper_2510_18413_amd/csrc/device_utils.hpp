// Small wave64 / workgroup helpers shared by the Adamas kernels (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adamas {

constexpr int kHeadDim = 128;
constexpr int kRowBytes = 32;        // packed code row of the method (2-bit codes)
// Code format and distance estimator, one id for both:
//   kMetricL1   2-bit codes, Eq. 6 (sum of |a - b|, 0..384): the method
//   kMetricL2   2-bit codes, squared differences (Section 4.4 ablation, 0..1152)
//   kMetricB1   1-bit codes, Eq. 6 = Hamming distance (Section 4.4, 0..128)
//   kMetricB3   3-bit codes, Eq. 6 (Section 4.4, 0..896)
// A code row is four words of kBits 32-bit planes (16 * kBits bytes): plane p of
// word g holds, at bit j, bit p of the code of coefficient 32g + j.
// D is the head dimension (128 in the paper's models; 64 and 256 are built for
// the method itself): D / 32 words per row, distances up to 3 * D.
constexpr int kMetricL1 = 0, kMetricL2 = 1, kMetricB1 = 2, kMetricB3 = 3;
template <int METRIC, int D = 128>
struct Dist {
  static constexpr int kBits = METRIC == kMetricB1 ? 1 : METRIC == kMetricB3 ? 3 : 2;
  static constexpr int kWords = D / 32;                 // words per row, kBits planes each
  static constexpr int kRowBytes = kWords * 4 * kBits;  // 32 for the method at D = 128
  static constexpr int kMaxDist =  // largest distance between two code vectors
      (METRIC == kMetricL1 ? 3 : METRIC == kMetricL2 ? 9 : METRIC == kMetricB1 ? 1 : 7) * D;
  static constexpr int kBins = kMaxDist + 1;  // distinct distance values: 385 for the method
  // A tile histogram travels as kPairs 32-bit words of two 16-bit bins each (a
  // tile has at most 4096 tokens): [head][tile][word].  (Word-major rows, which
  // would let the select kernel fetch 16 tiles of a word with four 16-byte loads,
  // make every scan workgroup scatter 4-byte stores over lines that workgroups
  // on other XCDs write too: measured 0.6 us slower for the scan.)
  static constexpr int kPairs = (kBins + 1) / 2;
  // a row is fetched in pieces of the largest power of two (up to 16 bytes) that divides it
  static constexpr int kPiece = kRowBytes % 16 == 0 ? 16 : kRowBytes % 8 == 0 ? 8 : 4;
  // Distance plane between the scan and the select kernel.  Distances up to 511
  // travel as one byte (the low eight bits) per token, plus, when they can exceed
  // 255, a plane of ninth bits (one 64-bit word per 64 consecutive tokens);
  // larger ranges travel as uint16.
  static constexpr bool kByteDist = kMaxDist <= 511;
  static constexpr bool kHighPlane = kByteDist && kMaxDist > 255;
  static constexpr int kDistBytes = kByteDist ? 1 : 2;
};

// One aligned load of BYTES (16, 8 or 4) into consecutive 32-bit words.
template <int BYTES>
__device__ __forceinline__ void load_piece(const uint8_t* src, uint32_t* w) {
  if constexpr (BYTES == 16) {
    const uint4 v = *reinterpret_cast<const uint4*>(src);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if constexpr (BYTES == 8) {
    const uint2 v = *reinterpret_cast<const uint2*>(src);
    w[0] = v.x; w[1] = v.y;
  } else {
    w[0] = *reinterpret_cast<const uint32_t*>(src);
  }
}
// What the kernels derive from the head dimension D = 2^n * m, m = 1, 12 or 20
// (Section 2: H_D = H_{2^n} (x) H_m), a multiple of 32.
template <int D>
struct HeadDim {
  static_assert(D % 32 == 0, "a code row is D / 32 words");
  static constexpr bool kPow2 = (D & (D - 1)) == 0;
  static constexpr int kBase = kPow2 ? 1 : (D % 3 == 0 ? 12 : 20);  // m
  static_assert(kPow2 || (D % kBase == 0 && ((D / kBase) & (D / kBase - 1)) == 0), "D = 2^n * 12 or 2^n * 20");
  // One wave encodes one vector.  Powers of two: lane l holds elements l + 64 e,
  // e < D / 64.  Otherwise lane l < D / (m / 4) holds the m / 4 consecutive
  // elements from l * m / 4 on, so that a quad of lanes holds one block of m.
  static constexpr int kEncElems = kPow2 ? D / 64 : kBase / 4;
  static constexpr int kEncLanes = kPow2 ? 64 : D / kEncElems;
  __device__ __forceinline__ static int enc_index(int lane, int e) {
    return kPow2 ? lane + 64 * e : lane * kEncElems + e;
  }
  // Attention: a row takes D / 8 lanes of 8 dims inside an aligned group of
  // 8, 16 or 32 lanes (the next power of two; the other lanes of the group idle).
  static constexpr int kRowLanes = D / 8;
  static constexpr int kRowGroup = kRowLanes <= 8 ? 8 : kRowLanes <= 16 ? 16 : 32;
};

// floats per attention partial of a head of dimension d: m, l, pad, pad, o[d]
constexpr int partial_stride(int d) { return d + 4; }
constexpr int kWave = 64;

// Query head -> KV head without a division: magic = ceil(2^32 / group) from the
// host (0 for a group of one); exact for every head index below 2^29.
__device__ __forceinline__ int kv_head_of(int hq, uint32_t group_magic) {
  return group_magic == 0u ? hq : (int)__umulhi((uint32_t)hq, group_magic);
}

// Loads of values that every lane of the workgroup reads from one address and
// that no kernel of the library writes (sequence lengths and starts, page-table
// entries), in two flavours:
//  - scalar: through the constant address space, so that the compiler emits
//    scalar loads.  They have their own counter, so waiting for them does not
//    wait for vector loads in flight (the scan kernel, which cannot address its
//    rows without them and has conditional vector loads in front of them);
//  - vector: plain loads.  Vector loads return in issue order, so a kernel that
//    requests these first and its speculative data afterwards can wait for
//    these alone (the select kernel; a scalar load would share its counter with
//    kernel-argument loads the data loads have to wait for).
__device__ __forceinline__ int32_t scalar_load(const int32_t* p) {
  return *(const __attribute__((address_space(4))) int32_t*)(uintptr_t)p;
}
__device__ __forceinline__ int64_t scalar_load(const int64_t* p) {
  return *(const __attribute__((address_space(4))) int64_t*)(uintptr_t)p;
}

// Length of sequence b as the kernels use it: a sequence whose (device-side,
// unvalidated) start / length would reach outside the pool or beyond
// max_seq_len is treated as empty instead of being read out of bounds.
// The kernels request the raw values first of all (request), issue their
// speculative loads, and only then look at the values (length).
struct SeqInfo {
  int32_t len_raw;
  int64_t start;  // 0 for a paged cache
  template <bool PAGED, bool SCALAR>
  __device__ __forceinline__ static SeqInfo request(const int32_t* seq_len, const int64_t* seq_start, int b) {
    SeqInfo s;
    s.len_raw = SCALAR ? scalar_load(seq_len + b) : seq_len[b];
    s.start = 0;
    if constexpr (!PAGED) s.start = SCALAR ? scalar_load(seq_start + b) : seq_start[b];
    return s;
  }
  // after vector loads have arrived: tells the compiler that the values are wave-uniform
  __device__ __forceinline__ void make_uniform() {
    len_raw = __builtin_amdgcn_readfirstlane(len_raw);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)start);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)start >> 32));
    start = (int64_t)(((uint64_t)hi << 32) | lo);
  }
  // contiguous cache: the sequence must lie inside the pool
  __device__ __forceinline__ int length(int64_t max_seq_len, int64_t pool_tokens) const {
    const int64_t L = len_raw;
    const bool ok = (L >= 0) & (L <= max_seq_len) & (start >= 0) & (start + L <= pool_tokens);
    return ok ? (int)L : 0;
  }
  // paged cache: the sequence must fit the pages its table row can name
  __device__ __forceinline__ int paged_length(int64_t max_seq_len, int64_t table_tokens) const {
    const int64_t L = len_raw;
    return ((L >= 0) & (L <= max_seq_len) & (L <= table_tokens)) ? (int)L : 0;
  }
};

// Everything requested from memory so far has been issued before anything
// after this point is looked at: keeps the compiler from sinking speculative
// loads below the first wait for the sequence length, or hoisting that wait.
__device__ __forceinline__ void loads_issued_before_here() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ int safe_seq_len(const int32_t* seq_len, const int64_t* seq_start, int b,
                                            int64_t max_seq_len, int64_t pool_tokens) {
  return SeqInfo::request<false, true>(seq_len, seq_start, b).length(max_seq_len, pool_tokens);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) {
  return __uint_as_float(packed & 0xffff0000u);
}

// 2^x for x <= 0 (softmax weights): the hardware instruction as it is.  Results
// below the normal range come out as 0, which is what a weight of 2^-127 is worth.
__device__ __forceinline__ float exp2_neg(float x) { return __builtin_amdgcn_exp2f(x); }

// Per-half-word subtraction of two packed uint16 pairs (no borrow across halves).
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b) {
  const ushort2_t d = __builtin_bit_cast(ushort2_t, a) - __builtin_bit_cast(ushort2_t, b);
  return __builtin_bit_cast(uint32_t, d);
}

// ---- phase stamps (profiling builds only: -DADAMAS_PHASE_TRACE) -------------
// Thread 0 of a workgroup notes the 100 MHz wall clock at phase boundaries and
// writes the notes to record `blockIdx` of a trace buffer when it leaves.  In
// ordinary builds all of this compiles to nothing.
constexpr int kTraceSlots = 16;  // 64-bit words per workgroup record
#ifdef ADAMAS_PHASE_TRACE
struct PhaseTrace {
  uint64_t t[kTraceSlots];
  __device__ __forceinline__ PhaseTrace() {
#pragma unroll
    for (int i = 0; i < kTraceSlots; ++i) t[i] = 0;
  }
  // wait: first waits for this wave's outstanding memory operations (stores
  // included), so that the note marks the point where the phase's data has arrived
  __device__ __forceinline__ void stamp(int i, bool wait = true) {
    if (wait) __builtin_amdgcn_s_waitcnt(0);
    if (threadIdx.x == 0) t[i] = wall_clock64();
  }
  __device__ __forceinline__ void flush(uint64_t* buf, int64_t n_records) const {
    const int64_t wg = ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (threadIdx.x == 0 && buf != nullptr && wg < n_records) {
#pragma unroll
      for (int i = 0; i < kTraceSlots; ++i) buf[wg * kTraceSlots + i] = t[i];
    }
  }
};
#else
struct PhaseTrace {
  __device__ __forceinline__ void stamp(int, bool = true) {}
  __device__ __forceinline__ void flush(uint64_t*, int64_t) const {}
};
#endif

// ---- data-parallel-primitive (DPP) cross-lane moves: one VALU instruction each,
// no LDS round trip.  A "row" is 16 consecutive lanes.
constexpr int kDppQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kDppRowShr = 0x110;        // + n: lane i reads lane i-n of its row
constexpr int kDppRowMirror = 0x140;     // lane i reads lane 15-i of its row
constexpr int kDppRowHalfMirror = 0x141; // lane i reads lane 7-i of its half row
constexpr int kDppRowBcast15 = 0x142;    // lane 15 of each row -> the next row
constexpr int kDppRowBcast31 = 0x143;    // lane 31 -> rows 2 and 3

template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  // lanes with no source (shifted in, masked rows) receive 0
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Lane `lane` (0..3) of v receives the wave-uniform value x; the other lanes keep theirs.
__device__ __forceinline__ void write_lane(uint32_t& v, uint32_t x, int lane) {
  switch (lane) {
    case 0: asm("v_writelane_b32 %0, %1, 0" : "+v"(v) : "s"(x)); break;
    case 1: asm("v_writelane_b32 %0, %1, 1" : "+v"(v) : "s"(x)); break;
    case 2: asm("v_writelane_b32 %0, %1, 2" : "+v"(v) : "s"(x)); break;
    default: asm("v_writelane_b32 %0, %1, 3" : "+v"(v) : "s"(x)); break;
  }
}

// Sum over each aligned group of LANES lanes (8, 16 or 32); every lane of the
// group receives the total.  After the two quad steps all lanes of a quad
// agree, so mirroring inside the half row pairs quad 0 with quad 1, mirroring
// the row pairs the halves, and a 32-lane group adds its other DPP row.
template <int LANES>
__device__ __forceinline__ float lanes_sum_f32(float v) {
  v += dpp_f32<kDppQuadXor1>(v);
  v += dpp_f32<kDppQuadXor2>(v);
  v += dpp_f32<kDppRowHalfMirror>(v);
  if constexpr (LANES >= 16) v += dpp_f32<kDppRowMirror>(v);
  if constexpr (LANES >= 32) v += __shfl_xor(v, 16, kWave);
  return v;
}

// The same for doubles (two 32-bit moves per step).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  // every lane has a valid source under these patterns: no previous value needed
  const uint32_t lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)b, CTRL, 0xf, 0xf, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, true);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
template <int LANES>
__device__ __forceinline__ double lanes_sum_f64(double v) {
  v += dpp_f64<kDppQuadXor1>(v);
  v += dpp_f64<kDppQuadXor2>(v);
  v += dpp_f64<kDppRowHalfMirror>(v);
  if constexpr (LANES >= 16) v += dpp_f64<kDppRowMirror>(v);
  if constexpr (LANES >= 32) v += __shfl_xor(v, 16, kWave);
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wave (Hillis-Steele inside each
// row, then the row totals are carried across rows with the two broadcasts).
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
  v += dpp_u32<kDppRowShr + 1>(v);
  v += dpp_u32<kDppRowShr + 2>(v);
  v += dpp_u32<kDppRowShr + 4>(v);
  v += dpp_u32<kDppRowShr + 8>(v);
  v += dpp_u32<kDppRowBcast15, 0xa>(v);  // rows 1 and 3 += total of the row before
  v += dpp_u32<kDppRowBcast31, 0xc>(v);  // rows 2 and 3 += total of lanes 0..31
  return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan_u32(v), 63);
}

}  // namespace adamas
