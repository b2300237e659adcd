// Instantiates every kernel of ONE (head dimension, metric) pair and exports
// their launchers as a KernelSet.  Compiled once per pair with
//   -DADAMAS_INST_D=<64|96|128|160|192|256> -DADAMAS_INST_METRIC=<0..3>
// (see kernel_set.hpp and build.py).
#include "kernel_set.hpp"

#if !defined(ADAMAS_INST_D) || !defined(ADAMAS_INST_METRIC)
#error "compile with -DADAMAS_INST_D=... -DADAMAS_INST_METRIC=..."
#endif

namespace adamas {
namespace {

constexpr int D = ADAMAS_INST_D;
constexpr int METRIC = ADAMAS_INST_METRIC;
constexpr int BITS = Dist<METRIC, D>::kBits;
constexpr int kSelThreads = 256;

template <int G, bool FUSED, bool PAGED>
void launch_scan_tile(int tile_tokens, dim3 grid, hipStream_t st, const ScanParams& sp) {
  switch (tile_tokens) {
    case 1024: hipLaunchKernelGGL((scan_kernel<G, FUSED, 4, METRIC, PAGED, D>), grid, dim3(256), 0, st, sp); break;
    case 2048: hipLaunchKernelGGL((scan_kernel<G, FUSED, 8, METRIC, PAGED, D>), grid, dim3(512), 0, st, sp); break;
    default: hipLaunchKernelGGL((scan_kernel<G, FUSED, 16, METRIC, PAGED, D>), grid, dim3(1024), 0, st, sp); break;
  }
}

template <int G>
void launch_scan_g(bool fused, int tile_tokens, dim3 grid, hipStream_t st, const ScanParams& sp) {
  if (!fused) return launch_scan_tile<G, false, false>(tile_tokens, grid, st, sp);
  if (sp.page_table != nullptr) return launch_scan_tile<G, true, true>(tile_tokens, grid, st, sp);
  launch_scan_tile<G, true, false>(tile_tokens, grid, st, sp);
}

void launch_scan(bool fused, int G, int tile_tokens, dim3 grid, hipStream_t st, const ScanParams& sp) {
  switch (G) {
    case 1: launch_scan_g<1>(fused, tile_tokens, grid, st, sp); break;
    case 2: launch_scan_g<2>(fused, tile_tokens, grid, st, sp); break;
    case 3: launch_scan_g<3>(fused, tile_tokens, grid, st, sp); break;
    case 4: launch_scan_g<4>(fused, tile_tokens, grid, st, sp); break;
    case 5: launch_scan_g<5>(fused, tile_tokens, grid, st, sp); break;
    case 6: launch_scan_g<6>(fused, tile_tokens, grid, st, sp); break;
    case 7: launch_scan_g<7>(fused, tile_tokens, grid, st, sp); break;
    default: launch_scan_g<8>(fused, tile_tokens, grid, st, sp); break;
  }
}

template <int CHUNK>
void launch_select_chunk(bool attn, bool paged, dim3 grid, hipStream_t st, const SelectParams& sl) {
  if (!attn)
    hipLaunchKernelGGL((select_kernel<kSelThreads, false, METRIC, false, D, CHUNK>), grid, dim3(kSelThreads), 0, st, sl);
  else if (paged)
    hipLaunchKernelGGL((select_kernel<kSelThreads, true, METRIC, true, D, CHUNK>), grid, dim3(kSelThreads), 0, st, sl);
  else
    hipLaunchKernelGGL((select_kernel<kSelThreads, true, METRIC, false, D, CHUNK>), grid, dim3(kSelThreads), 0, st, sl);
}

void launch_select(bool attn, bool paged, dim3 grid, hipStream_t st, const SelectParams& sl) {
  // segments of more than two passes (4096 tokens each) share one barrier among up to eight passes;
  // only planes of byte distances have that form
  if (Dist<METRIC, D>::kByteDist && sl.seg_len > 2 * 4096) launch_select_chunk<8>(attn, paged, grid, st, sl);
  else launch_select_chunk<1>(attn, paged, grid, st, sl);
}

// The launchers below are templates so that a set that does not export them
// does not instantiate their kernels either.
template <int BITS_>
void launch_encode_rows(hipStream_t st, const uint16_t* src, uint8_t* dst, int64_t head_stride_rows,
                        int64_t row_begin, int64_t n_rows, int64_t n_vec, const Thresholds& thr) {
  // vectors per 256-thread workgroup and pass: D / 32 lanes per vector, or D / m lanes for D = 2^n * m (m = 12, 20)
  const int64_t per_wg = 256 / (HeadDim<D>::kPow2 ? D / 32 : D / HeadDim<D>::kBase);
  const int64_t want = (n_vec + per_wg - 1) / per_wg;
  const int grid = (int)(want < 16384 ? want : 16384);
  Divisor32 by_rows{};  // mul = 0: the kernel divides in 64 bits
  if (n_vec < ((int64_t)1 << 32) && n_rows >= 1) by_rows = Divisor32::of((uint32_t)n_rows);
  hipLaunchKernelGGL((encode_rows_kernel<BITS_, D>), dim3(grid), dim3(256), 0, st, src, dst,
                     head_stride_rows, row_begin, n_rows, n_vec, thr, by_rows);
}

template <int D_>
void launch_sparse_attn(dim3 grid, hipStream_t st, const AttnParams& ap) {
  hipLaunchKernelGGL(sparse_attn_kernel<D_>, grid, dim3(kAttnThreads), 0, st, ap);
}

template <int D_>
void launch_merge(dim3 grid, hipStream_t st, const MergeParams& mp) {
  hipLaunchKernelGGL(merge_kernel<D_>, grid, dim3(D_), 0, st, mp);
}

template <int G, int D_>
void launch_full_g(dim3 grid, hipStream_t st, const FullAttnParams& fp) {
  hipLaunchKernelGGL((full_attn_kernel<G, D_>), grid, dim3(kFullThreads), 0, st, fp);
}

template <int D_>
void launch_full(int G, dim3 grid, hipStream_t st, const FullAttnParams& fp) {
  switch (G) {
    case 1: launch_full_g<1, D_>(grid, st, fp); break;
    case 2: launch_full_g<2, D_>(grid, st, fp); break;
    case 3: launch_full_g<3, D_>(grid, st, fp); break;
    case 4: launch_full_g<4, D_>(grid, st, fp); break;
    case 5: launch_full_g<5, D_>(grid, st, fp); break;
    case 6: launch_full_g<6, D_>(grid, st, fp); break;
    case 7: launch_full_g<7, D_>(grid, st, fp); break;
    default: launch_full_g<8, D_>(grid, st, fp); break;
  }
}

template <int D_>
void launch_merge_parts(dim3 grid, hipStream_t st, const float* partial, float* out, int Hq,
                        int n_parts) {
  hipLaunchKernelGGL(merge_parts_kernel<D_>, grid, dim3(kMergeThreads), 0, st, partial, out, Hq, n_parts);
}

template <int M>
KernelSet make_set() {
  KernelSet ks{};
  ks.scan = launch_scan;
  ks.select = launch_select;
  if constexpr (M != kMetricL2) ks.encode_rows = launch_encode_rows<BITS>;
  if constexpr (M == kMetricL1) {
    ks.sparse_attn = launch_sparse_attn<D>;
    ks.merge = launch_merge<D>;
    ks.full_attn = launch_full<D>;
    ks.merge_parts = launch_merge_parts<D>;
  }
  return ks;
}

}  // namespace

template <>
const KernelSet& kernel_set<ADAMAS_INST_D, ADAMAS_INST_METRIC>() {
  static const KernelSet ks = make_set<ADAMAS_INST_METRIC>();
  return ks;
}

}  // namespace adamas
