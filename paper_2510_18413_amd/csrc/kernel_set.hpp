// Launchers of the kernels of one (head dimension, metric) pair.
//
// The kernels are templates over the head dimension, the code format / distance
// estimator ("metric"), the query-group size, the scan tile and the cache
// layout.  Each (head dimension, metric) pair is instantiated in a translation
// unit of its own (kernels_inst.hip compiled once per pair), so that the pairs
// build in parallel; the C ABI in adamas.hip only sees these tables of plain
// function pointers.
#pragma once

#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "encode.hpp"
#include "full_attn.hpp"
#include "scan.hpp"
#include "select_attn.hpp"

namespace adamas {

struct KernelSet {
  // Distance scan.  fused: query encode + append in the prologue (decode step);
  // paged cache iff sp.page_table != nullptr (fused only).  G = query heads per
  // workgroup (1..8), tile_tokens = 1024, 2048 or 4096.
  void (*scan)(bool fused, int G, int tile_tokens, dim3 grid, hipStream_t st, const ScanParams& sp);
  // Top-k (+ gather + attention when attn).  256 threads per workgroup.
  void (*select)(bool attn, bool paged, dim3 grid, hipStream_t st, const SelectParams& sl);
  // Bulk encode of n_vec vectors.  Null in the squared-distance set: its code
  // rows are those of kMetricL1.
  void (*encode_rows)(hipStream_t st, const uint16_t* src, uint8_t* dst, int64_t head_stride_rows,
                      int64_t row_begin, int64_t n_rows, int64_t n_vec, const Thresholds& thr);
  // Kernels that depend on the head dimension only: set in the kMetricL1 set, null elsewhere.
  void (*sparse_attn)(dim3 grid, hipStream_t st, const AttnParams& ap);
  void (*merge)(dim3 grid, hipStream_t st, const MergeParams& mp);
  void (*full_attn)(int G, dim3 grid, hipStream_t st, const FullAttnParams& fp);
  void (*merge_parts)(dim3 grid, hipStream_t st, const float* partial, float* out, int Hq, int n_parts);
};

// Defined by kernels_inst.hip for the pair it is compiled for.
template <int D, int METRIC>
const KernelSet& kernel_set();

// Head dimensions and metrics that are built: one translation unit per pair.
#define ADAMAS_FOR_EACH_HEAD_DIM(X) X(64) X(96) X(128) X(160) X(192) X(256)
#define ADAMAS_FOR_EACH_METRIC(X, D) X(D, kMetricL1) X(D, kMetricL2) X(D, kMetricB1) X(D, kMetricB3)

}  // namespace adamas
