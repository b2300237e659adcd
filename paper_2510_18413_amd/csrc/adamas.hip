// C ABI of the Adamas decode path for MI355X (gfx950): argument checks, the
// launch plan and the kernel launches.  See include/adamas.h for the contract.
#include "adamas.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>

#include "kernel_set.hpp"

// Scratch of adamas_decode_step_static.  In host code this name is only a handle
// for hipGetSymbolAddress, never a device address: kernels get the looked-up
// pointer (static_scratch()).
static __device__ __align__(256) unsigned char scratch[ADAMAS_STATIC_SCRATCH_BYTES];

namespace {

using namespace adamas;

thread_local int g_last_hip_error = 0;

// Profiling builds: where the kernels leave their phase stamps (adamas_phase_trace).
uint64_t* g_trace_scan = nullptr;
uint64_t* g_trace_select = nullptr;
int64_t g_trace_records = 0;

// Device address of `scratch` on the current device (every GPU holds its own
// copy of the array at its own address), looked up once per device.  Returns
// nullptr and records the HIP error if the runtime refuses.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

void* static_scratch() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidDevice);
    return nullptr;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr != nullptr) return ptr;
  e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));  // same answer from every thread
  if (e != hipSuccess || ptr == nullptr) {
    g_last_hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidSymbol);
    return nullptr;
  }
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  return ptr;
}

constexpr int kTargetWorkgroups = 256;  // one per compute unit of an MI355X
constexpr int kSegGranule = 4096;
constexpr double kLog2e = 1.4426950408889634;

// How one call is cut into workgroups and where its scratch lives in the workspace.
struct Plan {
  int tile_tokens;   // tokens per scan workgroup (threads = tile_tokens / 4): 1024, 2048 or 4096
  int n_tiles;       // scan tiles per (sequence, KV head)
  int seg_len;       // tokens per select workgroup, kSegGranule times a power of two (a multiple of the tile)
  int n_segs;        // select workgroups per (sequence, query head)
  int metric;        // code format + distance estimator (struct Dist)
  int head_dim;      // 64, 128 or 256
  int g_split;       // scan workgroups per (tile, KV head), each with a share of the query group
  int64_t dist_stride;
  size_t off_dist, off_high, off_hist, off_partial, total;
};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ceil(2^32 / group), 0 for a group of one (kv_head_of in the kernels)
uint32_t group_magic_of(const adamas_config* c) {
  const uint64_t g = (uint64_t)(c->num_q_heads / c->num_kv_heads);
  return g == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + g - 1) / g);
}

int log2_of(int64_t pow2) {
  int s = 0;
  while (((int64_t)1 << s) < pow2) ++s;
  return s;
}

int code_bits(const adamas_config* c) { return c->code_bits == 0 ? 2 : c->code_bits; }

// Code format + distance estimator id (see struct Dist).
int metric_of(const adamas_config* c) {
  if (code_bits(c) == 1) return kMetricB1;
  if (code_bits(c) == 3) return kMetricB3;
  return (c->variant & ADAMAS_VARIANT_L2) ? kMetricL2 : kMetricL1;
}

// Largest distance of a metric (Dist<METRIC, D>::kMaxDist for run-time arguments).
int max_dist_of(int metric, int head_dim) {
  const int per_dim = metric == kMetricL1 ? 3 : metric == kMetricL2 ? 9 : metric == kMetricB1 ? 1 : 7;
  return per_dim * head_dim;
}

// 32-bit words of a tile histogram (Dist<METRIC, D>::kPairs)
size_t hist_pairs_of(int metric, int head_dim) { return (size_t)(max_dist_of(metric, head_dim) + 2) / 2; }

// Bytes per token of the distance plane, and whether a plane of ninth bits goes
// with it (Dist<METRIC, D>::kDistBytes, kHighPlane).
int dist_bytes_of(int metric, int head_dim) { return max_dist_of(metric, head_dim) <= 511 ? 1 : 2; }
bool high_plane_of(int metric, int head_dim) {
  const int m = max_dist_of(metric, head_dim);
  return m > 255 && m <= 511;
}

// The kernels of a (head dimension, metric) pair; nullptr if that pair is not built.
const KernelSet* find_kernel_set(int head_dim, int metric) {
#ifdef ADAMAS_ONLY_D  // developer build of a single pair (build.py, only=...)
  if (head_dim == ADAMAS_ONLY_D && metric == ADAMAS_ONLY_METRIC)
    return &kernel_set<ADAMAS_ONLY_D, ADAMAS_ONLY_METRIC>();
  return nullptr;
#endif
#define ADAMAS_SET_CASE(D, M) \
  if (head_dim == D && metric == M) return &kernel_set<D, M>();
#define ADAMAS_SET_CASES(D) ADAMAS_FOR_EACH_METRIC(ADAMAS_SET_CASE, D)
  ADAMAS_FOR_EACH_HEAD_DIM(ADAMAS_SET_CASES)
#undef ADAMAS_SET_CASES
#undef ADAMAS_SET_CASE
  return nullptr;
}

bool head_dim_built(int head_dim) { return find_kernel_set(head_dim, kMetricL1) != nullptr; }

int check_config(const adamas_config* c) {
  if (c == nullptr) return ADAMAS_ERR_BAD_ARG;
  if (c->num_q_heads < 1 || c->num_kv_heads < 1 || c->pool_tokens < 1)
    return ADAMAS_ERR_BAD_ARG;
  if (c->num_q_heads % c->num_kv_heads != 0) return ADAMAS_ERR_BAD_ARG;
  if (c->num_q_heads > 65535) return ADAMAS_ERR_BAD_ARG;
  if (c->code_bits < 0 || c->code_bits > 3) return ADAMAS_ERR_BAD_ARG;
  const int n_thr = (1 << code_bits(c)) - 1;
  for (const float* t : {c->thr_k, c->thr_q}) {
    for (int i = 0; i < n_thr; ++i) {
      if (!std::isfinite(t[i])) return ADAMAS_ERR_BAD_ARG;
      if (i > 0 && !(t[i - 1] < t[i])) return ADAMAS_ERR_BAD_ARG;
    }
  }
  if (!std::isfinite(c->sm_scale) || c->sm_scale < 0.f) return ADAMAS_ERR_BAD_ARG;
  if (!head_dim_built(c->head_dim)) return ADAMAS_ERR_UNSUPPORTED;
  if (c->variant & ~(ADAMAS_VARIANT_NO_HADAMARD | ADAMAS_VARIANT_L2)) return ADAMAS_ERR_UNSUPPORTED;
  if ((c->variant & ADAMAS_VARIANT_L2) && code_bits(c) != 2) return ADAMAS_ERR_UNSUPPORTED;
  if (c->num_q_heads / c->num_kv_heads > ADAMAS_MAX_GROUP) return ADAMAS_ERR_UNSUPPORTED;
  return ADAMAS_OK;
}

int check_sizes(int32_t batch, int64_t max_seq_len, int32_t k) {
  if (batch < 1 || batch > 65535 || max_seq_len < 1 || k < 1) return ADAMAS_ERR_BAD_ARG;
  if (k > ADAMAS_MAX_K || max_seq_len > ADAMAS_MAX_SEQ_LEN) return ADAMAS_ERR_UNSUPPORTED;
  return ADAMAS_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

Plan make_plan(const adamas_config* c, int32_t batch, int64_t max_seq_len, int32_t k) {
  (void)k;  // the budget does not change the plan: the workspace holds every distance whatever k is
  Plan pl{};
  pl.metric = metric_of(c);
  pl.head_dim = c->head_dim;
  const int64_t planes = (int64_t)batch * c->num_kv_heads;
  // Scan tile (measured on MI355X): large tiles amortise the per-workgroup
  // prologue and leave the select kernel fewer tile histograms to read, small
  // ones fit more workgroups on a compute unit.
  auto n_wg = [&](int tile) { return planes * ((max_seq_len + tile - 1) / tile); };
  if (n_wg(4096) >= 4 * kTargetWorkgroups) {
    // many rounds of workgroups per compute unit: residency matters most
    pl.tile_tokens = 1024;
  } else if (n_wg(4096) >= kTargetWorkgroups) {
    // Half-size workgroups balance better over the compute units (0.4 us on a
    // 32 MiB plane) as long as a head keeps at most one batch of tile
    // histograms for the select kernel to read.
    pl.tile_tokens = (max_seq_len + 2047) / 2048 <= kHistBatch ? 2048 : 4096;
  } else if (n_wg(2048) >= kTargetWorkgroups / 2) {
    pl.tile_tokens = 2048;
  } else {
    pl.tile_tokens = 1024;
  }
  pl.n_tiles = (int)((max_seq_len + pl.tile_tokens - 1) / pl.tile_tokens);
  // Few planes and a query group: the scan is then bound by the distance
  // arithmetic of the workgroups that exist, not by memory, so the group is cut
  // in two (each half re-reads the rows) until there is a workgroup per compute unit.
  pl.g_split = 1;
  const int group = c->num_q_heads / c->num_kv_heads;
  if (group % 2 == 0 && n_wg(pl.tile_tokens) * 2 <= kTargetWorkgroups) pl.g_split = 2;
  // Select + attention: a head is cut into segments, one workgroup each (a
  // single compute unit is too slow to compact a whole 32K-token head or to
  // gather all of its rows), and the segments' attention partials are merged
  // afterwards (by the last segment to finish, or by the merge kernel in staged
  // calls).  With many heads in flight there is parallelism enough
  // already: fewer segments mean fewer re-reads of the head's histograms, and a
  // head that fits one segment needs no merge at all.
  const int64_t n_heads = (int64_t)batch * c->num_q_heads;
  int64_t want = (2 * kTargetWorkgroups + n_heads - 1) / n_heads;
  if (want > kMaxParts) want = kMaxParts;
  // a power of two (the select kernel shifts instead of dividing) and a multiple of every tile size
  int64_t seg = kSegGranule;
  while (seg * want < max_seq_len) seg *= 2;
  pl.seg_len = (int)seg;
  pl.n_segs = (int)((max_seq_len + seg - 1) / seg);
  pl.dist_stride = (max_seq_len + 127) & ~(int64_t)127;
  const size_t heads = (size_t)batch * c->num_q_heads;
  size_t off = 0;
  pl.off_dist = off;
  off = align256(off + heads * (size_t)pl.dist_stride * dist_bytes_of(pl.metric, c->head_dim));
  pl.off_high = off;
  if (high_plane_of(pl.metric, c->head_dim)) off = align256(off + heads * (size_t)pl.dist_stride / 8);
  pl.off_hist = off;
  // + kHistBatch rows: the select kernel reads whole batches of tile rows, also behind the last head's
  off = align256(off + (heads * (size_t)pl.n_tiles + kHistBatch) * hist_pairs_of(pl.metric, c->head_dim) *
                           sizeof(uint32_t));
  pl.off_partial = off;
  off = align256(off + heads * (size_t)kMaxParts * partial_stride(c->head_dim) * sizeof(float));
  pl.total = off;
  return pl;
}

// Whether the select kernel requests its first K / V lines ahead of the gather
// (SelectParams::early_rows).  Measured on MI355X: it gains 0.25 to 0.6 us
// where at most two workgroups share a compute unit and a segment takes at most
// four passes (contexts of 32K to 128K at batch 1 to 4), is neutral to slightly
// harmful with eight passes per segment (16 ragged sequences, one segment per
// head), and costs 6 us of 48 with 2048 short heads in flight.
int early_rows_pay(const Plan& pl, int64_t n_heads) {
  return n_heads * pl.n_segs <= 2 * kTargetWorkgroups && pl.seg_len <= 4 * kSegGranule ? 1 : 0;
}

// Thresholds as the kernels compare them (see struct Thresholds).
Thresholds scaled(const adamas_config* c, const float* thr) {
  Thresholds t{};
  t.transform = (c->variant & ADAMAS_VARIANT_NO_HADAMARD) ? 0 : 1;
  const double root = t.transform ? std::sqrt((double)c->head_dim) : 1.0;
  const int n_thr = (1 << code_bits(c)) - 1;
  for (int i = 0; i < n_thr; ++i) t.tau[i] = (double)thr[i] * root;
  // single-precision copies for the bulk encode's certified attempt
  t.fast = 1;
  double worst = 0.0;
  for (int i = 0; i < n_thr; ++i) {
    t.tau32[i] = (float)t.tau[i];
    const double back = (double)t.tau32[i];
    if (!std::isfinite(t.tau32[i]) || (back > 0.0) != (t.tau[i] > 0.0) || (back < 0.0) != (t.tau[i] < 0.0))
      t.fast = 0;
    worst = std::fmax(worst, std::fabs(back - t.tau[i]));
  }
  // rounded up: a bound must not shrink when it is stored as a float
  t.dtau = worst == 0.0 ? 0.f : std::nextafter((float)(worst * 1.000001), INFINITY);
  if (!std::isfinite(t.dtau)) t.fast = 0;
  t.symmetric = n_thr == 3 && t.tau[1] == 0.0 && t.tau[2] > 0.0 && t.tau[0] == -t.tau[2];
  return t;
}

const KernelSet& set_of(const adamas_config* c) { return *find_kernel_set(c->head_dim, metric_of(c)); }

// The bulk encode and the kernels that depend on the head dimension only live in
// the set of the method's own metric (same code rows for the squared distance).
const KernelSet& encode_set_of(const adamas_config* c) {
  const int m = metric_of(c);
  return *find_kernel_set(c->head_dim, m == kMetricL2 ? kMetricL1 : m);
}
const KernelSet& dim_set_of(const adamas_config* c) { return *find_kernel_set(c->head_dim, kMetricL1); }

double scale_log2e(const adamas_config* c) {
  const double s = c->sm_scale > 0.f ? (double)c->sm_scale : 1.0 / std::sqrt((double)c->head_dim);
  return s * kLog2e;
}

// Drops an error an earlier, unrelated HIP call may have left on this thread,
// so that launch_status() reports only this library's launches.
void clear_stale_error() { (void)hipGetLastError(); }

int launch_status() {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    g_last_hip_error = (int)e;
    return ADAMAS_ERR_HIP;
  }
  return ADAMAS_OK;
}

// pl.tile_tokens is 1024, 2048 or 4096 (make_plan).
void launch_scan(const adamas_config* c, bool fused, const Plan& pl, int batch, hipStream_t st,
                 ScanParams sp) {
  const int group = c->num_q_heads / c->num_kv_heads;
  sp.g_split = group % pl.g_split == 0 ? pl.g_split : 1;
  const dim3 grid(pl.n_tiles, c->num_kv_heads * sp.g_split, batch);
  set_of(c).scan(fused, group / sp.g_split, pl.tile_tokens, grid, st, sp);
}

struct FullPlan {
  int n_splits, chunk;
  size_t total;
};

// About four workgroups per compute unit; a split covers a multiple of 256 tokens.
FullPlan make_full_plan(const adamas_config* c, int32_t batch, int64_t max_seq_len) {
  FullPlan fp{};
  const int64_t planes = (int64_t)batch * c->num_kv_heads;
  int64_t want = (4 * kTargetWorkgroups + planes - 1) / planes;
  if (want > kFullMaxSplits) want = kFullMaxSplits;
  int64_t chunk = (max_seq_len + want - 1) / want;
  chunk = (chunk + 255) / 256 * 256;
  fp.chunk = (int)chunk;
  fp.n_splits = (int)((max_seq_len + chunk - 1) / chunk);
  fp.total = align256((size_t)batch * c->num_q_heads * fp.n_splits * partial_stride(c->head_dim) * sizeof(float));
  return fp;
}

// Read-only streaming probe in the scan's access pattern (two 32-byte rows per
// lane, lanes of a wave on consecutive rows): what the memory system delivers
// when nothing else is done with the rows.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src,
                                                          uint32_t* __restrict__ sink,
                                                          int64_t n_rows) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t wave = tid >> 6;
  const int lane = (int)(tid & 63);
  uint4 v[4];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int64_t row = min((wave * 2 + i) * kWave + lane, n_rows - 1);
    v[2 * i] = src[row * 2];
    v[2 * i + 1] = src[row * 2 + 1];
  }
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive
}

uint8_t* ws_at(void* ws, size_t off) { return static_cast<uint8_t*>(ws) + off; }

}  // namespace

extern "C" {

const char* adamas_status_string(int status) {
  switch (status) {
    case ADAMAS_OK: return "ok";
    case ADAMAS_ERR_BAD_ARG: return "bad argument";
    case ADAMAS_ERR_UNSUPPORTED: return "unsupported configuration";
    case ADAMAS_ERR_WORKSPACE: return "workspace too small";
    case ADAMAS_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

#ifndef ADAMAS_BUILD_ID
#define ADAMAS_BUILD_ID "unknown"
#endif
const char* adamas_build_id(void) {
  // the tag lets a build script read the id out of the file without loading it
  static const char tagged[] = "ADAMAS_BUILD_ID=" ADAMAS_BUILD_ID;
  return tagged + sizeof("ADAMAS_BUILD_ID=") - 1;
}

int adamas_last_hip_error(void) { return g_last_hip_error; }

int adamas_phase_trace(void* scan_records, void* select_records, int64_t n_records) {
#ifdef ADAMAS_PHASE_TRACE
  if (n_records < 0 || ((scan_records || select_records) && n_records == 0)) return ADAMAS_ERR_BAD_ARG;
  g_trace_scan = static_cast<uint64_t*>(scan_records);
  g_trace_select = static_cast<uint64_t*>(select_records);
  g_trace_records = n_records;
  return ADAMAS_OK;
#else
  (void)scan_records; (void)select_records; (void)n_records;
  return ADAMAS_ERR_UNSUPPORTED;
#endif
}

size_t adamas_workspace_bytes(const adamas_config* cfg, int32_t batch, int64_t max_seq_len,
                              int32_t k) {
  if (check_config(cfg) != ADAMAS_OK || check_sizes(batch, max_seq_len, k) != ADAMAS_OK) return 0;
  return make_plan(cfg, batch, max_seq_len, k).total;
}

int adamas_encode_keys(const adamas_config* cfg, const void* K, void* codes, int64_t row_begin,
                       int64_t n_rows, void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (K == nullptr || codes == nullptr || row_begin < 0 || n_rows < 0) return ADAMAS_ERR_BAD_ARG;
  if (row_begin + n_rows > cfg->pool_tokens) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(K) || !aligned16(codes)) return ADAMAS_ERR_BAD_ARG;
  if (n_rows == 0) return ADAMAS_OK;
  clear_stale_error();
  const int64_t n_vec = n_rows * cfg->num_kv_heads;
  encode_set_of(cfg).encode_rows((hipStream_t)stream, static_cast<const uint16_t*>(K),
                                 static_cast<uint8_t*>(codes), cfg->pool_tokens, row_begin, n_rows,
                                 n_vec, scaled(cfg, cfg->thr_k));
  return launch_status();
}

int adamas_encode_query(const adamas_config* cfg, const void* q, void* qcodes, int32_t batch,
                        void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (q == nullptr || qcodes == nullptr || batch < 1 || batch > 65535) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(q) || !aligned16(qcodes)) return ADAMAS_ERR_BAD_ARG;
  clear_stale_error();
  const int64_t n_vec = (int64_t)batch * cfg->num_q_heads;
  // queries form one "head" of n_vec consecutive rows
  encode_set_of(cfg).encode_rows((hipStream_t)stream, static_cast<const uint16_t*>(q),
                                 static_cast<uint8_t*>(qcodes), 0, 0, n_vec, n_vec,
                                 scaled(cfg, cfg->thr_q));
  return launch_status();
}

int adamas_manhattan_distance(const adamas_config* cfg, const void* qcodes, const void* codes,
                              const int64_t* seq_start, const int32_t* seq_len, int32_t batch,
                              uint16_t* dist_out, int64_t max_seq_len, void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (int rc = check_sizes(batch, max_seq_len, 1)) return rc;
  if (!qcodes || !codes || !seq_start || !seq_len || !dist_out) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(codes) || !aligned16(qcodes)) return ADAMAS_ERR_BAD_ARG;
  clear_stale_error();
  const Plan pl = make_plan(cfg, batch, max_seq_len, 1);
  ScanParams sp{};
  sp.codes = static_cast<const uint8_t*>(codes);
  sp.qcodes = static_cast<const uint8_t*>(qcodes);
  sp.seq_start = seq_start;
  sp.seq_len = seq_len;
  sp.dist_user = dist_out;
  sp.dist_user_stride = max_seq_len;
  sp.pool_tokens = cfg->pool_tokens;
  sp.max_seq_len = max_seq_len;
  sp.Hq = cfg->num_q_heads;
  sp.Hkv = cfg->num_kv_heads;
  sp.n_tiles = pl.n_tiles;
  launch_scan(cfg, false, pl, batch, (hipStream_t)stream, sp);
  return launch_status();
}

int adamas_select_topk(const adamas_config* cfg, const void* qcodes, const void* codes,
                       const int64_t* seq_start, const int32_t* seq_len, int32_t batch, int32_t k,
                       int32_t* idx_out, uint16_t* dist_out, int64_t max_seq_len, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (int rc = check_sizes(batch, max_seq_len, k)) return rc;
  if (!qcodes || !codes || !seq_start || !seq_len || !idx_out || !workspace) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(codes) || !aligned16(qcodes)) return ADAMAS_ERR_BAD_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return ADAMAS_ERR_BAD_ARG;
  const Plan pl = make_plan(cfg, batch, max_seq_len, k);
  if (workspace_bytes < pl.total) return ADAMAS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();

  ScanParams sp{};
  sp.codes = static_cast<const uint8_t*>(codes);
  sp.qcodes = static_cast<const uint8_t*>(qcodes);
  sp.seq_start = seq_start;
  sp.seq_len = seq_len;
  sp.dist = ws_at(workspace, pl.off_dist);
  sp.dist_high = reinterpret_cast<uint64_t*>(ws_at(workspace, pl.off_high));
  sp.dist_stride = pl.dist_stride;
  sp.dist_user = dist_out;
  sp.dist_user_stride = max_seq_len;
  sp.tilehist = reinterpret_cast<uint32_t*>(ws_at(workspace, pl.off_hist));
  sp.pool_tokens = cfg->pool_tokens;
  sp.max_seq_len = max_seq_len;
  sp.Hq = cfg->num_q_heads;
  sp.Hkv = cfg->num_kv_heads;
  sp.n_tiles = pl.n_tiles;
  launch_scan(cfg, false, pl, batch, st, sp);
  if (int rc = launch_status()) return rc;

  SelectParams sl{};
  sl.dist = sp.dist;
  sl.dist_high = sp.dist_high;
  sl.dist_stride = pl.dist_stride;
  sl.tilehist = sp.tilehist;
  sl.seq_start = seq_start;
  sl.seq_len = seq_len;
  sl.idx_out = idx_out;
  sl.pool_tokens = cfg->pool_tokens;
  sl.max_seq_len = max_seq_len;
  sl.Hq = cfg->num_q_heads;
  sl.Hkv = cfg->num_kv_heads;
  sl.k = k;
  sl.group_magic = group_magic_of(cfg);
  sl.n_tiles = pl.n_tiles;
  sl.tile_tokens = pl.tile_tokens;
  sl.seg_len = pl.seg_len;
  sl.tile_shift = log2_of(pl.tile_tokens);
  sl.seg_shift = log2_of(pl.seg_len);
  sl.early_rows = early_rows_pay(pl, (int64_t)batch * cfg->num_q_heads);
  set_of(cfg).select(false, false, dim3(pl.n_segs, cfg->num_q_heads, batch), st, sl);
  return launch_status();
}

int adamas_sparse_attn(const adamas_config* cfg, const void* q, const void* K, const void* V,
                       const int64_t* seq_start, const int32_t* idx, int32_t batch, int32_t k,
                       float* out, int64_t max_seq_len, void* workspace, size_t workspace_bytes,
                       void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (int rc = check_sizes(batch, max_seq_len, k)) return rc;
  if (!q || !K || !V || !seq_start || !idx || !out || !workspace) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V)) return ADAMAS_ERR_BAD_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return ADAMAS_ERR_BAD_ARG;
  const Plan pl = make_plan(cfg, batch, max_seq_len, k);
  if (workspace_bytes < pl.total) return ADAMAS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  AttnParams ap{};
  ap.q = static_cast<const uint16_t*>(q);
  ap.K = static_cast<const uint16_t*>(K);
  ap.V = static_cast<const uint16_t*>(V);
  ap.seq_start = seq_start;
  ap.idx = idx;
  ap.out = out;
  ap.partial = reinterpret_cast<float*>(ws_at(workspace, pl.off_partial));
  ap.pool_tokens = cfg->pool_tokens;
  ap.Hq = cfg->num_q_heads;
  ap.Hkv = cfg->num_kv_heads;
  ap.k = k;
  ap.group_magic = group_magic_of(cfg);
  // about 32 rows per workgroup, at most kAttnPartsMax workgroups per head
  int parts = (k + 31) / 32;
  if (parts > kMaxParts) parts = kMaxParts;
  ap.chunk = (k + parts - 1) / parts;
  ap.n_parts = (k + ap.chunk - 1) / ap.chunk;
  ap.scale_log2e = scale_log2e(cfg);
  dim_set_of(cfg).sparse_attn(dim3(ap.n_parts, cfg->num_q_heads, batch), st, ap);
  if (int rc = launch_status()) return rc;
  if (ap.n_parts == 1) return ADAMAS_OK;
  MergeParams mp{};
  mp.partial = ap.partial;
  mp.out = out;
  mp.seq_start = seq_start;
  mp.Hq = cfg->num_q_heads;
  mp.n_parts = ap.n_parts;
  mp.seg_len = 0;
  dim_set_of(cfg).merge(dim3(cfg->num_q_heads, batch), st, mp);
  return launch_status();
}

namespace {
int decode_step_impl(const adamas_config* cfg, const void* q, const void* k_new, const void* v_new,
                     void* K, void* V, void* codes, const int64_t* seq_start,
                     const int32_t* page_table, int32_t max_pages, int32_t page_shift,
                     const int32_t* seq_len, int32_t batch, int32_t k, float* out, int32_t* idx_out,
                     int64_t max_seq_len, void* workspace, size_t workspace_bytes, void* stream,
                     uint32_t stages);
}  // namespace

int adamas_decode_step(const adamas_config* cfg, const void* q, const void* k_new,
                       const void* v_new, void* K, void* V, void* codes, const int64_t* seq_start,
                       const int32_t* seq_len, int32_t batch, int32_t k, float* out,
                       int32_t* idx_out, int64_t max_seq_len, void* workspace,
                       size_t workspace_bytes, void* stream) {
  return adamas_decode_step_stages(cfg, q, k_new, v_new, K, V, codes, seq_start, seq_len, batch, k,
                                   out, idx_out, max_seq_len, workspace, workspace_bytes, stream,
                                   ADAMAS_STAGE_ALL);
}

int adamas_decode_step_static(const adamas_config* cfg, const void* q, const void* k_new,
                              const void* v_new, void* K, void* V, void* codes,
                              const int64_t* seq_start, const int32_t* seq_len, int32_t batch,
                              int32_t k, float* out, int32_t* idx_out, int64_t max_seq_len,
                              void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (int rc = check_sizes(batch, max_seq_len, k)) return rc;
  if (make_plan(cfg, batch, max_seq_len, k).total > (size_t)ADAMAS_STATIC_SCRATCH_BYTES)
    return ADAMAS_ERR_WORKSPACE;
  if (!q || !K || !V || !codes || !seq_start || !seq_len || !out) return ADAMAS_ERR_BAD_ARG;
  void* ws = static_scratch();
  if (ws == nullptr) return ADAMAS_ERR_HIP;
  // Nothing in the scratch has to start at zero: the scan kernel clears the
  // arrival counters it hands to the select kernel, everything else is written
  // before it is read.
  return adamas_decode_step(cfg, q, k_new, v_new, K, V, codes, seq_start, seq_len, batch, k, out,
                            idx_out, max_seq_len, ws, (size_t)ADAMAS_STATIC_SCRATCH_BYTES, stream);
}

int adamas_decode_step_stages(const adamas_config* cfg, const void* q, const void* k_new,
                              const void* v_new, void* K, void* V, void* codes,
                              const int64_t* seq_start, const int32_t* seq_len, int32_t batch,
                              int32_t k, float* out, int32_t* idx_out, int64_t max_seq_len,
                              void* workspace, size_t workspace_bytes, void* stream,
                              uint32_t stages) {
  if (seq_start == nullptr) return ADAMAS_ERR_BAD_ARG;
  return decode_step_impl(cfg, q, k_new, v_new, K, V, codes, seq_start, nullptr, 0, 0, seq_len,
                          batch, k, out, idx_out, max_seq_len, workspace, workspace_bytes, stream,
                          stages);
}

int adamas_decode_step_paged(const adamas_config* cfg, const void* q, const void* k_new,
                             const void* v_new, void* K, void* V, void* codes,
                             const int32_t* page_table, int32_t max_pages, int32_t page_tokens,
                             const int32_t* seq_len, int32_t batch, int32_t k, float* out,
                             int32_t* idx_out, int64_t max_seq_len, void* workspace,
                             size_t workspace_bytes, void* stream, uint32_t stages) {
  if (int rc = check_config(cfg)) return rc;
  if (page_table == nullptr || max_pages < 1) return ADAMAS_ERR_BAD_ARG;
  if (stages != ADAMAS_STAGE_ALL && stages != ADAMAS_STAGE_SCAN) return ADAMAS_ERR_BAD_ARG;
  if (page_tokens < 64 || page_tokens > 4096 || (page_tokens & (page_tokens - 1)) != 0)
    return ADAMAS_ERR_UNSUPPORTED;
  if (cfg->pool_tokens % page_tokens != 0 || cfg->pool_tokens > 0x7fffffff) return ADAMAS_ERR_BAD_ARG;
  if (max_seq_len > (int64_t)max_pages * page_tokens) return ADAMAS_ERR_BAD_ARG;
  int shift = 0;
  while ((1 << shift) < page_tokens) ++shift;
  return decode_step_impl(cfg, q, k_new, v_new, K, V, codes, nullptr, page_table, max_pages, shift,
                          seq_len, batch, k, out, idx_out, max_seq_len, workspace, workspace_bytes,
                          stream, stages);
}

}  // extern "C"

namespace {
int decode_step_impl(const adamas_config* cfg, const void* q, const void* k_new, const void* v_new,
                     void* K, void* V, void* codes, const int64_t* seq_start,
                     const int32_t* page_table, int32_t max_pages, int32_t page_shift,
                     const int32_t* seq_len, int32_t batch, int32_t k, float* out, int32_t* idx_out,
                     int64_t max_seq_len, void* workspace, size_t workspace_bytes, void* stream,
                     uint32_t stages) {
  if (int rc = check_config(cfg)) return rc;
  if (stages < 1u || stages > ADAMAS_STAGE_ALL) return ADAMAS_ERR_BAD_ARG;
  if (int rc = check_sizes(batch, max_seq_len, k)) return rc;
  if (!q || !K || !V || !codes || !seq_len || !out || !workspace) return ADAMAS_ERR_BAD_ARG;
  if (seq_start == nullptr && page_table == nullptr) return ADAMAS_ERR_BAD_ARG;
  if ((k_new == nullptr) != (v_new == nullptr)) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(codes)) return ADAMAS_ERR_BAD_ARG;
  if (k_new && (!aligned16(k_new) || !aligned16(v_new))) return ADAMAS_ERR_BAD_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return ADAMAS_ERR_BAD_ARG;
  const Plan pl = make_plan(cfg, batch, max_seq_len, k);
  if (workspace_bytes < pl.total) return ADAMAS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();

  ScanParams sp{};
  sp.codes = static_cast<const uint8_t*>(codes);
  sp.codes_w = static_cast<uint8_t*>(codes);
  sp.q = static_cast<const uint16_t*>(q);
  sp.k_new = static_cast<const uint16_t*>(k_new);
  sp.v_new = static_cast<const uint16_t*>(v_new);
  sp.K = static_cast<uint16_t*>(K);
  sp.V = static_cast<uint16_t*>(V);
  sp.seq_start = seq_start;
  sp.seq_len = seq_len;
  sp.dist = ws_at(workspace, pl.off_dist);
  sp.dist_high = reinterpret_cast<uint64_t*>(ws_at(workspace, pl.off_high));
  sp.dist_stride = pl.dist_stride;
  sp.tilehist = reinterpret_cast<uint32_t*>(ws_at(workspace, pl.off_hist));
  sp.pool_tokens = cfg->pool_tokens;
  sp.max_seq_len = max_seq_len;
  sp.Hq = cfg->num_q_heads;
  sp.Hkv = cfg->num_kv_heads;
  sp.n_tiles = pl.n_tiles;
  sp.thr_q = scaled(cfg, cfg->thr_q);
  sp.thr_k = scaled(cfg, cfg->thr_k);
  sp.page_table = page_table;
  sp.max_pages = max_pages;
  sp.page_shift = page_shift;
  // segment counters live in the unused words of each head's first partial slot
  sp.arrivals = reinterpret_cast<uint32_t*>(ws_at(workspace, pl.off_partial)) + 2;
  sp.arrivals_stride = (int64_t)kMaxParts * partial_stride(cfg->head_dim);
  sp.trace = g_trace_scan;
  sp.trace_records = g_trace_records;
  if (stages & ADAMAS_STAGE_SCAN) {
    launch_scan(cfg, true, pl, batch, st, sp);
    if (int rc = launch_status()) return rc;
  }
  if (!(stages & ADAMAS_STAGE_SELECT_ATTN)) return ADAMAS_OK;

  SelectParams sl{};
  sl.dist = sp.dist;
  sl.dist_high = sp.dist_high;
  sl.dist_stride = pl.dist_stride;
  sl.tilehist = sp.tilehist;
  sl.seq_start = seq_start;
  sl.seq_len = seq_len;
  sl.idx_out = idx_out;
  sl.q = sp.q;
  sl.K = sp.K;
  sl.V = sp.V;
  sl.out = out;
  sl.partial = reinterpret_cast<float*>(ws_at(workspace, pl.off_partial));
  sl.arrivals = (stages & ADAMAS_STAGE_SCAN) ? sp.arrivals : nullptr;
  sl.arrivals_stride = sp.arrivals_stride;
  sl.pool_tokens = cfg->pool_tokens;
  sl.max_seq_len = max_seq_len;
  sl.Hq = cfg->num_q_heads;
  sl.Hkv = cfg->num_kv_heads;
  sl.k = k;
  sl.group_magic = group_magic_of(cfg);
  sl.n_tiles = pl.n_tiles;
  sl.tile_tokens = pl.tile_tokens;
  sl.seg_len = pl.seg_len;
  sl.tile_shift = log2_of(pl.tile_tokens);
  sl.seg_shift = log2_of(pl.seg_len);
  sl.early_rows = early_rows_pay(pl, (int64_t)batch * cfg->num_q_heads);
  sl.scale_log2e = scale_log2e(cfg);
  sl.page_table = page_table;
  sl.max_pages = max_pages;
  sl.page_shift = page_shift;
  sl.trace = g_trace_select;
  sl.trace_records = g_trace_records;
  set_of(cfg).select(true, page_table != nullptr, dim3(pl.n_segs, cfg->num_q_heads, batch), st, sl);
  if (int rc = launch_status()) return rc;
  if (pl.n_segs == 1 || sl.arrivals != nullptr) return ADAMAS_OK;  // the select kernel wrote `out` itself
  MergeParams mp{};
  mp.partial = sl.partial;
  mp.out = out;
  mp.seq_start = seq_start;
  mp.seq_len = seq_len;
  mp.pool_tokens = cfg->pool_tokens;
  mp.max_seq_len = max_seq_len;
  mp.Hq = cfg->num_q_heads;
  mp.n_parts = pl.n_segs;
  mp.seg_len = pl.seg_len;
  dim_set_of(cfg).merge(dim3(cfg->num_q_heads, batch), st, mp);
  return launch_status();
}
}  // namespace

extern "C" {

size_t adamas_full_attn_workspace_bytes(const adamas_config* cfg, int32_t batch,
                                        int64_t max_seq_len) {
  if (check_config(cfg) != ADAMAS_OK || check_sizes(batch, max_seq_len, 1) != ADAMAS_OK) return 0;
  return make_full_plan(cfg, batch, max_seq_len).total;
}

int adamas_full_attn(const adamas_config* cfg, const void* q, const void* K, const void* V,
                     const int64_t* seq_start, const int32_t* seq_len, int32_t batch, float* out,
                     int64_t max_seq_len, void* workspace, size_t workspace_bytes, void* stream) {
  if (int rc = check_config(cfg)) return rc;
  if (int rc = check_sizes(batch, max_seq_len, 1)) return rc;
  if (!q || !K || !V || !seq_start || !seq_len || !out || !workspace) return ADAMAS_ERR_BAD_ARG;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V)) return ADAMAS_ERR_BAD_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return ADAMAS_ERR_BAD_ARG;
  const FullPlan pl = make_full_plan(cfg, batch, max_seq_len);
  if (workspace_bytes < pl.total) return ADAMAS_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  FullAttnParams fp{};
  fp.q = static_cast<const uint16_t*>(q);
  fp.K = static_cast<const uint16_t*>(K);
  fp.V = static_cast<const uint16_t*>(V);
  fp.seq_start = seq_start;
  fp.seq_len = seq_len;
  fp.partial = static_cast<float*>(workspace);
  fp.pool_tokens = cfg->pool_tokens;
  fp.max_seq_len = max_seq_len;
  fp.Hq = cfg->num_q_heads;
  fp.Hkv = cfg->num_kv_heads;
  fp.n_splits = pl.n_splits;
  fp.chunk = pl.chunk;
  fp.scale_log2e = (float)scale_log2e(cfg);
  const dim3 grid(pl.n_splits, cfg->num_kv_heads, batch);
  dim_set_of(cfg).full_attn(cfg->num_q_heads / cfg->num_kv_heads, grid, st, fp);
  if (int rc = launch_status()) return rc;
  dim_set_of(cfg).merge_parts(dim3(cfg->num_q_heads, batch), st, fp.partial, out, cfg->num_q_heads,
                              pl.n_splits);
  return launch_status();
}

int adamas_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (src == nullptr || sink == nullptr || !aligned16(src) || (bytes & 31u) != 0)
    return ADAMAS_ERR_BAD_ARG;
  if ((reinterpret_cast<uintptr_t>(sink) & 3u) != 0) return ADAMAS_ERR_BAD_ARG;
  if (bytes == 0) return ADAMAS_OK;
  const int64_t n_rows = (int64_t)(bytes / kRowBytes);
  const int64_t rows_per_wg = 256 * 2;
  const int64_t grid = (n_rows + rows_per_wg - 1) / rows_per_wg;
  if (grid > 0x7fffffff) return ADAMAS_ERR_UNSUPPORTED;
  clear_stale_error();
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)grid), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const uint4*>(src), static_cast<uint32_t*>(sink), n_rows);
  return launch_status();
}

}  // extern "C"
