// Shared host-side plumbing: error text, HIP checks, the timed-launch bracket,
// the graph handle, and the few device helpers every kernel file uses.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "gnn_fused.h"

namespace gnn {

constexpr int kWave = 64;

// ---- error reporting --------------------------------------------------------
void set_error(const char* fmt, ...);
void clear_error();

#define GNN_HIP(expr)                                                                  \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) {                                                            \
      ::gnn::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                       __LINE__);                                                      \
      return GNN_ERR_HIP;                                                              \
    }                                                                                  \
  } while (0)

#define GNN_REQUIRE(cond, status, ...) \
  do {                                 \
    if (!(cond)) {                     \
      ::gnn::set_error(__VA_ARGS__);   \
      return (status);                 \
    }                                  \
  } while (0)

#define GNN_TRY(expr)                 \
  do {                                \
    gnn_status_t s_ = (expr);         \
    if (s_ != GNN_OK) return s_;      \
  } while (0)

// ---- timed launches ---------------------------------------------------------
// prof_begin/prof_end record HIP events around a launch when profiling is on.  The
// bookkeeping is process-wide and guarded by a mutex; prof_begin returns the slot of the
// bracket (-1 when profiling is off or no event could be created).
int64_t prof_begin(const char* name, hipStream_t s);
void prof_end(int64_t slot, hipStream_t s);

struct ProfScope {
  hipStream_t s;
  int64_t slot;
  ProfScope(const char* name, hipStream_t st) : s(st), slot(prof_begin(name, st)) {}
  ~ProfScope() { prof_end(slot, s); }
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;
};

// Call right after a kernel launch.
#define GNN_LAUNCH_CHECK() GNN_HIP(hipGetLastError())

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace (256-byte granules).
struct Workspace {
  char* base;
  size_t size, used;
  Workspace(void* p, size_t n) : base(static_cast<char*>(p)), size(n), used(0) {}
  template <typename T>
  T* take(size_t count) {
    size_t bytes = align_up(count * sizeof(T), 256);
    T* r = reinterpret_cast<T*>(base + used);
    used += bytes;
    return r;
  }
  bool ok() const { return used <= size && (base != nullptr || used == 0); }
};
inline size_t ws_granule(size_t bytes) { return align_up(bytes, 256); }

// most column blocks one launch of a blocked kernel covers
constexpr int kMaxMerge = 8;
// step counters of the persistent kernels: kClockStride ints apart, one per XCD
constexpr int kXcds = 8;
constexpr int kClockStride = 32;

// ---- tuning knobs (runtime.hip) -------------------------------------------------
enum ConfigKey { kCfgBlockCols = 0, kCfgForceSimple = 1, kCfgLdsScalarTable = 2, kCfgGcnMapping = 3, kCfgGmmMapping = 4, kCfgBlockedMinEdges = 5,
                 kCfgGatherPrecision = 6, kCfgMergeBlocks = 7, kCfgWideOffsets = 8, kCfgResidentSums = 9, kCfgResidentSpin = 10, kCfgResidentSyncEvery = 11, kCfgCount };
int64_t config_get(ConfigKey k);
int device_cu_count();  // compute units of the current device (256 when the query fails)

// ---- dense products (gemm.hip) ------------------------------------------------
// c[M,N] = op(a) op(b), fp32 MFMA.  a_kmajor: a is stored [K,M] (m contiguous)
// instead of [M,K]; b_kcontig: b is stored [N,K] (k contiguous) instead of [K,N].
// split_k > 1 writes split_k partial products into `partials` and sums them in a
// fixed order (deterministic).  partials needs split_k*M*N floats.
gnn_status_t gemm_f32(int64_t M, int N, int64_t K, const float* a, int64_t lda, bool a_kmajor,
                      const float* b, int64_t ldb, bool b_kcontig, float* c, int64_t ldc,
                      int split_k, float* partials, hipStream_t s);
int gemm_pick_split_k(int64_t M, int N, int64_t K);
// z[M, heads*f] = x[M, K] w[K, heads*f] with the attention halves el = <a_l, z>, er = <a_r, z> ([M, heads])
// taken from the accumulators; gemm_attn_epilogue_ok says for which head widths this exists
bool gemm_attn_epilogue_ok(int heads, int f);
gnn_status_t gemm_f32_attn(int64_t M, int heads, int f, int64_t K, const float* x, const float* w,
                           const float* a_l, const float* a_r, float* z, float* el, float* er,
                           hipStream_t s);
// out[i] = sum over z < parts of partials[z*count + i], in a fixed order (reproducible)
gnn_status_t sum_partials(int64_t count, int parts, const float* partials, float* out, hipStream_t s);
constexpr int kSumChunk = 64;
int sum_partials_scratch_rows(int parts);
// two levels for very many parts; scratch holds sum_partials_scratch_rows(parts) * count floats
gnn_status_t sum_partials_two_level(int64_t count, int parts, const float* partials, float* scratch,
                                    float* out, hipStream_t s);
// same with a distance of `stride` floats between consecutive parts
gnn_status_t sum_partials_strided(int64_t count, int parts, const float* partials, int64_t stride,
                                  float* out, hipStream_t s);
// partials is [parts][2][count]: first halves into out0, second halves into out1, one launch
gnn_status_t sum_partials_pair(int64_t count, int parts, const float* partials, float* out0, float* out1,
                               hipStream_t s);

}  // namespace gnn

// Static scalar per edge (App. A.2 "GCN": e_uv), copied once into every order the kernels walk.
struct gnn_edge_weights {
  const gnn_graph* graph;
  int64_t nnz;
  float* w_side[2];  // side 0: CSR order (as given); side 1: order of the CSC transpose
  float* w_blk[2];   // order of the column-blocked edge list of each side; null without blocks
};

// The graph handle: borrowed CSR plus the plan tables it owns.
struct gnn_graph {
  int32_t n;
  int64_t nnz;
  const int32_t* indptr;   // borrowed
  const int32_t* indices;  // borrowed
  int32_t* indptr_t;       // owned from here on
  int32_t* indices_t;
  int32_t* eid_t;
  int32_t* bucket_of[2];
  int32_t* order[2];
  int32_t* bucket_offsets[2];            // device copies
  int32_t h_bucket_offsets[2][GNN_NUM_BUCKETS + 1];  // host copies
  int32_t max_degree[2];
  // column-blocked edge lists (present when nblk > 1)
  int32_t block_cols;
  int32_t nblk;
  int32_t* bptr[2];
  int32_t* bcol[2];
  int32_t* bseg[2];  // (begin, end) of row order[r] in block b at [b*n + r], two ints each
  // Step counters of the persistent ("resident sums") kernels, one per XCD on a 128-byte line of
  // its own; a launch zeroes them first.  Calls on one graph that overlap in time share them:
  // their results stay right (the counters only pace the workgroups), their cache hit rates suffer.
  int32_t* phase_clock;
  std::vector<int32_t> h_block_begin[2];  // host: first edge of block b (nblk + 1 entries)
  // Launch groups of the column-blocked kernels: group j covers the blocks h_group[side][a][j] ..
  // h_group[side][a][j + 1] - 1 in one launch (adjacent sparse blocks are merged, so that a row's
  // running sums are read and written once for all of them); a = 0 for kernels that keep one
  // running sum per row, 1 for those that keep two.
  std::vector<int32_t> h_group[2][2];
  // The column-blocked kernels visit every row once per block; that pays only when a row has
  // enough edges inside a block (configuration key "blocked_min_edges", mean over rows and blocks).
  bool blocked_pays() const {
    return nblk > 1 && nnz >= gnn::config_get(gnn::kCfgBlockedMinEdges) * (int64_t)n * nblk;
  }
  int8_t gcn_edge_balanced[2];  // per side: -1 not tuned, 0 / 1 what gnn_gcn_tune found faster
  int8_t gmm_edge_balanced;     // forward aggregation: -1 not tuned, 0 / 1 what gnn_gmm_tune found faster
  int8_t gmm_bwd_edge_balanced[2];  // backward, destination / source side: the same from gnn_gmm_tune_bwd
};
