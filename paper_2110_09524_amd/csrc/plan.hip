// Graph plan: device-side validation of the CSR arrays, the CSC transpose
// (stable radix sort by source), and the degree order / degree buckets of both
// sides.  Integer work only; every table is a pure function of the input.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

#include "common.h"

namespace gnn {

// largest value over the wavefront (all 64 lanes take part), then one atomic per wavefront
__device__ __forceinline__ void wave_atomic_max(int* __restrict__ dst, int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
  if ((threadIdx.x & 63) == 0 && v > 0) atomicMax(dst, v);
}

// bad[0]: error flags; bad[1]: the largest in-degree (it sets the width of the degree sort's keys)
__global__ void k_validate_indptr(int32_t n, int64_t nnz, const int32_t* __restrict__ indptr,
                                  int* __restrict__ bad) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  int deg = 0;
  if (i <= n) {
    int32_t a = indptr[i];
    if (i == 0 && a != 0) atomicOr(bad, 1);
    if (i == n && (int64_t)a != nnz) atomicOr(bad, 2);
    if (i < n) {
      deg = indptr[i + 1] - a;
      if (deg < 0) atomicOr(bad, 4);
    }
    if (a < 0 || (int64_t)a > nnz) atomicOr(bad, 4);
  }
  wave_atomic_max(bad + 1, deg);
}

// *out = max(*out, largest of v[0..count))
__global__ void k_max_i32(int64_t count, const int32_t* __restrict__ v, int* __restrict__ out) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  wave_atomic_max(out, i < count ? v[i] : 0);
}

__global__ void k_validate_indices_and_count(int32_t n, int64_t nnz,
                                             const int32_t* __restrict__ indices,
                                             int32_t* __restrict__ outdeg, int* __restrict__ bad) {
  int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  int32_t u = indices[e];
  if (u < 0 || u >= n) {
    atomicOr(bad, 8);
    return;
  }
  atomicAdd(&outdeg[u], 1);  // integer count: the result does not depend on the order
}

__global__ void k_iota(int64_t count, int32_t* __restrict__ out) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < count) out[i] = (int32_t)i;
}

// indices_t[i] = destination row that contains CSR position eid_t[i]
__global__ void k_dst_of_position(int32_t n, int64_t nnz, const int32_t* __restrict__ indptr,
                                  const int32_t* __restrict__ eid_t, int32_t* __restrict__ indices_t) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= nnz) return;
  int32_t p = eid_t[i];
  // largest v with indptr[v] <= p (rows may be empty, so take the upper bound)
  int32_t lo = 0, hi = n;  // invariant: indptr[lo] <= p < indptr[hi]
  while (hi - lo > 1) {
    int32_t mid = lo + ((hi - lo) >> 1);
    if (indptr[mid] <= p) lo = mid; else hi = mid;
  }
  indices_t[i] = lo;
}

// The histogram is counted per workgroup in LDS first, one vote per distinct bucket of a
// wavefront: graphs whose vertices all have the same degree (k-nearest-neighbour graphs) would
// otherwise send every vertex's atomic to one address.
__global__ __launch_bounds__(256) void k_degree_and_bucket(int32_t n, const int32_t* __restrict__ ptr,
                                                           uint32_t* __restrict__ deg,
                                                           int32_t* __restrict__ bucket,
                                                           int32_t* __restrict__ hist) {
  __shared__ int l_hist[GNN_NUM_BUCKETS];
  if (threadIdx.x < GNN_NUM_BUCKETS) l_hist[threadIdx.x] = 0;
  __syncthreads();
  const int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  const bool ok = v < n;
  int b = -1;
  if (ok) {
    const uint32_t d = (uint32_t)(ptr[v + 1] - ptr[v]);
    b = d == 0 ? 32 : __clz((int)d);
    deg[v] = d;
    bucket[v] = b;
  }
  const int lane = threadIdx.x & 63;
  unsigned long long todo = __ballot(ok);
  while (todo) {  // uniform over the wavefront
    const int first = __ffsll((long long)todo) - 1;
    const int bb = __shfl(b, first, 64);
    const unsigned long long same = __ballot(ok && b == bb);
    if (lane == first) atomicAdd(&l_hist[bb], __popcll(same));
    todo &= ~same;
  }
  __syncthreads();
  if (threadIdx.x < GNN_NUM_BUCKETS && l_hist[threadIdx.x] != 0) atomicAdd(&hist[threadIdx.x], l_hist[threadIdx.x]);
}

// key of an edge for the column-blocked order: (block of its column) * n + its row.
// One wavefront per row, lanes strided over the row's edges (coalesced, no search).
__global__ void k_block_keys(int32_t n, int64_t nnz, const int32_t* __restrict__ ptr,
                             const int32_t* __restrict__ cols, int32_t block_cols,
                             uint64_t* __restrict__ keys, int32_t* __restrict__ counts) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 6;
  if (row >= n) return;
  const int32_t beg = ptr[row], end = ptr[row + 1];
  // The lanes of a wavefront share the row, and within a row equal blocks usually sit next to each
  // other (sorted columns): only the first lane of a run of equal blocks adds the run's length
  // (one atomic per run instead of one per edge; integer counts, so the order does not matter).
  for (int32_t i0 = beg; i0 < end; i0 += 64) {
    const int32_t i = i0 + lane;
    const bool valid = i < end;
    const int32_t b = valid ? cols[i] / block_cols : -1;
    const uint64_t key = (uint64_t)(uint32_t)b * (uint64_t)n + (uint64_t)row;
    if (valid) keys[i] = key;
    const int32_t b_prev = __shfl_up(b, 1, 64);
    const bool head = valid && (lane == 0 || b != b_prev);
    const uint64_t heads = __ballot(head);
    const int nvalid = min(64, end - i0);  // the valid lanes are a prefix
    if (head) {
      const uint64_t later = lane == 63 ? 0ull : heads >> (lane + 1);
      const int next = later != 0 ? lane + 1 + __builtin_ctzll(later) : nvalid;
      atomicAdd(&counts[key], next - lane);
    }
  }
}

// bseg[b*n + r] = (bptr[b*n + row], bptr[b*n + row + 1]) with row = order[r]: the blocked
// kernels hand out rows in degree order and read their bounds with one coalesced load
__global__ void k_block_segments(int32_t n, int32_t nblk, const int32_t* __restrict__ bptr,
                                 const int32_t* __restrict__ order, int2* __restrict__ bseg) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= (int64_t)n * nblk) return;
  const int64_t b = i / n, r = i - b * n;
  const int64_t j = b * n + order[r];
  bseg[i] = make_int2(bptr[j], bptr[j + 1]);
}

// dst[i] = src[i * stride]
__global__ void k_gather_strided(int count, const int32_t* __restrict__ src, int64_t stride,
                                 int32_t* __restrict__ dst) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) dst[i] = src[(int64_t)i * stride];
}

// ---- device memory for plan tables and temporaries ---------------------------------------
// Graphs that are rebuilt all the time (a k-nearest-neighbour graph per training step) would
// otherwise spend more time in hipMalloc / hipFree than in the plan kernels.  Blocks of up to
// 64 MB are rounded up to a power of two and, when released, kept on a free list (at most
// 512 MB in total) for the next plan of a similar size; larger blocks go straight to the
// driver.  A block is only released once nothing on the device can still touch it (the
// callers below synchronise first), so handing it out again needs no further care.
constexpr size_t kPoolMaxBlock = (size_t)64 << 20;
constexpr size_t kPoolMaxCached = (size_t)512 << 20;
static std::mutex g_pool_mu;  // guards the three objects below
static std::unordered_multimap<size_t, void*> g_pool_free;  // capacity -> idle block
static std::unordered_map<void*, size_t> g_pool_capacity;   // every pooled block, idle or in use
static size_t g_pool_cached = 0;

static void pool_trim();

static hipError_t pool_alloc(void** out, size_t bytes) {
  *out = nullptr;
  if (bytes == 0) bytes = 1;
  if (bytes > kPoolMaxBlock) {
    hipError_t e = hipMalloc(out, bytes);
    if (e == hipErrorOutOfMemory) {
      (void)hipGetLastError();
      pool_trim();
      e = hipMalloc(out, bytes);
    }
    return e;
  }
  size_t cap = 256;
  while (cap < bytes) cap <<= 1;
  {
    std::lock_guard<std::mutex> lk(g_pool_mu);
    auto it = g_pool_free.find(cap);
    if (it != g_pool_free.end()) {
      *out = it->second;
      g_pool_free.erase(it);
      g_pool_cached -= cap;
      return hipSuccess;
    }
  }
  hipError_t e = hipMalloc(out, cap);
  if (e == hipErrorOutOfMemory) {
    // idle blocks of other sizes may be what fills the device: hand them back and try once more
    (void)hipGetLastError();
    pool_trim();
    e = hipMalloc(out, cap);
  }
  if (e == hipSuccess) {
    std::lock_guard<std::mutex> lk(g_pool_mu);
    g_pool_capacity[*out] = cap;
  }
  return e;
}

// the block must be idle on the device
static void pool_free(void* p) {
  if (!p) return;
  {
    std::lock_guard<std::mutex> lk(g_pool_mu);
    auto it = g_pool_capacity.find(p);
    if (it != g_pool_capacity.end()) {
      if (g_pool_cached + it->second <= kPoolMaxCached) {
        g_pool_free.emplace(it->second, p);
        g_pool_cached += it->second;
        return;
      }
      g_pool_capacity.erase(it);
    }
  }
  (void)hipFree(p);
}

// returns every idle block to the driver
static void pool_trim() {
  std::unordered_multimap<size_t, void*> idle;
  {
    std::lock_guard<std::mutex> lk(g_pool_mu);
    idle.swap(g_pool_free);
    for (auto& kv : idle) g_pool_capacity.erase(kv.second);
    g_pool_cached = 0;
  }
  for (auto& kv : idle) (void)hipFree(kv.second);
}

static void free_all(gnn_graph* g) {
  if (!g) return;
  (void)hipDeviceSynchronize();  // kernels that read the tables have finished (hipFree used to wait, too)
  pool_free(g->indptr_t);
  pool_free(g->indices_t);
  pool_free(g->eid_t);
  for (int s = 0; s < 2; ++s) {
    pool_free(g->bucket_of[s]);
    pool_free(g->order[s]);
    pool_free(g->bucket_offsets[s]);
    pool_free(g->bptr[s]);
    pool_free(g->bcol[s]);
    pool_free(g->bseg[s]);
  }
  pool_free(g->phase_clock);
  delete g;
}

struct TempBuffers {
  void* p[24] = {};
  int count = 0;
  hipStream_t st;
  explicit TempBuffers(hipStream_t stream) : st(stream) {}
  ~TempBuffers() {
    if (count) (void)hipStreamSynchronize(st);  // also on error paths: nothing may still be writing
    for (int i = 0; i < count; ++i) pool_free(p[i]);
  }
  template <typename T>
  hipError_t alloc(T** out, size_t elems) {
    void* q = nullptr;
    *out = nullptr;
    if (count == 24) return hipErrorOutOfMemory;  // more temporaries than slots: a bug, not a device state
    hipError_t e = pool_alloc(&q, elems ? elems * sizeof(T) : sizeof(T));
    if (e == hipSuccess) p[count++] = q;
    *out = static_cast<T*>(q);
    return e;
  }
};

static int bits_for(uint32_t max_value) {
  int b = 1;
  while (b < 32 && (max_value >> b) != 0) ++b;
  return b;
}

// Small results the host needs (error flags, bucket histograms, largest degrees) are copied into
// pinned memory, so that the copies are asynchronous and one wait at the end of the build
// serves all of them.  One staging block per host thread, allocated on first use and kept.
struct PlanStage {
  int32_t hist[2][GNN_NUM_BUCKETS];
  int head[3];  // error flags, largest in-degree, largest out-degree
};
static PlanStage* plan_stage() {
  static thread_local PlanStage* stage = nullptr;
  if (!stage) {
    void* p = nullptr;
    if (hipHostMalloc(&p, sizeof(PlanStage), hipHostMallocDefault) != hipSuccess) return nullptr;
    stage = static_cast<PlanStage*>(p);
  }
  return stage;
}

__global__ void k_bucket_offsets(const int32_t* __restrict__ hist, int32_t* __restrict__ offsets) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int32_t run = 0;
    offsets[0] = 0;
    for (int b = 0; b < GNN_NUM_BUCKETS; ++b) {
      run += hist[b];
      offsets[b + 1] = run;
    }
  }
}

// enqueues the degree order and buckets of one side; finish_side completes it after the wait
static gnn_status_t build_side(gnn_graph* g, int side, const int32_t* ptr, TempBuffers& tmp,
                               PlanStage* stage, hipStream_t st) {
  // the sort's keys are as wide as the largest degree (one 8-bit pass for a kNN graph instead of four)
  const int key_bits = bits_for((uint32_t)g->max_degree[side]);
  const int32_t n = g->n;
  const int thr = 256;
  uint32_t *deg = nullptr, *deg_sorted = nullptr;
  int32_t *ids = nullptr, *hist = nullptr;
  GNN_HIP(tmp.alloc(&deg, n));
  GNN_HIP(tmp.alloc(&deg_sorted, n));
  GNN_HIP(tmp.alloc(&ids, n));
  GNN_HIP(tmp.alloc(&hist, GNN_NUM_BUCKETS));
  GNN_HIP(pool_alloc((void**)&g->bucket_of[side], sizeof(int32_t) * (n ? n : 1)));
  GNN_HIP(pool_alloc((void**)&g->order[side], sizeof(int32_t) * (n ? n : 1)));
  GNN_HIP(pool_alloc((void**)&g->bucket_offsets[side], sizeof(int32_t) * (GNN_NUM_BUCKETS + 1)));
  GNN_HIP(hipMemsetAsync(hist, 0, sizeof(int32_t) * GNN_NUM_BUCKETS, st));
  if (n > 0) {
    k_degree_and_bucket<<<cdiv(n, thr), thr, 0, st>>>(n, ptr, deg, g->bucket_of[side], hist);
    GNN_LAUNCH_CHECK();
  }
  k_bucket_offsets<<<1, 64, 0, st>>>(hist, g->bucket_offsets[side]);
  GNN_LAUNCH_CHECK();
  if (n > 0) {
    k_iota<<<cdiv(n, thr), thr, 0, st>>>(n, ids);
    GNN_LAUNCH_CHECK();
    // stable descending sort by degree: ties keep ascending vertex id
    size_t bytes = 0;
    GNN_HIP(rocprim::radix_sort_pairs_desc(nullptr, bytes, deg, deg_sorted, ids, g->order[side],
                                           (size_t)n, 0, key_bits, st));
    void* scratch = nullptr;
    GNN_HIP(tmp.alloc((char**)&scratch, bytes));
    GNN_HIP(rocprim::radix_sort_pairs_desc(scratch, bytes, deg, deg_sorted, ids, g->order[side],
                                           (size_t)n, 0, key_bits, st));
    GNN_HIP(hipMemcpyAsync(stage->hist[side], hist, sizeof(stage->hist[side]), hipMemcpyDeviceToHost, st));
  }
  return GNN_OK;
}

// after the stream has been waited for: the host copies of the bucket table
static void finish_side(gnn_graph* g, int side, const PlanStage* stage) {
  g->h_bucket_offsets[side][0] = 0;
  for (int b = 0; b < GNN_NUM_BUCKETS; ++b)
    g->h_bucket_offsets[side][b + 1] = g->h_bucket_offsets[side][b] + stage->hist[side][b];
}

// Column-blocked copy of one side's edge list: edges stable-sorted by
// (column / block_cols, row); bptr[b*n + r] .. bptr[b*n + r + 1] is the range of
// row r inside block b.  Only built when the vertex set spans several blocks.

// Launch groups of the column-blocked kernels.  One launch over w adjacent blocks costs, in units
// of one gathered edge per row: a fixed part (the row's running sums are read and written once,
// its segment bounds and scalars fetched) plus d * (1 + spill * log2(columns / 24576)) for its d
// edges per row, because a wider set of gathered row slices no longer sits in the L2.  Measured
// with the Reddit-scale GAT layer (1 KB rows): the per-edge part grows from 0.076 ms per million
// edges at 24576 columns to 0.099 at twice and 0.128 at four times that; the fixed part that
// gives the fastest partition is worth 8 to 12 gathered rows per row for kernels with two running
// sums (of 4, 8, 12, 16, 24 tried), about half of that with one.  The partition of the block
// sequence with the least total cost comes from a dynamic programme; it merges the sparse tail
// blocks of a power-law graph and leaves dense blocks alone.
static std::vector<int32_t> launch_groups(const std::vector<int32_t>& begin, int32_t n, int32_t block_cols,
                                          bool merge, double kFixed) {
  constexpr double kSpill = 0.32, kFitCols = 24576.0;
  const int nb = (int)begin.size() - 1;
  std::vector<int32_t> groups;
  if (nb < 1) return groups;
  if (!merge || n <= 0) {
    for (int b = 0; b <= nb; ++b) groups.push_back(b);
    return groups;
  }
  std::vector<double> best((size_t)nb + 1, 0.0);
  std::vector<int> width((size_t)nb + 1, 1);
  for (int e = 1; e <= nb; ++e) {
    best[e] = -1.0;
    for (int w = 1; w <= kMaxMerge && w <= e; ++w) {
      const double d = (double)((int64_t)begin[e] - begin[e - w]) / (double)n;
      const double over = std::log2((double)w * (double)block_cols / kFitCols);
      const double c = best[e - w] + kFixed + d * (1.0 + kSpill * (over > 0.0 ? over : 0.0));
      if (best[e] < 0.0 || c < best[e]) {
        best[e] = c;
        width[e] = w;
      }
    }
  }
  for (int e = nb; e > 0; e -= width[e]) groups.push_back(e);
  groups.push_back(0);
  std::reverse(groups.begin(), groups.end());
  return groups;
}

static gnn_status_t build_blocked(gnn_graph* g, int side, const int32_t* ptr, const int32_t* cols,
                                  hipStream_t st) {
  const int32_t n = g->n;
  const int64_t nnz = g->nnz;
  const int thr = 256;
  const int64_t slots = (int64_t)g->nblk * n;
  TempBuffers tmp(st);
  uint64_t *keys = nullptr, *keys_sorted = nullptr;
  int32_t* counts = nullptr;
  GNN_HIP(tmp.alloc(&keys, (size_t)nnz));
  GNN_HIP(tmp.alloc(&keys_sorted, (size_t)nnz));
  GNN_HIP(tmp.alloc(&counts, (size_t)slots + 1));
  GNN_HIP(pool_alloc((void**)&g->bptr[side], sizeof(int32_t) * ((size_t)slots + 1)));
  GNN_HIP(pool_alloc((void**)&g->bcol[side], sizeof(int32_t) * (size_t)nnz));
  GNN_HIP(hipMemsetAsync(counts, 0, sizeof(int32_t) * ((size_t)slots + 1), st));
  k_block_keys<<<cdiv((int64_t)n * 64, thr), thr, 0, st>>>(n, nnz, ptr, cols, g->block_cols, keys, counts);
  GNN_LAUNCH_CHECK();
  {
    size_t bytes = 0;
    GNN_HIP(rocprim::exclusive_scan(nullptr, bytes, counts, g->bptr[side], (int32_t)0,
                                    (size_t)slots + 1, rocprim::plus<int32_t>(), st));
    void* scratch = nullptr;
    GNN_HIP(tmp.alloc((char**)&scratch, bytes));
    GNN_HIP(rocprim::exclusive_scan(scratch, bytes, counts, g->bptr[side], (int32_t)0,
                                    (size_t)slots + 1, rocprim::plus<int32_t>(), st));
  }
  {
    int end_bit = 1;
    while (end_bit < 64 && ((uint64_t)(slots - 1) >> end_bit) != 0) ++end_bit;
    size_t bytes = 0;
    GNN_HIP(rocprim::radix_sort_pairs(nullptr, bytes, keys, keys_sorted, cols, g->bcol[side],
                                      (size_t)nnz, 0, end_bit, st));
    void* scratch = nullptr;
    GNN_HIP(tmp.alloc((char**)&scratch, bytes));
    GNN_HIP(rocprim::radix_sort_pairs(scratch, bytes, keys, keys_sorted, cols, g->bcol[side],
                                      (size_t)nnz, 0, end_bit, st));
  }
  GNN_HIP(pool_alloc((void**)&g->bseg[side], sizeof(int32_t) * 2 * (size_t)slots));
  k_block_segments<<<cdiv(slots, thr), thr, 0, st>>>(n, g->nblk, g->bptr[side], g->order[side],
                                                     reinterpret_cast<int2*>(g->bseg[side]));
  GNN_LAUNCH_CHECK();
  // edges per block, for the host's choice of kernel variant: bptr[b * n], b = 0 .. nblk
  g->h_block_begin[side].assign((size_t)g->nblk + 1, 0);
  int32_t* starts = nullptr;
  GNN_HIP(tmp.alloc(&starts, (size_t)g->nblk + 1));
  k_gather_strided<<<cdiv((int64_t)g->nblk + 1, thr), thr, 0, st>>>(g->nblk + 1, g->bptr[side], n, starts);
  GNN_LAUNCH_CHECK();
  GNN_HIP(hipMemcpyAsync(g->h_block_begin[side].data(), starts, sizeof(int32_t) * ((size_t)g->nblk + 1),
                         hipMemcpyDeviceToHost, st));
  GNN_HIP(hipStreamSynchronize(st));
  const bool merge = config_get(kCfgMergeBlocks) != 0;
  g->h_group[side][0] = launch_groups(g->h_block_begin[side], n, g->block_cols, merge, 6.0);
  g->h_group[side][1] = launch_groups(g->h_block_begin[side], n, g->block_cols, merge, 10.0);
  return GNN_OK;
}

static gnn_status_t build(gnn_graph* g, hipStream_t st) {
  const int32_t n = g->n;
  const int64_t nnz = g->nnz;
  const int thr = 256;
  TempBuffers tmp(st);
  PlanStage* stage = plan_stage();
  GNN_REQUIRE(stage != nullptr, GNN_ERR_HIP, "gnn_graph_create: no pinned staging memory");
  std::memset(stage, 0, sizeof(PlanStage));
  int* bad = nullptr;
  GNN_HIP(tmp.alloc(&bad, 3));  // error flags, largest in-degree, largest out-degree
  GNN_HIP(hipMemsetAsync(bad, 0, 3 * sizeof(int), st));

  GNN_HIP(pool_alloc((void**)&g->indptr_t, sizeof(int32_t) * (size_t)(n + 1)));
  GNN_HIP(pool_alloc((void**)&g->indices_t, sizeof(int32_t) * (size_t)(nnz ? nnz : 1)));
  GNN_HIP(pool_alloc((void**)&g->eid_t, sizeof(int32_t) * (size_t)(nnz ? nnz : 1)));

  int32_t* outdeg = nullptr;
  GNN_HIP(tmp.alloc(&outdeg, (size_t)n + 1));
  GNN_HIP(hipMemsetAsync(outdeg, 0, sizeof(int32_t) * ((size_t)n + 1), st));

  k_validate_indptr<<<cdiv((int64_t)n + 1, thr), thr, 0, st>>>(n, nnz, g->indptr, bad);
  GNN_LAUNCH_CHECK();
  if (nnz > 0) {
    k_validate_indices_and_count<<<cdiv(nnz, thr), thr, 0, st>>>(n, nnz, g->indices, outdeg, bad);
    GNN_LAUNCH_CHECK();
    k_max_i32<<<cdiv((int64_t)n, thr), thr, 0, st>>>(n, outdeg, bad + 2);
    GNN_LAUNCH_CHECK();
  }
  // the kernels below index with the source ids, so this one has to be waited for
  GNN_HIP(hipMemcpyAsync(stage->head, bad, sizeof(stage->head), hipMemcpyDeviceToHost, st));
  GNN_HIP(hipStreamSynchronize(st));
  const int h_bad = stage->head[0];
  g->max_degree[0] = stage->head[1];
  g->max_degree[1] = stage->head[2];
  GNN_REQUIRE(h_bad == 0, GNN_ERR_BAD_GRAPH,
              "gnn_graph_create: malformed CSR (%s%s%s%s)", (h_bad & 1) ? "indptr[0] != 0; " : "",
              (h_bad & 2) ? "indptr[n] != nnz; " : "", (h_bad & 4) ? "indptr not monotone; " : "",
              (h_bad & 8) ? "source id outside [0, n)" : "");

  // indptr_t = exclusive prefix sum of the out-degrees (n+1 entries; the last input is 0)
  {
    size_t bytes = 0;
    GNN_HIP(rocprim::exclusive_scan(nullptr, bytes, outdeg, g->indptr_t, (int32_t)0, (size_t)n + 1,
                                    rocprim::plus<int32_t>(), st));
    void* scratch = nullptr;
    GNN_HIP(tmp.alloc((char**)&scratch, bytes));
    GNN_HIP(rocprim::exclusive_scan(scratch, bytes, outdeg, g->indptr_t, (int32_t)0, (size_t)n + 1,
                                    rocprim::plus<int32_t>(), st));
  }
  if (nnz > 0) {
    // stable sort of (source, CSR position): positions stay ascending inside a source
    uint32_t* keys_out = nullptr;
    int32_t* pos = nullptr;
    GNN_HIP(tmp.alloc(&keys_out, (size_t)nnz));
    GNN_HIP(tmp.alloc(&pos, (size_t)nnz));
    k_iota<<<cdiv(nnz, thr), thr, 0, st>>>(nnz, pos);
    GNN_LAUNCH_CHECK();
    const uint32_t* keys_in = reinterpret_cast<const uint32_t*>(g->indices);
    const int end_bit = bits_for(n > 0 ? (uint32_t)(n - 1) : 0u);
    size_t bytes = 0;
    GNN_HIP(rocprim::radix_sort_pairs(nullptr, bytes, keys_in, keys_out, pos, g->eid_t, (size_t)nnz,
                                      0, end_bit, st));
    void* scratch = nullptr;
    GNN_HIP(tmp.alloc((char**)&scratch, bytes));
    GNN_HIP(rocprim::radix_sort_pairs(scratch, bytes, keys_in, keys_out, pos, g->eid_t, (size_t)nnz,
                                      0, end_bit, st));
    k_dst_of_position<<<cdiv(nnz, thr), thr, 0, st>>>(n, nnz, g->indptr, g->eid_t, g->indices_t);
    GNN_LAUNCH_CHECK();
  }
  GNN_TRY(build_side(g, 0, g->indptr, tmp, stage, st));
  GNN_TRY(build_side(g, 1, g->indptr_t, tmp, stage, st));
  g->block_cols = (int32_t)config_get(kCfgBlockCols);
  g->nblk = 1;
  // the (block, row) pointer table has nblk * n entries: keep it below 2^28.  A graph too sparse
  // for the column-blocked kernels to pay (fewer than "blocked_min_edges" edges per row and block:
  // a kNN graph rebuilt every step, say) gets no lists, which are most of a small plan's launches.
  if (g->block_cols > 0 && n > g->block_cols && nnz > 0 &&
      cdiv(n, g->block_cols) * (int64_t)n < ((int64_t)1 << 28) &&
      nnz >= config_get(kCfgBlockedMinEdges) * (int64_t)n * cdiv(n, g->block_cols)) {
    g->nblk = (int32_t)cdiv(n, g->block_cols);
    GNN_TRY(build_blocked(g, 0, g->indptr, g->indices, st));
    GNN_TRY(build_blocked(g, 1, g->indptr_t, g->indices_t, st));
    GNN_HIP(pool_alloc((void**)&g->phase_clock, sizeof(int32_t) * kXcds * kClockStride));
  }
  GNN_HIP(hipStreamSynchronize(st));
  finish_side(g, 0, stage);
  finish_side(g, 1, stage);
  return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" gnn_status_t gnn_release_cached_memory(void) {
  clear_error();
  pool_trim();
  return GNN_OK;
}

extern "C" gnn_status_t gnn_graph_create(int32_t n, int64_t nnz, const int32_t* indptr,
                                         const int32_t* indices, void* stream, gnn_graph_t** graph) {
  clear_error();
  GNN_REQUIRE(graph != nullptr, GNN_ERR_INVALID_ARG, "gnn_graph_create: graph is null");
  *graph = nullptr;
  GNN_REQUIRE(n >= 0 && nnz >= 0, GNN_ERR_INVALID_ARG, "gnn_graph_create: negative size");
  GNN_REQUIRE(nnz < (int64_t)INT32_MAX, GNN_ERR_UNSUPPORTED,
              "gnn_graph_create: nnz = %lld does not fit 32-bit edge offsets", (long long)nnz);
  GNN_REQUIRE(indptr != nullptr, GNN_ERR_INVALID_ARG, "gnn_graph_create: indptr is null");
  GNN_REQUIRE(indices != nullptr || nnz == 0, GNN_ERR_INVALID_ARG,
              "gnn_graph_create: indices is null");
  gnn_graph* g = new gnn_graph();
  g->n = n;
  g->nnz = nnz;
  g->indptr = indptr;
  g->indices = indices;
  g->gcn_edge_balanced[0] = g->gcn_edge_balanced[1] = -1;
  g->gmm_edge_balanced = -1;
  g->gmm_bwd_edge_balanced[0] = g->gmm_bwd_edge_balanced[1] = -1;
  gnn_status_t s = build(g, static_cast<hipStream_t>(stream));
  if (s != GNN_OK) {
    free_all(g);
    return s;
  }
  *graph = g;
  return GNN_OK;
}

extern "C" gnn_status_t gnn_graph_destroy(gnn_graph_t* graph) {
  clear_error();
  free_all(graph);
  return GNN_OK;
}

// ---- static edge weights -----------------------------------------------------------------
__global__ void k_block_keys_only(int32_t n, const int32_t* __restrict__ ptr, const int32_t* __restrict__ cols,
                                  int32_t block_cols, uint64_t* __restrict__ keys) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 6;
  if (row >= n) return;
  const int32_t beg = ptr[row], end = ptr[row + 1];
  for (int32_t i = beg + lane; i < end; i += 64)
    keys[i] = (uint64_t)(cols[i] / block_cols) * (uint64_t)n + (uint64_t)row;
}

__global__ void k_gather_f32(int64_t count, const int32_t* __restrict__ idx, const float* __restrict__ src,
                             float* __restrict__ dst) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < count) dst[i] = src[idx[i]];
}

static void free_weights(gnn_edge_weights* w) {
  if (!w) return;
  (void)hipDeviceSynchronize();  // kernels that read the copies have finished
  for (int s = 0; s < 2; ++s) {
    pool_free(w->w_side[s]);
    pool_free(w->w_blk[s]);
  }
  delete w;
}

static gnn_status_t build_weights(gnn_edge_weights* w, const float* edge_w, hipStream_t st) {
  const gnn_graph* g = w->graph;
  const int64_t nnz = g->nnz;
  const int thr = 256;
  if (nnz == 0) return GNN_OK;
  for (int s = 0; s < 2; ++s) GNN_HIP(pool_alloc((void**)&w->w_side[s], sizeof(float) * (size_t)nnz));
  GNN_HIP(hipMemcpyAsync(w->w_side[0], edge_w, sizeof(float) * (size_t)nnz, hipMemcpyDeviceToDevice, st));
  k_gather_f32<<<(unsigned)cdiv(nnz, thr), thr, 0, st>>>(nnz, g->eid_t, edge_w, w->w_side[1]);
  GNN_LAUNCH_CHECK();
  if (g->nblk > 1) {
    // The blocked lists are a stable sort of each side's edges by (column block, row); sorting the
    // weights with the same keys and the same stable radix sort puts them in the same order.
    TempBuffers tmp(st);
    uint64_t *keys = nullptr, *keys_sorted = nullptr;
    GNN_HIP(tmp.alloc(&keys, (size_t)nnz));
    GNN_HIP(tmp.alloc(&keys_sorted, (size_t)nnz));
    const int64_t slots = (int64_t)g->nblk * g->n;
    int end_bit = 1;
    while (end_bit < 64 && ((uint64_t)(slots - 1) >> end_bit) != 0) ++end_bit;
    for (int s = 0; s < 2; ++s) {
      GNN_HIP(pool_alloc((void**)&w->w_blk[s], sizeof(float) * (size_t)nnz));
      const int32_t* ptr = s == 0 ? g->indptr : g->indptr_t;
      const int32_t* cols = s == 0 ? g->indices : g->indices_t;
      k_block_keys_only<<<(unsigned)cdiv((int64_t)g->n * 64, thr), thr, 0, st>>>(g->n, ptr, cols, g->block_cols, keys);
      GNN_LAUNCH_CHECK();
      size_t bytes = 0;
      GNN_HIP(rocprim::radix_sort_pairs(nullptr, bytes, keys, keys_sorted, w->w_side[s], w->w_blk[s],
                                        (size_t)nnz, 0, end_bit, st));
      void* scratch = nullptr;
      GNN_HIP(tmp.alloc((char**)&scratch, bytes));
      GNN_HIP(rocprim::radix_sort_pairs(scratch, bytes, keys, keys_sorted, w->w_side[s], w->w_blk[s],
                                        (size_t)nnz, 0, end_bit, st));
    }
  }
  GNN_HIP(hipStreamSynchronize(st));
  return GNN_OK;
}

extern "C" gnn_status_t gnn_edge_weights_create(const gnn_graph_t* g, const float* edge_w, void* stream,
                                                gnn_edge_weights_t** out) {
  clear_error();
  GNN_REQUIRE(g != nullptr && out != nullptr, GNN_ERR_INVALID_ARG, "gnn_edge_weights_create: null argument");
  GNN_REQUIRE(g->nnz == 0 || edge_w != nullptr, GNN_ERR_INVALID_ARG, "gnn_edge_weights_create: edge_w is null");
  *out = nullptr;
  gnn_edge_weights* w = new (std::nothrow) gnn_edge_weights();
  GNN_REQUIRE(w != nullptr, GNN_ERR_HIP, "gnn_edge_weights_create: out of host memory");
  w->graph = g;
  w->nnz = g->nnz;
  w->w_side[0] = w->w_side[1] = w->w_blk[0] = w->w_blk[1] = nullptr;
  gnn_status_t s = build_weights(w, edge_w, static_cast<hipStream_t>(stream));
  if (s != GNN_OK) {
    free_weights(w);
    return s;
  }
  *out = w;
  return GNN_OK;
}

extern "C" gnn_status_t gnn_edge_weights_destroy(gnn_edge_weights_t* w) {
  clear_error();
  free_weights(w);
  return GNN_OK;
}

extern "C" gnn_status_t gnn_graph_get_csc(const gnn_graph_t* g, int32_t* indptr_t, int32_t* indices_t,
                                          int32_t* eid_t, void* stream) {
  clear_error();
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "gnn_graph_get_csc: graph is null");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (indptr_t)
    GNN_HIP(hipMemcpyAsync(indptr_t, g->indptr_t, sizeof(int32_t) * ((size_t)g->n + 1),
                           hipMemcpyDeviceToDevice, st));
  if (indices_t && g->nnz)
    GNN_HIP(hipMemcpyAsync(indices_t, g->indices_t, sizeof(int32_t) * (size_t)g->nnz,
                           hipMemcpyDeviceToDevice, st));
  if (eid_t && g->nnz)
    GNN_HIP(hipMemcpyAsync(eid_t, g->eid_t, sizeof(int32_t) * (size_t)g->nnz,
                           hipMemcpyDeviceToDevice, st));
  return GNN_OK;
}

extern "C" gnn_status_t gnn_graph_get_buckets(const gnn_graph_t* g, int side, int32_t* bucket_of_vertex,
                                              int32_t* order, int32_t* bucket_offsets, void* stream) {
  clear_error();
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "gnn_graph_get_buckets: graph is null");
  GNN_REQUIRE(side == 0 || side == 1, GNN_ERR_INVALID_ARG, "gnn_graph_get_buckets: side must be 0 or 1");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (bucket_of_vertex && g->n)
    GNN_HIP(hipMemcpyAsync(bucket_of_vertex, g->bucket_of[side], sizeof(int32_t) * (size_t)g->n,
                           hipMemcpyDeviceToDevice, st));
  if (order && g->n)
    GNN_HIP(hipMemcpyAsync(order, g->order[side], sizeof(int32_t) * (size_t)g->n,
                           hipMemcpyDeviceToDevice, st));
  if (bucket_offsets)
    GNN_HIP(hipMemcpyAsync(bucket_offsets, g->bucket_offsets[side],
                           sizeof(int32_t) * (GNN_NUM_BUCKETS + 1), hipMemcpyDeviceToDevice, st));
  return GNN_OK;
}

extern "C" gnn_status_t gnn_graph_get_blocked(const gnn_graph_t* g, int side, int32_t* num_blocks,
                                              int32_t* block_cols, int32_t* bptr, int32_t* bcol,
                                              void* stream) {
  clear_error();
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "gnn_graph_get_blocked: graph is null");
  GNN_REQUIRE(side == 0 || side == 1, GNN_ERR_INVALID_ARG, "gnn_graph_get_blocked: side must be 0 or 1");
  if (num_blocks) *num_blocks = g->nblk;
  if (block_cols) *block_cols = g->block_cols;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (g->nblk > 1) {
    if (bptr)
      GNN_HIP(hipMemcpyAsync(bptr, g->bptr[side], sizeof(int32_t) * ((size_t)g->nblk * g->n + 1),
                             hipMemcpyDeviceToDevice, st));
    if (bcol)
      GNN_HIP(hipMemcpyAsync(bcol, g->bcol[side], sizeof(int32_t) * (size_t)g->nnz,
                             hipMemcpyDeviceToDevice, st));
  }
  return GNN_OK;
}

extern "C" gnn_status_t gnn_graph_get_launch_groups(const gnn_graph_t* g, int side, int sums,
                                                    int32_t* groups, int32_t* count) {
  clear_error();
  GNN_REQUIRE(g != nullptr && count != nullptr, GNN_ERR_INVALID_ARG, "gnn_graph_get_launch_groups: null argument");
  GNN_REQUIRE(side == 0 || side == 1, GNN_ERR_INVALID_ARG, "gnn_graph_get_launch_groups: side must be 0 or 1");
  GNN_REQUIRE(sums == 1 || sums == 2, GNN_ERR_INVALID_ARG, "gnn_graph_get_launch_groups: sums must be 1 or 2");
  const std::vector<int32_t>& v = g->h_group[side][sums - 1];
  *count = v.empty() ? 0 : (int32_t)v.size() - 1;
  if (groups)
    for (size_t i = 0; i < v.size(); ++i) groups[i] = v[i];
  return GNN_OK;
}
