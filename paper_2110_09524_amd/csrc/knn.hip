// k-nearest-neighbour graph of batched point clouds, built on the GPU (the EdgeConv model of
// Sec. 7.2 derives its graph from the points: k = 20 / 40 neighbours inside each cloud of a
// batch; the paper counts this construction as part of an end-to-end step).
//
// Definition: for every point the k points of its own cloud with the smallest squared
// Euclidean distance, itself included, ties towards the lower index; edges run from the
// neighbours to the point, so the result is the CSR by destination with k sources per row,
// ascending.  Floating point decides integers here, so the arithmetic is pinned down: the
// squared distance is accumulated in float32, coordinate by coordinate in index order, every
// subtraction, product and sum rounded on its own (no fused multiply-add).
//
// One wavefront per query point, no LDS and no cross-lane data movement: lane l keeps the
// distance bits of candidates l, l+64, ... in registers (non-negative floats order like
// unsigned integers).  The k-th smallest distance T is found by bisection on the 32-bit
// pattern; each probe counts the candidates at or below it with one wave-wide vote and a
// scalar population count per register slot.  Everything below T is chosen, and of the
// candidates exactly at T the lowest indices fill up to k.  Positions in the output row come
// from the same votes (candidates before me that are chosen), which leaves the row in
// ascending index order because index = lane + 64 * slot.
#include "common.h"

namespace gnn {

constexpr int kKnnThreads = 256;
constexpr int kKnnQueries = kKnnThreads / kWave;
constexpr int kKnnMaxPoints = 2048;  // 32 register slots per lane
constexpr uint32_t kKeyNone = 0xFFFFFFFFu;  // above every distance pattern

template <int NSLOT>
__global__ __launch_bounds__(kKnnThreads) void k_knn(int64_t n, int points, int dim, int k,
                                                     const float* __restrict__ coords,
                                                     int32_t* __restrict__ indices) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t q = (int64_t)blockIdx.x * kKnnQueries + w;
  if (q >= n) return;  // whole wavefront
  const int64_t base = q / points * points;
  const float* a = coords + q * dim;

  uint32_t key[NSLOT];
#pragma unroll
  for (int t = 0; t < NSLOT; ++t) {
    const int j = lane + kWave * t;
    uint32_t bits = kKeyNone;
    if (j < points) {
      const float* b = coords + (base + j) * dim;
      float acc = 0.f;
      for (int d = 0; d < dim; ++d) {
        const float diff = __fsub_rn(a[d], b[d]);
        const float sq = __fmul_rn(diff, diff);
        acc = d == 0 ? sq : __fadd_rn(acc, sq);
      }
      bits = __float_as_uint(acc);
    }
    key[t] = bits;
  }

  // T = the smallest pattern with at least k candidates at or below it; the count is uniform
  // over the wavefront, so this loop is scalar control flow
  uint32_t lo = 0u, hi = kKeyNone - 1u;  // all `points` >= k candidates are <= hi
  while (lo < hi) {
    const uint32_t mid = lo + ((hi - lo) >> 1);
    int cnt = 0;
#pragma unroll
    for (int t = 0; t < NSLOT; ++t) cnt += __popcll(__ballot(key[t] <= mid));
    if (cnt >= k) hi = mid; else lo = mid + 1u;
  }
  const uint32_t T = lo;
  int below = 0;
#pragma unroll
  for (int t = 0; t < NSLOT; ++t) below += __popcll(__ballot(key[t] < T));
  const int ties_wanted = k - below;  // >= 1: candidates exactly at T, lowest indices first

  const unsigned long long before_me = (1ull << lane) - 1ull;
  int ties_seen = 0, chosen_seen = 0;
#pragma unroll
  for (int t = 0; t < NSLOT; ++t) {
    const bool tie = key[t] == T;
    const unsigned long long tie_vote = __ballot(tie);
    const int tie_rank = ties_seen + __popcll(tie_vote & before_me);
    const bool chosen = key[t] < T || (tie && tie_rank < ties_wanted);
    const unsigned long long vote = __ballot(chosen);
    if (chosen) indices[q * k + chosen_seen + __popcll(vote & before_me)] = (int32_t)(base + lane + kWave * t);
    ties_seen += __popcll(tie_vote);
    chosen_seen += __popcll(vote);
  }
}

__global__ void k_knn_indptr(int64_t n, int k, int32_t* __restrict__ indptr) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i <= n) indptr[i] = (int32_t)(i * k);
}

}  // namespace gnn

using namespace gnn;

extern "C" gnn_status_t gnn_knn_graph(int clouds, int points, int dim, int k, const float* coords,
                                      int32_t* indptr, int32_t* indices, void* stream) {
  clear_error();
  GNN_REQUIRE(clouds >= 0 && points > 0 && dim > 0 && k > 0, GNN_ERR_INVALID_ARG,
              "gnn_knn_graph: sizes must be positive");
  GNN_REQUIRE(k <= points, GNN_ERR_UNSUPPORTED, "gnn_knn_graph: k = %d exceeds the cloud size %d", k, points);
  GNN_REQUIRE(points <= kKnnMaxPoints, GNN_ERR_UNSUPPORTED, "gnn_knn_graph: %d points per cloud exceed %d",
              points, kKnnMaxPoints);
  const int64_t n = (int64_t)clouds * points;
  GNN_REQUIRE(n * k < (int64_t)INT32_MAX, GNN_ERR_UNSUPPORTED, "gnn_knn_graph: edge count does not fit 32 bits");
  GNN_REQUIRE(indptr != nullptr, GNN_ERR_INVALID_ARG, "gnn_knn_graph: indptr is null");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope p("knn_graph", st);
  k_knn_indptr<<<(unsigned)cdiv(n + 1, 256), 256, 0, st>>>(n, k, indptr);
  GNN_LAUNCH_CHECK();
  if (n == 0) return GNN_OK;
  GNN_REQUIRE(coords && indices, GNN_ERR_INVALID_ARG, "gnn_knn_graph: null pointer");
  const unsigned grid = (unsigned)cdiv(n, kKnnQueries);
#define GNN_KNN_CASE(NSLOT_)                                                                    \
  k_knn<NSLOT_><<<grid, kKnnThreads, 0, st>>>(n, points, dim, k, coords, indices)
  const int slots = (int)cdiv(points, kWave);  // register slots a lane needs
  if (slots <= 1) GNN_KNN_CASE(1);
  else if (slots <= 2) GNN_KNN_CASE(2);
  else if (slots <= 4) GNN_KNN_CASE(4);
  else if (slots <= 8) GNN_KNN_CASE(8);
  else if (slots <= 16) GNN_KNN_CASE(16);
  else GNN_KNN_CASE(32);
#undef GNN_KNN_CASE
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}
