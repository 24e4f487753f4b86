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
// One wavefront per query point.  Every candidate becomes a 64-bit key (distance bits in the
// high word - non-negative floats order like unsigned integers - and the candidate's index in
// the low word), kept in LDS; lane l owns the candidates l, l+64, ...  The k smallest keys are
// drawn one by one: a butterfly minimum over the lanes' current minima, then the owning lane
// strikes the winner out and rescans its own list.  A rank sort over the k winners puts
// them in ascending index order.
#include "common.h"

namespace gnn {

constexpr int kKnnThreads = 256;
constexpr int kKnnQueries = kKnnThreads / kWave;
constexpr int kKnnMaxPoints = 2048;  // 4 wavefronts x 2048 keys x 8 B = 64 KB of LDS
constexpr unsigned long long kKeyGone = ~0ull;

__global__ __launch_bounds__(kKnnThreads) void k_knn(int64_t n, int points, int dim, int k,
                                                     const float* __restrict__ coords,
                                                     int32_t* __restrict__ indices) {
  extern __shared__ unsigned long long knn_keys[];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t q = (int64_t)blockIdx.x * kKnnQueries + w;
  if (q >= n) return;  // whole wavefront; nothing below synchronises across wavefronts
  const int64_t base = q / points * points;
  unsigned long long* my = knn_keys + (size_t)w * points;
  const float* a = coords + q * dim;

  unsigned long long best = kKeyGone;
  for (int j = lane; j < points; j += kWave) {
    const float* b = coords + (base + j) * dim;
    float acc = 0.f;
    for (int d = 0; d < dim; ++d) {
      const float diff = __fsub_rn(a[d], b[d]);
      const float sq = __fmul_rn(diff, diff);
      acc = d == 0 ? sq : __fadd_rn(acc, sq);
    }
    const unsigned long long key = ((unsigned long long)__float_as_uint(acc) << 32) | (unsigned)j;
    my[j] = key;
    best = key < best ? key : best;
  }

  int mine = 0;  // lane r keeps the r-th winner
  for (int r = 0; r < k; ++r) {
    unsigned long long win = best;
    for (int off = 1; off < kWave; off <<= 1) {
      const unsigned long long o = __shfl_xor(win, off, 64);
      win = o < win ? o : win;
    }
    const int j = (int)(unsigned)(win & 0xffffffffull);
    if (lane == r) mine = j;
    if (lane == (j & 63)) {  // the owner strikes it out and looks for its next minimum
      my[j] = kKeyGone;
      best = kKeyGone;
      for (int t = lane; t < points; t += kWave) {
        const unsigned long long key = my[t];
        best = key < best ? key : best;
      }
    }
  }
  // ascending index order: the rank of a winner is the number of smaller winners
  int rank = 0;
  for (int r = 0; r < k; ++r) {
    const int other = __shfl(mine, r, 64);
    rank += other < mine ? 1 : 0;
  }
  if (lane < k) indices[q * k + rank] = (int32_t)(base + mine);
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
  GNN_REQUIRE(k <= points && k <= kWave, GNN_ERR_UNSUPPORTED,
              "gnn_knn_graph: k = %d must not exceed the cloud size or 64", k);
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
  const size_t lds = sizeof(unsigned long long) * (size_t)kKnnQueries * points;
  k_knn<<<(unsigned)cdiv(n, kKnnQueries), kKnnThreads, lds, st>>>(n, points, dim, k, coords, indices);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}
