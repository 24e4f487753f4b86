// Bench-only comparators for the forward pass of EdgeConv and GMM in their original
// dataflow, one operator per kernel with every per-edge intermediate in HBM.
// EdgeConv (App. A.2, Fig. 3(a) left column applied to Sec. 7.2's layer): u_sub_v -> E x fin,
// the linear layer Theta on EDGES (the redundant form the reorganization removes; the
// caller runs it with the library's own MFMA product), e_add_v with the vertex-side Phi
// product, reduce_max.  GMM (App. A.2): pseudo-coordinates -> E x 2, Gaussian weights ->
// E x K, u_mul_e + reduce_sum.  Not part of the library; only bench.py --compare-unfused and
// its test load it.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr int kThreads = 256;
inline unsigned blocks(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }

// Scatter u_sub_v: E0[e,:] = x[src[e],:] - x[dst[e],:]   (width % 4 == 0)
__global__ void k_u_sub_v(int64_t quads, int q_per_row, const int32_t* src, const int32_t* dst,
                          const float* x, float* E0) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= quads) return;
  const int64_t e = i / q_per_row;
  const int q = (int)(i - e * q_per_row);
  const int64_t w = 4 * (int64_t)q_per_row;
  const float4 a = ld4(x + src[e] * w + 4 * q), b = ld4(x + dst[e] * w + 4 * q);
  st4(E0 + e * w + 4 * q, make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w));
}

// Scatter e_add_v: E2[e,:] = E1[e,:] + N1[dst[e],:]
__global__ void k_e_add_v(int64_t quads, int q_per_row, const int32_t* dst, const float* E1,
                          const float* N1, float* E2) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= quads) return;
  const int64_t e = i / q_per_row;
  const int q = (int)(i - e * q_per_row);
  const int64_t w = 4 * (int64_t)q_per_row;
  const float4 a = ld4(E1 + e * w + 4 * q), b = ld4(N1 + dst[e] * w + 4 * q);
  st4(E2 + e * w + 4 * q, make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w));
}

// Gather reduce_max over the in-edges; one thread per (vertex, 4 columns); earliest edge wins ties
__global__ void k_seg_max(int64_t quads, int q_per_row, const int32_t* indptr, const float* E2,
                          float* out, int32_t* argmax) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= quads) return;
  const int64_t v = i / q_per_row;
  const int q = (int)(i - v * q_per_row);
  const int64_t w = 4 * (int64_t)q_per_row;
  const int32_t beg = indptr[v], end = indptr[v + 1];
  float4 best = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  int4 arg = make_int4(-1, -1, -1, -1);
  for (int32_t e = beg; e < end; ++e) {
    const float4 r = ld4(E2 + e * w + 4 * q);
    if (r.x > best.x) { best.x = r.x; arg.x = e; }
    if (r.y > best.y) { best.y = r.y; arg.y = e; }
    if (r.z > best.z) { best.z = r.z; arg.z = e; }
    if (r.w > best.w) { best.w = r.w; arg.w = e; }
  }
  if (beg == end) best = make_float4(0.f, 0.f, 0.f, 0.f);
  st4(out + v * w + 4 * q, best);
  *reinterpret_cast<int4*>(argmax + v * w + 4 * q) = arg;
}

// Scatter: pseudo-coordinates P[e] = (c[src], c[dst])
__global__ void k_pseudo(int64_t E, const int32_t* src, const int32_t* dst, const float* c, float2* P) {
  int64_t e = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (e < E) P[e] = make_float2(c[src[e]], c[dst[e]]);
}

// ApplyEdge: W[e,k] = exp(-1/2 sum_d ((P[e,d] - mu[k,d]) inv_sigma[k,d])^2)
__global__ void k_gauss(int64_t EK, int K, const float2* P, const float* mu, const float* inv_sigma,
                        float* W) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= EK) return;
  const int64_t e = i / K;
  const int k = (int)(i - e * K);
  const float2 p = P[e];
  const float t0 = (p.x - mu[2 * k]) * inv_sigma[2 * k], t1 = (p.y - mu[2 * k + 1]) * inv_sigma[2 * k + 1];
  W[i] = __expf(-0.5f * (t0 * t0 + t1 * t1));
}

// Aggregate u_mul_e + reduce_sum: out[v,:] = (1/K) sum_e sum_k W[e,k] hk[src[e],k,:];
// one wavefront per vertex: 64 / (F/4) edge slots of F/4 lanes each take the in-edges
// round-robin and are added at the end (a row-split SpMM)
__global__ void k_u_mul_e_sum(int32_t n, int K, int F, const int32_t* indptr, const int32_t* indices,
                              const float* W, const float* hk, float* out) {
  const int L = F / 4, slots = 64 / L;
  const int lane = threadIdx.x & 63;
  const int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (v >= n) return;
  const int li = lane % L, slot = lane / L;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int32_t e = indptr[v] + slot; e < indptr[v + 1]; e += slots) {
    const float* row = hk + (int64_t)indices[e] * K * F + 4 * li;
    for (int k = 0; k < K; ++k) {
      const float w = W[(int64_t)e * K + k];
      const float4 r = ld4(row + k * F);
      acc.x += w * r.x; acc.y += w * r.y; acc.z += w * r.z; acc.w += w * r.w;
    }
  }
  for (int off = L; off < 64; off <<= 1) {
    acc.x += __shfl_xor(acc.x, off, 64); acc.y += __shfl_xor(acc.y, off, 64);
    acc.z += __shfl_xor(acc.z, off, 64); acc.w += __shfl_xor(acc.w, off, 64);
  }
  const float s = 1.f / (float)K;
  if (slot == 0) st4(out + v * F + 4 * li, make_float4(acc.x * s, acc.y * s, acc.z * s, acc.w * s));
}

}  // namespace

// step 1 of the EdgeConv forward: E0 = u_sub_v(x).  fin % 4 == 0.
extern "C" int unfused_ec_u_sub_v(int64_t nnz, int fin, const int32_t* src, const int32_t* dst,
                                  const float* x, float* E0, void* stream) {
  if (fin % 4) return 4;
  const int64_t quads = nnz * (fin / 4);
  k_u_sub_v<<<blocks(quads), kThreads, 0, static_cast<hipStream_t>(stream)>>>(quads, fin / 4, src, dst, x, E0);
  return (int)hipGetLastError();
}

// steps 4 and 5: E2 = e_add_v(E1, N1), out / argmax = reduce_max(E2).  fout % 4 == 0.
extern "C" int unfused_ec_add_max(int32_t n, int64_t nnz, int fout, const int32_t* indptr, const int32_t* dst,
                                  const float* E1, const float* N1, float* E2, float* out, int32_t* argmax,
                                  void* stream) {
  if (fout % 4) return 4;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t eq = nnz * (fout / 4), vq = (int64_t)n * (fout / 4);
  k_e_add_v<<<blocks(eq), kThreads, 0, st>>>(eq, fout / 4, dst, E1, N1, E2);
  k_seg_max<<<blocks(vq), kThreads, 0, st>>>(vq, fout / 4, indptr, E2, out, argmax);
  return (int)hipGetLastError();
}

// GMM forward graph operators: P, W materialised.  F/4 must divide 64.
extern "C" int unfused_gmm_graph_fwd(int32_t n, int64_t nnz, int K, int F, const int32_t* indptr,
                                     const int32_t* indices, const int32_t* dst, const float* c,
                                     const float* mu, const float* inv_sigma, const float* hk, float* P,
                                     float* W, float* out, void* stream) {
  if (F % 4 || F > 256 || 64 % (F / 4)) return 4;
  hipStream_t st = static_cast<hipStream_t>(stream);
  k_pseudo<<<blocks(nnz), kThreads, 0, st>>>(nnz, indices, dst, c, reinterpret_cast<float2*>(P));
  k_gauss<<<blocks(nnz * K), kThreads, 0, st>>>(nnz * K, K, reinterpret_cast<const float2*>(P), mu, inv_sigma, W);
  const int rows_per_wg = kThreads / 64;
  k_u_mul_e_sum<<<(unsigned)((n + rows_per_wg - 1) / rows_per_wg), kThreads, 0, st>>>(n, K, F, indptr, indices, W,
                                                                                    hk, out);
  return (int)hipGetLastError();
}

// Marker launches: an empty kernel whose name carries `id`, so that a per-dispatch counter
// trace of a bench run can be cut into "unfused" and "fused" sections by dispatch order.
namespace {
template <int ID>
__global__ void k_marker() {}
}  // namespace

extern "C" int unfused_marker(int id, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  switch (id) {
    case 0: k_marker<0><<<1, 64, 0, st>>>(); break;
    case 1: k_marker<1><<<1, 64, 0, st>>>(); break;
    case 2: k_marker<2><<<1, 64, 0, st>>>(); break;
    default: return 4;
  }
  return (int)hipGetLastError();
}
