// Bench-only comparator: the graph-related operators of one GAT layer run ONE OPERATOR
// PER KERNEL, every intermediate written to HBM and stashed for the backward pass: the
// "without fusion" arm of the ablations (Sec. 7.3; operator list of App. A.2: u_add_v,
// LeakyReLU, edge_softmax as two ReduceScatter steps, reduce_sum).  It is NOT part of
// the library and no product path calls it; bench.py --compare-unfused times it next
// to the fused kernels on the same inputs to report IO and memory ratios (Sec. 5, Sec. 6).
// The dense projection, the attention halves and the parameter gradients are the same
// vertex-side work in both arms and are left out of the comparison.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

constexpr int kThreads = 256;
inline unsigned blocks(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// Scatter u_add_v: M0[e,h] = el[src,h] + er[dst,h]
__global__ void k_u_add_v(int64_t EH, int H, const int32_t* src, const int32_t* dst, const float* el,
                          const float* er, float* M0) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= EH) return;
  int64_t e = i / H;
  int h = (int)(i - e * H);
  M0[i] = el[(int64_t)src[e] * H + h] + er[(int64_t)dst[e] * H + h];
}

// ApplyEdge LeakyReLU
__global__ void k_leaky(int64_t EH, float slope, const float* M0, float* M1) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= EH) return;
  float x = M0[i];
  M1[i] = x > 0.f ? x : slope * x;
}

// Gather (segment reduce by destination), one wavefront per vertex, lanes = (edge, head)
template <bool MAX>
__global__ void k_seg_reduce(int32_t n, int H, int Hp_log2, const int32_t* indptr, const float* vals,
                             float* out, float empty) {
  const int lane = threadIdx.x & 63;
  const int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (v >= n) return;
  const int Hp = 1 << Hp_log2, epc = 64 >> Hp_log2;
  const int e_loc = lane >> Hp_log2, h = lane & (Hp - 1);
  const int32_t beg = indptr[v], end = indptr[v + 1];
  float acc = MAX ? -INFINITY : 0.f;
  if (h < H)
    for (int32_t e = beg + e_loc; e < end; e += epc) {
      float x = vals[(int64_t)e * H + h];
      acc = MAX ? fmaxf(acc, x) : acc + x;
    }
  for (int off = Hp; off < 64; off <<= 1) {
    float o = __shfl_xor(acc, off, 64);
    acc = MAX ? fmaxf(acc, o) : acc + o;
  }
  if (e_loc == 0 && h < H) out[v * H + h] = beg == end ? empty : acc;
}

// ApplyEdge of the first ReduceScatter: EX[e,h] = exp(M1[e,h] - mx[dst,h])
__global__ void k_sub_exp(int64_t EH, int H, const int32_t* dst, const float* M1, const float* mx, float* EX) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= EH) return;
  int64_t e = i / H;
  int h = (int)(i - e * H);
  EX[i] = __expf(M1[i] - mx[(int64_t)dst[e] * H + h]);
}

// ApplyEdge of the second ReduceScatter: M2[e,h] = EX[e,h] / den[dst,h]
__global__ void k_div(int64_t EH, int H, const int32_t* dst, const float* EX, const float* den, float* M2) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= EH) return;
  int64_t e = i / H;
  int h = (int)(i - e * H);
  M2[i] = EX[i] / den[(int64_t)dst[e] * H + h];
}

// Aggregate reduce_sum: out[row] = sum over the row's edges w[eid,h] * feat[col]; one
// wavefront per row, HF = 256 (lane owns one float4).  eid: edge id per position or null.
__global__ void k_spmm256(int32_t n, int H, int F, const int32_t* ptr, const int32_t* cols,
                          const int32_t* eid, const float* w, const float* feat, float* out) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (r >= n) return;
  const int h = (lane * 4) / F;
  const int32_t beg = ptr[r], end = ptr[r + 1];
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int32_t i = beg; i < end; ++i) {
    const int32_t c = cols[i];
    const int64_t e = eid ? eid[i] : i;
    const float a = w[e * H + h];
    const float4 x = ld4(feat + (int64_t)c * 256 + lane * 4);
    acc.x += a * x.x; acc.y += a * x.y; acc.z += a * x.z; acc.w += a * x.w;
  }
  *reinterpret_cast<float4*>(out + r * 256 + lane * 4) = acc;
}

// SDDMM of the backward pass: dM2[e,h] = <gout[dst,h,:], z[src,h,:]>, HF = 256, F = 64
__global__ void k_sddmm256(int32_t n, int H, const int32_t* indptr, const int32_t* indices,
                           const float* gout, const float* z, float* dM2) {
  const int lane = threadIdx.x & 63;
  const int64_t v = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (v >= n) return;
  const float4 g = ld4(gout + v * 256 + lane * 4);
  const int32_t beg = indptr[v], end = indptr[v + 1];
  for (int32_t e = beg; e < end; ++e) {
    const float4 x = ld4(z + (int64_t)indices[e] * 256 + lane * 4);
    float p = g.x * x.x + g.y * x.y + g.z * x.z + g.w * x.w;
    for (int off = 1; off < 16; off <<= 1) p += __shfl_xor(p, off, 64);  // 16 lanes per head
    if ((lane & 15) == 0) dM2[(int64_t)e * H + (lane >> 4)] = p;
  }
}

__global__ void k_mul(int64_t EH, const float* a, const float* b, float* c) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i < EH) c[i] = a[i] * b[i];
}

// softmax and LeakyReLU backward: dM0 = M2 (dM2 - t[dst]) LeakyReLU'(M0)
__global__ void k_score_bwd(int64_t EH, int H, float slope, const int32_t* dst, const float* M0,
                            const float* M2, const float* dM2, const float* t, float* dM0) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= EH) return;
  int64_t e = i / H;
  int h = (int)(i - e * H);
  float d1 = M2[i] * (dM2[i] - t[(int64_t)dst[e] * H + h]);
  dM0[i] = M0[i] > 0.f ? d1 : slope * d1;
}

// del[u,h] = sum over out-edges of dM0 (CSC walk through the edge-id permutation)
__global__ void k_seg_sum_src(int32_t n, int H, const int32_t* ptr_t, const int32_t* eid_t,
                              const float* dM0, float* del) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= (int64_t)n * H) return;
  int64_t u = i / H;
  int h = (int)(i - u * H);
  float s = 0.f;
  for (int32_t k = ptr_t[u]; k < ptr_t[u + 1]; ++k) s += dM0[(int64_t)eid_t[k] * H + h];
  del[i] = s;
}

// dz[u,:] += a_l del[u] + a_r der[u]
__global__ void k_dz_close(int64_t NHF, int H, int F, const float* a_l, const float* a_r, const float* del,
                           const float* der, float* dz) {
  int64_t i = blockIdx.x * (int64_t)kThreads + threadIdx.x;
  if (i >= NHF) return;
  const int HF = H * F;
  int64_t u = i / HF;
  int c = (int)(i - u * HF);
  int h = c / F;
  dz[i] += a_l[c] * del[u * H + h] + a_r[c] * der[u * H + h];
}

}  // namespace

// Forward graph operators.  Stashed for backward: M0, M2 (and el, er, z as in the fused path).
extern "C" int unfused_gat_graph_fwd(int32_t n, int64_t nnz, int H, int F, float slope,
                                     const int32_t* indptr, const int32_t* indices, const int32_t* dst,
                                     const float* z, const float* el, const float* er, float* M0, float* M1,
                                     float* mx, float* EX, float* den, float* M2, float* out, void* stream) {
  if (H * F != 256 || F != 64) return 4;  // written for the 4 x 64 ablation setting only
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t EH = nnz * H;
  int hl = 0;
  while ((1 << hl) < H) ++hl;
  const unsigned wg = (unsigned)((n + 3) / 4);
  k_u_add_v<<<blocks(EH), kThreads, 0, st>>>(EH, H, indices, dst, el, er, M0);
  k_leaky<<<blocks(EH), kThreads, 0, st>>>(EH, slope, M0, M1);
  k_seg_reduce<true><<<wg, kThreads, 0, st>>>(n, H, hl, indptr, M1, mx, 0.f);
  k_sub_exp<<<blocks(EH), kThreads, 0, st>>>(EH, H, dst, M1, mx, EX);
  k_seg_reduce<false><<<wg, kThreads, 0, st>>>(n, H, hl, indptr, EX, den, 1.f);
  k_div<<<blocks(EH), kThreads, 0, st>>>(EH, H, dst, EX, den, M2);
  k_spmm256<<<wg, kThreads, 0, st>>>(n, H, F, indptr, indices, nullptr, M2, z, out);
  return (int)hipGetLastError();
}

// Backward graph operators from the stashed M0, M2: writes dz, der, del.
extern "C" int unfused_gat_graph_bwd(int32_t n, int64_t nnz, int H, int F, float slope,
                                     const int32_t* indptr, const int32_t* indices, const int32_t* dst,
                                     const int32_t* indptr_t, const int32_t* indices_t, const int32_t* eid_t,
                                     const float* z, const float* gout, const float* a_l, const float* a_r,
                                     const float* M0, const float* M2, float* dM2, float* tmp, float* t,
                                     float* dM0, float* der, float* del, float* dz, void* stream) {
  if (H * F != 256 || F != 64) return 4;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t EH = nnz * H;
  int hl = 0;
  while ((1 << hl) < H) ++hl;
  const unsigned wg = (unsigned)((n + 3) / 4);
  k_sddmm256<<<wg, kThreads, 0, st>>>(n, H, indptr, indices, gout, z, dM2);
  k_mul<<<blocks(EH), kThreads, 0, st>>>(EH, M2, dM2, tmp);
  k_seg_reduce<false><<<wg, kThreads, 0, st>>>(n, H, hl, indptr, tmp, t, 0.f);
  k_score_bwd<<<blocks(EH), kThreads, 0, st>>>(EH, H, slope, dst, M0, M2, dM2, t, dM0);
  k_seg_reduce<false><<<wg, kThreads, 0, st>>>(n, H, hl, indptr, dM0, der, 0.f);
  k_seg_sum_src<<<blocks((int64_t)n * H), kThreads, 0, st>>>(n, H, indptr_t, eid_t, dM0, del);
  k_spmm256<<<wg, kThreads, 0, st>>>(n, H, F, indptr_t, indices_t, eid_t, M2, gout, dz);
  k_dz_close<<<blocks((int64_t)n * H * F), kThreads, 0, st>>>((int64_t)n * H * F, H, F, a_l, a_r, del, der, dz);
  return (int)hipGetLastError();
}
