// Device helpers for the vertex-balanced mapping shared by all fused kernels
// (Sec. 5: a thread GROUP loops over the in-edge set of one vertex).
//
// A row group is L consecutive lanes of a 64-wide wavefront (L a power of two,
// 4..64).  It owns one row of the walked sparse matrix (a destination in the CSR
// walks, a source in the CSC walks).  Feature columns are spread over the group
// in float4 slots: lane li owns columns 4*(li + j*L) .. +3 for j < NV, so one
// gathered feature row is one coalesced run of 16-byte loads.
//
// Per-edge scalars (scores, softmax values, Gaussian weights) are computed in a
// "chunk phase" with the group's lanes spread over (edge, head) pairs, parked in
// LDS, and then broadcast-read in the "row phase" where lanes are spread over
// columns.  LDS traffic of one group never leaves its wavefront, so wavefront
// scope fences are enough.
#pragma once

#include <hip/hip_runtime.h>

namespace gnn {

__device__ __forceinline__ void wave_lds_fence() {
  // LDS operations of one wavefront execute in order; this keeps the compiler
  // from moving LDS accesses across the hand-off between the two phases.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// butterfly reductions over lane-index bits [lo_stride, L): lanes that differ only
// in those bits end up with the same value
template <int L>
__device__ __forceinline__ float group_max_from(float v, int lo_stride) {
  for (int off = lo_stride; off < L; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
template <int L>
__device__ __forceinline__ float group_sum_from(float v, int lo_stride) {
  for (int off = lo_stride; off < L; off <<= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void fma4(float4& acc, float s, const float4& v) {
  acc.x = fmaf(s, v.x, acc.x);
  acc.y = fmaf(s, v.y, acc.y);
  acc.z = fmaf(s, v.z, acc.z);
  acc.w = fmaf(s, v.w, acc.w);
}
__device__ __forceinline__ float dot4(const float4& a, const float4& b) {
  return fmaf(a.x, b.x, fmaf(a.y, b.y, fmaf(a.z, b.z, a.w * b.w)));
}
// acc = acc * s + part : folds a chunk's partial sum into the running total.  Summing
// in two levels (edges of a chunk, then chunks) keeps fp32 rounding of a long row
// near sqrt(chunks) ulps of the total instead of sqrt(edges).
__device__ __forceinline__ void fold4(float4& acc, float s, const float4& part) {
  acc.x = fmaf(acc.x, s, part.x);
  acc.y = fmaf(acc.y, s, part.y);
  acc.z = fmaf(acc.z, s, part.z);
  acc.w = fmaf(acc.w, s, part.w);
}
__device__ __forceinline__ void add4(float4& acc, const float4& part) {
  acc.x += part.x; acc.y += part.y; acc.z += part.z; acc.w += part.w;
}
__device__ __forceinline__ void scale4(float4& a, float s) {
  a.x *= s; a.y *= s; a.z *= s; a.w *= s;
}

// Host-side choice of the group shape for a row of `width` floats (width % 4 == 0).
struct GroupShape {
  int L;   // lanes per group
  int NV;  // float4 slots per lane
};
inline GroupShape pick_group(int width) {
  int q = width / 4;
  int L = 4;
  while (L < q && L < 64) L <<= 1;
  int NV = (q + L - 1) / L;
  return GroupShape{L, NV};
}
inline int next_pow2(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}
inline int ilog2(int p) {
  int l = 0;
  while ((1 << l) < p) ++l;
  return l;
}

}  // namespace gnn
