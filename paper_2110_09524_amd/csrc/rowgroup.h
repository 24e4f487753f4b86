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
// in those bits end up with the same value.  Over whole groups (lo_stride == 1) the
// steps inside a row of 16 lanes are DPP operations on the vector ALU (pairings: lane ^ 1
// and lane ^ 2 inside quads, then the mirrored halves of 8 and of 16 lanes, which pair the
// right quads because all lanes of a quad already agree); the results are the same bits as
// the xor butterfly's, without four dependent trips through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int L>
__device__ __forceinline__ float group_max_from(float v, int lo_stride) {
  if (lo_stride == 1) {
    if (L > 1) v = fmaxf(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
    if (L > 2) v = fmaxf(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
    if (L > 4) v = fmaxf(v, dpp_move<0x141>(v));  // row_half_mirror
    if (L > 8) v = fmaxf(v, dpp_move<0x140>(v));  // row_mirror
    for (int off = 16; off < L; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
  }
  for (int off = lo_stride; off < L; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
template <int L>
__device__ __forceinline__ float group_sum_from(float v, int lo_stride) {
  if (lo_stride == 1) {
    if (L > 1) v += dpp_move<0xB1>(v);
    if (L > 2) v += dpp_move<0x4E>(v);
    if (L > 4) v += dpp_move<0x141>(v);
    if (L > 8) v += dpp_move<0x140>(v);
    for (int off = 16; off < L; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
  }
  for (int off = lo_stride; off < L; off <<= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Pace of the persistent kernels.  Workgroups that share an L2 (one XCD) walk the column blocks
// step by step: a workgroup that has finished step `step` reports it on its XCD's counter and
// waits until all `nwg` workgroups of the XCD have done so.  The wait only keeps the gathered
// block cache-resident: results never depend on it, so it is bounded (`spin_limit` polls) and a
// workgroup that once ran into the bound stops waiting for the rest of the launch (with a limit
// of 0 nothing is ever waited for).  One thread does the reporting and waiting; the caller puts
// workgroup barriers around it, and whatever the other threads can prepare for the next step
// (the next row's bounds and indices) between the two.
struct PhaseClock {
  int32_t* counter;  // this XCD's counter, zero at launch; null: no pacing between workgroups
  int nwg, spin_limit;
  bool gave_up;
  int every;  // the workgroups meet after every `every`-th step only
};
__device__ __forceinline__ void phase_step_done(PhaseClock& pc, int step) {
  if (pc.counter == nullptr || threadIdx.x != 0 || (step + 1) % pc.every != 0) return;
  __hip_atomic_fetch_add(pc.counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const int target = pc.nwg * ((step + 1) / pc.every);
  int polls = 0;
  while (!pc.gave_up && __hip_atomic_load(pc.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
    if (++polls > pc.spin_limit) pc.gave_up = true;
    else __builtin_amdgcn_s_sleep(2);
  }
}

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
// streaming variants: data that is touched once per launch is marked non-temporal so that it
// does not displace the cache-resident gathered rows
typedef float nt_f4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld4_stream(const float* p) {
  const nt_f4 v = __builtin_nontemporal_load(reinterpret_cast<const nt_f4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4_stream(float* p, float4 v) {
  nt_f4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<nt_f4*>(p));
}
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

// ---- which row a group works on ---------------------------------------------------
// Normal launches give every group its own row.  Rows whose degree is many chunks
// long would make one group loop for a long time while the rest of the chip is idle
// (power-law hubs), so the heaviest rows (a prefix of the degree order) are launched
// "cooperatively": all groups of a workgroup share one row, take its chunks round-robin,
// and fold their partial sums through LDS in group order (deterministic).
// Row handed to a group when rows are taken in vertex order instead of degree order (graphs
// with near-uniform degrees, e.g. kNN batches, where neighbours have nearby ids): workgroups
// go to the 8 XCDs round-robin, so workgroup w serves XCD w % 8; giving XCD k the k-th
// contiguous eighth of the row blocks keeps each XCD's gathers inside 1/8 of the matrix,
// which its own L2 can hold.  The grid must be a multiple of 8 workgroups.
__device__ __forceinline__ int64_t xcd_contiguous_row(unsigned wg, unsigned nwg, int gpb, int grp) {
  const unsigned per_xcd = nwg / 8;
  return ((int64_t)(wg % 8) * per_xcd + wg / 8) * gpb + grp;
}
inline unsigned xcd_contiguous_grid(int64_t rows, int gpb) {
  const int64_t blocks = (rows + gpb - 1) / gpb;
  return (unsigned)((blocks + 7) / 8 * 8);
}

struct RowRange {
  int32_t begin, end;  // positions in the degree order
  int coop;            // 1: one row per workgroup
};

template <int GPB>
__device__ __forceinline__ bool pick_row(const RowRange& rr, int grp, int64_t& r, int& gi, int& ngrp) {
  if (rr.coop) {
    r = (int64_t)rr.begin + blockIdx.x;
    gi = grp;
    ngrp = GPB;
  } else {
    r = (int64_t)rr.begin + (int64_t)blockIdx.x * GPB + grp;
    gi = 0;
    ngrp = 1;
  }
  return r < rr.end;
}

// One launch serves both kinds of rows: its first n_hub workgroups take one hub row each
// (cooperatively), the others GPB rows of the rest each; the kind is uniform in a workgroup.
struct RowLaunch {
  int32_t n_hub, n_rows;
};
template <int GPB>
__device__ __forceinline__ bool pick_row(const RowLaunch& rl, int grp, RowRange& rr, int64_t& r, int& gi,
                                         int& ngrp) {
  if (blockIdx.x < (unsigned)rl.n_hub) {
    rr = RowRange{0, rl.n_hub, 1};
    r = blockIdx.x;
    gi = grp;
    ngrp = GPB;
  } else {
    rr = RowRange{rl.n_hub, rl.n_rows, 0};
    r = (int64_t)rl.n_hub + (int64_t)(blockIdx.x - (unsigned)rl.n_hub) * GPB + grp;
    gi = 0;
    ngrp = 1;
  }
  return r < rr.end;
}

// Adds the N per-lane values of groups 1..GPB-1 onto group 0's, in group order.  Every
// thread of the workgroup must call it; afterwards only group 0 holds the totals.
// buf: GPB * L * N floats of LDS.
template <int L, int N, int GPB>
__device__ __forceinline__ void coop_sum(float* buf, float (&v)[N], int grp, int li) {
  if (grp != 0) {
#pragma unroll
    for (int i = 0; i < N; ++i) buf[(grp * N + i) * L + li] = v[i];
  }
  __syncthreads();
  if (grp == 0) {
    for (int g = 1; g < GPB; ++g) {
#pragma unroll
      for (int i = 0; i < N; ++i) v[i] += buf[(g * N + i) * L + li];
    }
  }
  __syncthreads();
}

__device__ __forceinline__ void pack4(float* dst, const float4& a) {
  dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w;
}
__device__ __forceinline__ float4 unpack4(const float* src) {
  return make_float4(src[0], src[1], src[2], src[3]);
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

// Split of one side's degree order into a cooperative prefix (rows at least
// kCoopChunks chunks long) and the rest, with the grids of the two launches.
constexpr int kCoopChunks = 16;
struct RowSplit {
  RowRange hub, rest;
  unsigned hub_grid, rest_grid;
};
// The threshold drops from kCoopChunks to as few as kCoopMinChunks chunks while that adds no more
// than kCoopCheapRows cooperative rows: on a small graph the longest ordinary row is the critical
// path of the whole launch (a chunk is a chain of dependent loads), and a few hundred extra
// workgroups cost nothing there.
constexpr int kCoopMinChunks = 4;
constexpr int kCoopCheapRows = 1024;
inline RowSplit split_rows(const gnn_graph* g, int side, int chunk_edges, int gpb) {
  // degree >= 2^k  <=>  clz32(degree) <= 31 - k: a prefix of the degree order
  auto rows_at_least = [&](int k) { return k >= 31 ? 0 : g->h_bucket_offsets[side][32 - k]; };
  int k = ilog2(next_pow2(kCoopChunks * chunk_edges));  // degree threshold 2^k
  const int k_min = ilog2(next_pow2(kCoopMinChunks * chunk_edges));
  while (k > k_min && rows_at_least(k - 1) <= kCoopCheapRows) --k;
  const int32_t n_hub = rows_at_least(k);
  RowSplit s;
  s.hub = RowRange{0, n_hub, 1};
  s.rest = RowRange{n_hub, g->n, 0};
  s.hub_grid = (unsigned)n_hub;
  s.rest_grid = (unsigned)((g->n - n_hub + gpb - 1) / gpb);
  return s;
}

}  // namespace gnn
