// MoNet / GMMConv layer with general pseudo-coordinates (App. A.2 "GMMConv": w_k(m) for an
// r-dimensional m_uv; Sec. 7.2 uses r = 1, 2, 3), and the learnable projection of the degree
// pair that produces them.
//
//   w_k(e)  = exp(-1/2 sum_d ((m[e,d] - mu[k,d]) inv_sigma[k,d])^2)            (ApplyEdge)
//   out[v]  = (1/K) sum_in-edges sum_k w_k(e) hk[u,k,:]                         (Aggregate)
//
// m is a per-edge input [E, r] in CSR order (an input like the graph itself, not an
// intermediate: nothing else per-edge is stored).  Forward fuses the Gaussian weights with the
// aggregation as in the degree-pair layer.  Backward recomputes the weights:
//   destination side (CSR walk): dw_k(e) = <gout[v], hk[u,k,:]> / K needs one dot product per edge
//     and kernel here (the pseudo-coordinates vary freely along a row, so the dot product cannot
//     be postponed past the neighbourhood sum as in the degree-pair layer); from it
//     gmu, ginv_sigma (summed over all edges in a fixed two-stage order) and gm[e,:];
//   source side (CSC walk, no atomics): dhk[u,k,:] = (1/K) sum_out-edges w_k(e) gout[v,:],
//     with m read through the plan's CSC position -> CSR edge id table.
// At most 4 kernels and 4 pseudo-coordinate dimensions; fout <= 256.
#include <algorithm>
#include <type_traits>

#include "common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kPsBlock = 256;
constexpr int kPsK = 4;   // kernels
constexpr int kPsR = 4;   // pseudo-coordinate dimensions
constexpr int kPsVals = 2 * kPsK * kPsR;  // gmu and ginv_sigma entries per partial slot

struct PsParams {
  int K, R, F;
};

// the K x R means and inverse widths, zero-padded, in registers (uniform)
struct PsKernels {
  float mu[kPsK][kPsR], is[kPsK][kPsR];
};
__device__ __forceinline__ PsKernels load_kernels(const float* __restrict__ mu, const float* __restrict__ is,
                                                  int K, int R) {
  PsKernels p;
#pragma unroll
  for (int k = 0; k < kPsK; ++k)
#pragma unroll
    for (int d = 0; d < kPsR; ++d) {
      const bool ok = k < K && d < R;
      p.mu[k][d] = ok ? mu[k * R + d] : 0.f;
      p.is[k][d] = ok ? is[k * R + d] : 0.f;
    }
  return p;
}
__device__ __forceinline__ void load_pseudo(const float* __restrict__ m, int64_t e, int R, float (&out)[kPsR]) {
#pragma unroll
  for (int d = 0; d < kPsR; ++d) out[d] = d < R ? m[e * R + d] : 0.f;
}
__device__ __forceinline__ float gauss_k(const PsKernels& p, int k, const float (&m)[kPsR]) {
  float q = 0.f;
#pragma unroll
  for (int d = 0; d < kPsR; ++d) {  // padded dimensions have inv_sigma 0
    const float t = (m[d] - p.mu[k][d]) * p.is[k][d];
    q = fmaf(t, t, q);
  }
  return __expf(-0.5f * q);
}

// ---- forward: one row group per destination (hub rows: one workgroup), one edge at a time ----
template <int L>
__global__ __launch_bounds__(kPsBlock) void k_gmmp_fwd(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ hk, const float* __restrict__ pseudo,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma, PsParams pm, float* __restrict__ out) {
  constexpr int GPB = kPsBlock / L;
  __shared__ float coop_buf[GPB * L * 4];
  const int li = threadIdx.x & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  const int K = pm.K, R = pm.R, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  const PsKernels pk = load_kernels(mu, inv_sigma, K, R);
  const int32_t v = order[r];
  const int32_t beg = indptr[v], end = indptr[v + 1];
  const bool col_ok = 4 * li < F;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), part = acc;
  int folded = 0;
  for (int32_t e = beg + gi; e < end; e += ngrp) {
    const int32_t u = indices[e];
    float m[kPsR];
    load_pseudo(pseudo, e, R, m);
    if (col_ok) {
      float4 rowv[kPsK];
#pragma unroll
      for (int k = 0; k < kPsK; ++k)
        if (k < K) rowv[k] = ld4(hk + (int64_t)u * KF + k * F + 4 * li);
#pragma unroll
      for (int k = 0; k < kPsK; ++k)
        if (k < K) fma4(part, gauss_k(pk, k, m) * inv_k, rowv[k]);
    }
    if (++folded == 32) {  // two-level summation keeps long rows accurate
      add4(acc, part);
      part = make_float4(0.f, 0.f, 0.f, 0.f);
      folded = 0;
    }
  }
  add4(acc, part);
  if (rr.coop) {
    float vv[4];
    pack4(vv, acc);
    coop_sum<L, 4, GPB>(coop_buf, vv, grp, li);
    if (grp != 0) return;
    acc = unpack4(vv);
  }
  if (col_ok) st4(out + (int64_t)v * F + 4 * li, acc);
}

// ---- backward, destination side: gmu, ginv_sigma partials and gm[e,:] -------------------------
// partial[block][kPsVals]: entries k*R+d of gmu, then of ginv_sigma, summed over the block's edges
// in a fixed order (group slots, then groups in order).
template <int L>
__global__ __launch_bounds__(kPsBlock) void k_gmmp_bwd_dst(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ hk, const float* __restrict__ pseudo,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma, const float* __restrict__ gout,
    PsParams pm, float* __restrict__ partial, float* __restrict__ gpseudo /* nullable */) {
  constexpr int GPB = kPsBlock / L;
  __shared__ float blk[GPB][kPsVals];
  const int li = threadIdx.x & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  const bool active = pick_row<GPB>(rl, grp, rr, r, gi, ngrp);
  const int K = pm.K, R = pm.R, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  float gm_acc[kPsK][kPsR], gs_acc[kPsK][kPsR];  // every lane of the group keeps the same sums
#pragma unroll
  for (int k = 0; k < kPsK; ++k)
#pragma unroll
    for (int d = 0; d < kPsR; ++d) {
      gm_acc[k][d] = 0.f;
      gs_acc[k][d] = 0.f;
    }
  if (active) {
    const PsKernels pk = load_kernels(mu, inv_sigma, K, R);
    const int32_t v = order[r];
    const int32_t beg = indptr[v], end = indptr[v + 1];
    const bool col_ok = 4 * li < F;
    const float4 g4 = col_ok ? ld4(gout + (int64_t)v * F + 4 * li) : make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t e = beg + gi; e < end; e += ngrp) {
      const int32_t u = indices[e];
      float m[kPsR];
      load_pseudo(pseudo, e, R, m);
      float dots[kPsK];
#pragma unroll
      for (int k = 0; k < kPsK; ++k) {
        dots[k] = 0.f;
        if (k < K && col_ok) dots[k] = dot4(g4, ld4(hk + (int64_t)u * KF + k * F + 4 * li));
      }
      float gm[kPsR];
#pragma unroll
      for (int d = 0; d < kPsR; ++d) gm[d] = 0.f;
#pragma unroll
      for (int k = 0; k < kPsK; ++k) {
        if (k >= K) continue;
        const float dw = group_sum_from<L>(dots[k], 1) * inv_k;  // <gout[v], hk[u,k,:]> / K, in every lane
        const float dlog = dw * gauss_k(pk, k, m);
#pragma unroll
        for (int d = 0; d < kPsR; ++d) {
          const float diff = m[d] - pk.mu[k][d];
          const float is = pk.is[k][d];
          const float t = dlog * diff * is;  // padded dimensions: is = 0
          gm_acc[k][d] = fmaf(t, is, gm_acc[k][d]);
          gs_acc[k][d] = fmaf(-t, diff, gs_acc[k][d]);
          gm[d] = fmaf(-t, is, gm[d]);
        }
      }
      if (gpseudo != nullptr && li == 0) {
#pragma unroll
        for (int d = 0; d < kPsR; ++d)
          if (d < R) gpseudo[(int64_t)e * R + d] = gm[d];
      }
    }
  }
  // lane 0 of every group parks its sums; then one thread per entry adds the groups in order
  if (li == 0) {
#pragma unroll
    for (int k = 0; k < kPsK; ++k)
#pragma unroll
      for (int d = 0; d < kPsR; ++d) {
        blk[grp][k * kPsR + d] = gm_acc[k][d];
        blk[grp][kPsK * kPsR + k * kPsR + d] = gs_acc[k][d];
      }
  }
  __syncthreads();
  if (threadIdx.x < kPsVals) {
    float s = 0.f;
    for (int g2 = 0; g2 < GPB; ++g2) s += blk[g2][threadIdx.x];
    partial[(int64_t)blockIdx.x * kPsVals + threadIdx.x] = s;
  }
}

// totals [kPsVals] (padded K x R layout) -> gmu, ginv_sigma [K, R]
__global__ void k_gmmp_param_split(int K, int R, const float* __restrict__ totals, float* __restrict__ gmu,
                                   float* __restrict__ gis) {
  const int i = threadIdx.x;
  if (i >= K * R) return;
  const int k = i / R, d = i - k * R;
  gmu[i] = totals[k * kPsR + d];
  gis[i] = totals[kPsK * kPsR + k * kPsR + d];
}

// ---- backward, source side: dhk[u,k,:] = (1/K) sum over out-edges w_k(e) gout[v,:] ------------
template <int L>
__global__ __launch_bounds__(kPsBlock) void k_gmmp_bwd_src(
    RowLaunch rl, const int32_t* __restrict__ order_t, const int32_t* __restrict__ indptr_t,
    const int32_t* __restrict__ indices_t, const int32_t* __restrict__ eid_t,
    const float* __restrict__ pseudo, const float* __restrict__ pseudo_t /* nullable: pseudo in this walk's order */,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma,
    const float* __restrict__ gout, PsParams pm, float* __restrict__ dhk) {
  constexpr int GPB = kPsBlock / L;
  __shared__ float coop_buf[GPB * L * 4 * kPsK];
  const int li = threadIdx.x & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  const int K = pm.K, R = pm.R, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  const PsKernels pk = load_kernels(mu, inv_sigma, K, R);
  const int32_t u = order_t[r];
  const int32_t beg = indptr_t[u], end = indptr_t[u + 1];
  const bool col_ok = 4 * li < F;
  float4 acc[kPsK];
#pragma unroll
  for (int k = 0; k < kPsK; ++k) acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int32_t p = beg + gi; p < end; p += ngrp) {
    const int32_t v = indices_t[p];
    float m[kPsR];
    if (pseudo_t != nullptr) load_pseudo(pseudo_t, p, R, m);
    else load_pseudo(pseudo, eid_t[p], R, m);
    if (col_ok) {
      const float4 g4 = ld4(gout + (int64_t)v * F + 4 * li);
#pragma unroll
      for (int k = 0; k < kPsK; ++k)
        if (k < K) fma4(acc[k], gauss_k(pk, k, m) * inv_k, g4);
    }
  }
  if (rr.coop) {
    float vv[4 * kPsK];
#pragma unroll
    for (int k = 0; k < kPsK; ++k) pack4(vv + 4 * k, acc[k]);
    coop_sum<L, 4 * kPsK, GPB>(coop_buf, vv, grp, li);
    if (grp != 0) return;
#pragma unroll
    for (int k = 0; k < kPsK; ++k) acc[k] = unpack4(vv + 4 * k);
  }
  if (col_ok) {
#pragma unroll
    for (int k = 0; k < kPsK; ++k)
      if (k < K) st4(dhk + (int64_t)u * KF + k * F + 4 * li, acc[k]);
  }
}

// ---- narrow rows (K * fout <= 64 floats): chunks of edges, gathered rows in flight ------------
// With 16 hidden features (the paper's MoNet settings) a projected row hk[u] is 128-192 bytes.  The
// kernels above then spend their time on the per-edge chain index -> row -> arithmetic, taken one
// edge at a time (measured at Reddit scale with every gather served by the L2: forward 1.4 of 1.6 ms,
// so the fabric behind the L2s is not what bounds them).  Here a group of G lanes owns the row and
// one float4 of hk[u, :, :] per lane (lane li: kernel li / (F/4), columns 4 (li % (F/4))), and an edge
// set is walked in chunks of G edges in two phases, as in the attention kernels:
//   chunk phase: lane li takes edge li of the chunk: index, pseudo-coordinates, the K Gaussian
//                weights; index and weights are parked in LDS;
//   row phase:   every lane reads them back (broadcast reads) and has 8 row loads in flight.
// LDS traffic of a group stays inside its wavefront.
constexpr int kNrU = 8;  // gathered rows in flight per lane

// PROJ variants: the pseudo-coordinates are not read from an [E, r] array but made on the spot from the
// per-vertex scalar at the two ends of the edge, m[d] = tanh(P[d,0] c[u] + P[d,1] c[v] + pb[d]) (the
// paper's MoNet models project the degree pair this way): one more scalar gather per edge, no
// per-edge tensor at all.
struct ProjArgs {
  const float* c;   // [n]
  const float* P;   // [r, 2]
  const float* pb;  // [r]
};
struct ProjRegs {
  float p0[kPsR], p1[kPsR], b[kPsR];
};
__device__ __forceinline__ ProjRegs load_proj(const ProjArgs& a, int R) {
  ProjRegs q;
#pragma unroll
  for (int d = 0; d < kPsR; ++d) {
    const bool ok = d < R;
    q.p0[d] = ok ? a.P[2 * d] : 0.f;
    q.p1[d] = ok ? a.P[2 * d + 1] : 0.f;
    q.b[d] = ok ? a.pb[d] : 0.f;
  }
  return q;
}
__device__ __forceinline__ void project(const ProjRegs& q, int R, float cu, float cv, float (&m)[kPsR]) {
#pragma unroll
  for (int d = 0; d < kPsR; ++d) m[d] = d < R ? tanhf(fmaf(q.p0[d], cu, fmaf(q.p1[d], cv, q.b[d]))) : 0.f;
}
constexpr int kPsValsProj = kPsVals + 3 * kPsR;  // + (gP[d,0], gP[d,1], gpb[d]) per dimension

// LDS floats of a group: G indices, then kPsK x G weights (forward, source side) or G x G partial
// dot products (destination side)
template <int G>
constexpr int kNrGroupFloats = G + (kPsK > G ? kPsK : G) * G;

__device__ __forceinline__ void read8i(const int* p, int (&v)[kNrU]) {
  const int4 a = *reinterpret_cast<const int4*>(p), b = *reinterpret_cast<const int4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void read8f(const float* p, float (&v)[kNrU]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// forward: out[v, f] = (1/K) sum_e sum_k w_k(e) hk[u, k, f]; the sum over k is taken last, across lanes
template <int G, bool PROJ>
__global__ __launch_bounds__(kPsBlock) void k_gmmp_fwd_nr(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ hk, const float* __restrict__ pseudo,
    ProjArgs pa, const float* __restrict__ mu, const float* __restrict__ inv_sigma, PsParams pm,
    float* __restrict__ out) {
  constexpr int GPB = kPsBlock / G;
  constexpr int GS = kNrGroupFloats<G>;
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float coop_buf[GPB * G * 4];
  const int lane = threadIdx.x & 63;
  const int li = threadIdx.x & (G - 1);
  const int grp = threadIdx.x / G;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  const int K = pm.K, R = pm.R, F = pm.F, KF = K * F, F4 = F / 4;
  const float inv_k = 1.f / (float)K;
  const PsKernels pk = load_kernels(mu, inv_sigma, K, R);
  const int32_t v = order[r];
  const int32_t beg = indptr[v], end = indptr[v + 1];
  ProjRegs pq;
  float cv = 0.f;
  if (PROJ) {
    pq = load_proj(pa, R);
    cv = pa.c[v];
  }
  const bool col_ok = li < K * F4;
  const int myk = col_ok ? li / F4 : 0;
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + G;  // [kPsK][G]
  const float* my_row = hk + 4 * li;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), part = acc;
  int folded = 0;
  for (int32_t e0 = beg + gi * G; e0 < end; e0 += ngrp * G) {
    const bool e_ok = e0 + li < end;
    const int cnt = min(G, end - e0);
    int32_t u = 0;
    float m[kPsR];
#pragma unroll
    for (int d = 0; d < kPsR; ++d) m[d] = 0.f;
    if (e_ok) {
      u = indices[e0 + li];
      if (PROJ) project(pq, R, pa.c[u], cv, m);
      else load_pseudo(pseudo, e0 + li, R, m);
    }
    wave_lds_fence();  // the previous chunk's reads are done
    l_idx[li] = u;
#pragma unroll
    for (int k = 0; k < kPsK; ++k)
      if (k < K) l_w[k * G + li] = e_ok ? gauss_k(pk, k, m) * inv_k : 0.f;
    wave_lds_fence();
#pragma unroll
    for (int t0 = 0; t0 < G; t0 += kNrU) {
      if (t0 < cnt) {
        int idv[kNrU];
        float wv[kNrU];
        read8i(l_idx + t0, idv);
        float4 rowv[kNrU];
#pragma unroll
        for (int t = 0; t < kNrU; ++t)
          if (col_ok && t0 + t < cnt) rowv[t] = ld4(my_row + (int64_t)idv[t] * KF);
        read8f(l_w + myk * G + t0, wv);
#pragma unroll
        for (int t = 0; t < kNrU; ++t)
          if (col_ok && t0 + t < cnt) fma4(part, wv[t], rowv[t]);
      }
    }
    folded += G;
    if (folded >= 32) {  // two-level summation keeps long rows accurate
      add4(acc, part);
      part = make_float4(0.f, 0.f, 0.f, 0.f);
      folded = 0;
    }
  }
  add4(acc, part);
  // kernels 1 .. K-1 sit F/4 lanes further on: add them in order
  float4 tot = acc;
  const int base = lane & ~(G - 1);
  for (int k = 1; k < K; ++k) {
    const int srcl = base + ((li + k * F4) & (G - 1));
    tot.x += __shfl(acc.x, srcl, 64);
    tot.y += __shfl(acc.y, srcl, 64);
    tot.z += __shfl(acc.z, srcl, 64);
    tot.w += __shfl(acc.w, srcl, 64);
  }
  if (rr.coop) {
    float vv[4];
    pack4(vv, tot);
    coop_sum<G, 4, GPB>(coop_buf, vv, grp, li);
    if (grp != 0) return;
    tot = unpack4(vv);
  }
  if (li < F4) st4(out + (int64_t)v * F + 4 * li, tot);
}

// destination side of backward: the row phase leaves every lane's part of <gout[v], hk[u, k, :]> in
// LDS, and the lane that owns the edge adds the F/4 parts of each kernel in lane order
// PROJ: the gradient of the projection's parameters is summed here as well (slots kPsVals ... of a
// partial row), so gpseudo is never written
template <int G, bool PROJ>
__global__ __launch_bounds__(kPsBlock) void k_gmmp_bwd_dst_nr(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ hk, const float* __restrict__ pseudo,
    ProjArgs pa, const float* __restrict__ mu, const float* __restrict__ inv_sigma,
    const float* __restrict__ gout, PsParams pm, float* __restrict__ partial,
    float* __restrict__ gpseudo /* nullable */) {
  constexpr int GPB = kPsBlock / G;
  constexpr int GS = kNrGroupFloats<G>;
  constexpr int NVALS = PROJ ? kPsValsProj : kPsVals;
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float blk[GPB][NVALS];
  const int li = threadIdx.x & (G - 1);
  const int grp = threadIdx.x / G;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  const bool active = pick_row<GPB>(rl, grp, rr, r, gi, ngrp);
  const int K = pm.K, R = pm.R, F = pm.F, KF = K * F, F4 = F / 4;
  const float inv_k = 1.f / (float)K;
  float gm_acc[kPsK][kPsR], gs_acc[kPsK][kPsR];  // sums over the edges this lane owned
#pragma unroll
  for (int k = 0; k < kPsK; ++k)
#pragma unroll
    for (int d = 0; d < kPsR; ++d) {
      gm_acc[k][d] = 0.f;
      gs_acc[k][d] = 0.f;
    }
  float gp_acc[3 * kPsR];  // PROJ: (gP[d,0], gP[d,1], gpb[d])
#pragma unroll
  for (int i = 0; i < 3 * kPsR; ++i) gp_acc[i] = 0.f;
  if (active) {
    const PsKernels pk = load_kernels(mu, inv_sigma, K, R);
    const int32_t v = order[r];
    const int32_t beg = indptr[v], end = indptr[v + 1];
    ProjRegs pq;
    float cv = 0.f;
    if (PROJ) {
      pq = load_proj(pa, R);
      cv = pa.c[v];
    }
    const bool col_ok = li < K * F4;
    const int f4 = col_ok ? li % F4 : 0;
    const float4 g4 = col_ok ? ld4(gout + (int64_t)v * F + 4 * f4) : make_float4(0.f, 0.f, 0.f, 0.f);
    int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
    float* l_d = lds + grp * GS + G;  // [column lane][edge of the chunk]
    const float* my_row = hk + 4 * li;
    for (int32_t e0 = beg + gi * G; e0 < end; e0 += ngrp * G) {
      const bool e_ok = e0 + li < end;
      const int cnt = min(G, end - e0);
      int32_t u = 0;
      float m[kPsR];
      float cu = 0.f;
#pragma unroll
      for (int d = 0; d < kPsR; ++d) m[d] = 0.f;
      if (e_ok) {
        u = indices[e0 + li];
        if (PROJ) {
          cu = pa.c[u];
          project(pq, R, cu, cv, m);
        } else {
          load_pseudo(pseudo, e0 + li, R, m);
        }
      }
      wave_lds_fence();
      l_idx[li] = u;
      wave_lds_fence();
#pragma unroll
      for (int t0 = 0; t0 < G; t0 += kNrU) {
        if (t0 < cnt) {
          int idv[kNrU];
          read8i(l_idx + t0, idv);
          float4 rowv[kNrU];
#pragma unroll
          for (int t = 0; t < kNrU; ++t)
            if (col_ok && t0 + t < cnt) rowv[t] = ld4(my_row + (int64_t)idv[t] * KF);
          float dv[kNrU];
#pragma unroll
          for (int t = 0; t < kNrU; ++t) dv[t] = (col_ok && t0 + t < cnt) ? dot4(g4, rowv[t]) : 0.f;
          *reinterpret_cast<float4*>(l_d + li * G + t0) = make_float4(dv[0], dv[1], dv[2], dv[3]);
          *reinterpret_cast<float4*>(l_d + li * G + t0 + 4) = make_float4(dv[4], dv[5], dv[6], dv[7]);
        }
      }
      wave_lds_fence();
      if (e_ok) {
        float gm[kPsR];
#pragma unroll
        for (int d = 0; d < kPsR; ++d) gm[d] = 0.f;
#pragma unroll
        for (int k = 0; k < kPsK; ++k) {
          if (k >= K) continue;
          float dot = 0.f;
          for (int j = 0; j < F4; ++j) dot += l_d[(k * F4 + j) * G + li];
          const float dlog = dot * inv_k * gauss_k(pk, k, m);  // dw_k(e) w_k(e)
#pragma unroll
          for (int d = 0; d < kPsR; ++d) {
            const float diff = m[d] - pk.mu[k][d];
            const float is = pk.is[k][d];
            const float t = dlog * diff * is;  // padded dimensions: is = 0
            gm_acc[k][d] = fmaf(t, is, gm_acc[k][d]);
            gs_acc[k][d] = fmaf(-t, diff, gs_acc[k][d]);
            gm[d] = fmaf(-t, is, gm[d]);
          }
        }
        if (PROJ) {
#pragma unroll
          for (int d = 0; d < kPsR; ++d) {
            const float dpre = gm[d] * (1.f - m[d] * m[d]);  // through the tanh; padded dimensions: gm = 0
            gp_acc[3 * d] = fmaf(dpre, cu, gp_acc[3 * d]);
            gp_acc[3 * d + 1] = fmaf(dpre, cv, gp_acc[3 * d + 1]);
            gp_acc[3 * d + 2] += dpre;
          }
        } else if (gpseudo != nullptr) {
#pragma unroll
          for (int d = 0; d < kPsR; ++d)
            if (d < R) gpseudo[(int64_t)(e0 + li) * R + d] = gm[d];
        }
      }
    }
  }
  // the group's lanes are added in a fixed (butterfly) order, then the groups in order
#pragma unroll
  for (int k = 0; k < kPsK; ++k)
#pragma unroll
    for (int d = 0; d < kPsR; ++d) {
      if (k < K && d < R) {
        const float a = group_sum_from<G>(gm_acc[k][d], 1), b = group_sum_from<G>(gs_acc[k][d], 1);
        if (li == 0) {
          blk[grp][k * kPsR + d] = a;
          blk[grp][kPsK * kPsR + k * kPsR + d] = b;
        }
      } else if (li == 0) {
        blk[grp][k * kPsR + d] = 0.f;
        blk[grp][kPsK * kPsR + k * kPsR + d] = 0.f;
      }
    }
  if (PROJ) {
#pragma unroll
    for (int i = 0; i < 3 * kPsR; ++i) {
      float a = 0.f;
      if (i / 3 < R) a = group_sum_from<G>(gp_acc[i], 1);
      if (li == 0) blk[grp][kPsVals + i] = a;
    }
  }
  __syncthreads();
  if (threadIdx.x < NVALS) {
    float s = 0.f;
    for (int g2 = 0; g2 < GPB; ++g2) s += blk[g2][threadIdx.x];
    partial[(int64_t)blockIdx.x * NVALS + threadIdx.x] = s;
  }
}

// source side of backward: dhk[u, k, f] = (1/K) sum over out-edges w_k(e) gout[v, f]; the lanes of the K
// kernels read the same columns of gout[v]
template <int G, bool PROJ>
__global__ __launch_bounds__(kPsBlock) void k_gmmp_bwd_src_nr(
    RowLaunch rl, const int32_t* __restrict__ order_t, const int32_t* __restrict__ indptr_t,
    const int32_t* __restrict__ indices_t, const int32_t* __restrict__ eid_t,
    const float* __restrict__ pseudo, const float* __restrict__ pseudo_t /* nullable: pseudo in this walk's order */,
    ProjArgs pa, const float* __restrict__ mu, const float* __restrict__ inv_sigma,
    const float* __restrict__ gout, PsParams pm, float* __restrict__ dhk) {
  constexpr int GPB = kPsBlock / G;
  constexpr int GS = kNrGroupFloats<G>;
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float coop_buf[GPB * G * 4];
  const int li = threadIdx.x & (G - 1);
  const int grp = threadIdx.x / G;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  const int K = pm.K, R = pm.R, F = pm.F, KF = K * F, F4 = F / 4;
  const float inv_k = 1.f / (float)K;
  const PsKernels pk = load_kernels(mu, inv_sigma, K, R);
  const int32_t u = order_t[r];
  const int32_t beg = indptr_t[u], end = indptr_t[u + 1];
  ProjRegs pq;
  float cu = 0.f;
  if (PROJ) {
    pq = load_proj(pa, R);
    cu = pa.c[u];
  }
  const bool col_ok = li < K * F4;
  const int myk = col_ok ? li / F4 : 0;
  const int f4 = col_ok ? li % F4 : 0;
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + G;  // [kPsK][G]
  const float* my_row = gout + 4 * f4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f), part = acc;
  int folded = 0;
  for (int32_t p0 = beg + gi * G; p0 < end; p0 += ngrp * G) {
    const bool e_ok = p0 + li < end;
    const int cnt = min(G, end - p0);
    int32_t v = 0;
    float m[kPsR];
#pragma unroll
    for (int d = 0; d < kPsR; ++d) m[d] = 0.f;
    if (e_ok) {
      v = indices_t[p0 + li];
      if (PROJ) project(pq, R, cu, pa.c[v], m);
      else if (pseudo_t != nullptr) load_pseudo(pseudo_t, p0 + li, R, m);
      else load_pseudo(pseudo, eid_t[p0 + li], R, m);
    }
    wave_lds_fence();
    l_idx[li] = v;
#pragma unroll
    for (int k = 0; k < kPsK; ++k)
      if (k < K) l_w[k * G + li] = e_ok ? gauss_k(pk, k, m) * inv_k : 0.f;
    wave_lds_fence();
#pragma unroll
    for (int t0 = 0; t0 < G; t0 += kNrU) {
      if (t0 < cnt) {
        int idv[kNrU];
        float wv[kNrU];
        read8i(l_idx + t0, idv);
        float4 rowv[kNrU];
#pragma unroll
        for (int t = 0; t < kNrU; ++t)
          if (col_ok && t0 + t < cnt) rowv[t] = ld4(my_row + (int64_t)idv[t] * F);
        read8f(l_w + myk * G + t0, wv);
#pragma unroll
        for (int t = 0; t < kNrU; ++t)
          if (col_ok && t0 + t < cnt) fma4(part, wv[t], rowv[t]);
      }
    }
    folded += G;
    if (folded >= 32) {
      add4(acc, part);
      part = make_float4(0.f, 0.f, 0.f, 0.f);
      folded = 0;
    }
  }
  add4(acc, part);
  if (rr.coop) {
    float vv[4];
    pack4(vv, acc);
    coop_sum<G, 4, GPB>(coop_buf, vv, grp, li);
    if (grp != 0) return;
    acc = unpack4(vv);
  }
  if (col_ok) st4(dhk + (int64_t)u * KF + 4 * li, acc);
}

// ---- the projection that makes pseudo-coordinates from the degree pair ------------------------
// m[e,d] = tanh(P[d,0] c[u] + P[d,1] c[v] + pb[d]).  One wavefront per row of the walked list, lanes
// over its edges, four edges per lane in flight.  side 0: rows are destinations (CSR walk, the row's
// vertex is v); side 1: rows are sources (transposed list, the row's vertex is u) and the output is in
// that list's order.  What bounds a pass is the gather of c at the other end of every edge, one L1 line
// fill per edge (an edge-parallel version with perfectly even load took the same time).
__global__ void k_pseudo_proj_fwd(int32_t n, const int32_t* __restrict__ indptr,
                                  const int32_t* __restrict__ indices, const float* __restrict__ c, int R,
                                  const float* __restrict__ P, const float* __restrict__ pb, int side,
                                  float* __restrict__ pseudo) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 6;
  if (row >= n) return;
  const float c_row = c[row];
  const int32_t end = indptr[row + 1];
  for (int32_t e0 = indptr[row] + lane; e0 < end; e0 += 256) {
    float c_other[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) c_other[j] = e0 + 64 * j < end ? c[indices[e0 + 64 * j]] : 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (e0 + 64 * j >= end) continue;
      const float cu = side == 0 ? c_other[j] : c_row, cv = side == 0 ? c_row : c_other[j];
      for (int d = 0; d < R; ++d)
        pseudo[(int64_t)(e0 + 64 * j) * R + d] = tanhf(fmaf(P[2 * d], cu, fmaf(P[2 * d + 1], cv, pb[d])));
    }
  }
}

// partial[block][3 * kPsR]: (gP[d,0], gP[d,1], gpb[d]) for d < kPsR, summed over the block's rows.
// A wavefront takes every (number of wavefronts)-th row, so that the long rows of a power-law
// graph (they sit next to each other when vertices are numbered by weight) spread over the grid.
__global__ __launch_bounds__(kPsBlock) void k_pseudo_proj_bwd(
    int32_t n, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
    const float* __restrict__ c, int R, const float* __restrict__ pseudo, const float* __restrict__ gpseudo,
    float* __restrict__ partial) {
  __shared__ float red[kPsBlock / 64][3 * kPsR];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float s[3 * kPsR];
#pragma unroll
  for (int i = 0; i < 3 * kPsR; ++i) s[i] = 0.f;
  const int64_t waves = (int64_t)gridDim.x * (kPsBlock / 64);
  for (int64_t v = (int64_t)blockIdx.x * (kPsBlock / 64) + w; v < n; v += waves) {
    const float cv = c[v];
    const int32_t end = indptr[v + 1];
    for (int32_t e0 = indptr[v] + lane; e0 < end; e0 += 128) {  // two edges per lane in flight
      const int32_t e1 = e0 + 64;
      const bool ok1 = e1 < end;
      const float cu0 = c[indices[e0]], cu1 = ok1 ? c[indices[e1]] : 0.f;
#pragma unroll
      for (int d = 0; d < kPsR; ++d) {
        if (d >= R) continue;
        const float m0 = pseudo[(int64_t)e0 * R + d], q0 = gpseudo[(int64_t)e0 * R + d];
        const float m1 = ok1 ? pseudo[(int64_t)e1 * R + d] : 0.f, q1 = ok1 ? gpseudo[(int64_t)e1 * R + d] : 0.f;
        const float dpre0 = q0 * (1.f - m0 * m0), dpre1 = q1 * (1.f - m1 * m1);
        s[3 * d] = fmaf(dpre1, cu1, fmaf(dpre0, cu0, s[3 * d]));
        s[3 * d + 1] = fmaf(dpre1, cv, fmaf(dpre0, cv, s[3 * d + 1]));
        s[3 * d + 2] += dpre0 + dpre1;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 3 * kPsR; ++i) {
    float t = s[i];
    for (int off = 1; off < 64; off <<= 1) t += __shfl_xor(t, off, 64);
    if (lane == 0) red[w][i] = t;
  }
  __syncthreads();
  if (threadIdx.x < 3 * kPsR) {
    float t = 0.f;
    for (int q = 0; q < kPsBlock / 64; ++q) t += red[q][threadIdx.x];
    partial[(int64_t)blockIdx.x * 3 * kPsR + threadIdx.x] = t;
  }
}

__global__ void k_pseudo_proj_split(int R, const float* __restrict__ totals, float* __restrict__ gP,
                                    float* __restrict__ gpb) {
  const int d = threadIdx.x;
  if (d >= R) return;
  gP[2 * d] = totals[3 * d];
  gP[2 * d + 1] = totals[3 * d + 1];
  gpb[d] = totals[3 * d + 2];
}

// ---- host side --------------------------------------------------------------------------
template <int L>
static unsigned ps_grid(const gnn_graph_t* g, int side, RowLaunch& rl) {
  constexpr int GPB = kPsBlock / L;
  const RowSplit sp = split_rows(g, side, 4, GPB);  // edges are taken one at a time: count 4 as a chunk
  rl = RowLaunch{sp.hub.end, g->n};
  return sp.hub_grid + sp.rest_grid;
}

static int ps_lanes(int fout) { return pick_group(fout).L; }  // fout <= 256: one float4 slot per lane

// Lanes per group of the chunked kernels for narrow rows, 0 where they do not apply: the K * fout / 4
// float4 slots of a projected row must fit 16 lanes.
static int nr_lanes(int K, int fout) {
  const int q = K * fout / 4;
  if (q > 16 || config_get(kCfgForceSimple)) return 0;
  return q <= 8 ? 8 : 16;
}
template <int G>
static unsigned nr_grid(const gnn_graph_t* g, int side, RowLaunch& rl) {
  constexpr int GPB = kPsBlock / G;
  // an ordinary row is walked by one group, G edges at a time with 8 gathers in flight; rows from 64
  // such chunks on are shared by a workgroup
  const RowSplit sp = split_rows(g, side, 4 * G, GPB);
  rl = RowLaunch{sp.hub.end, g->n};
  return sp.hub_grid + sp.rest_grid;
}

// partial slots of the destination-side kernel: enough for either kernel family
static int64_t ps_dst_blocks(const gnn_graph_t* g, int fout) {
  RowLaunch rl;
  int64_t b;
  switch (ps_lanes(fout)) {
    case 4: b = ps_grid<4>(g, 0, rl); break;
    case 8: b = ps_grid<8>(g, 0, rl); break;
    case 16: b = ps_grid<16>(g, 0, rl); break;
    case 32: b = ps_grid<32>(g, 0, rl); break;
    default: b = ps_grid<64>(g, 0, rl); break;
  }
  const int64_t b8 = nr_grid<8>(g, 0, rl), b16 = nr_grid<16>(g, 0, rl);
  return std::max(b, std::max(b8, b16));
}

struct GmmpWs {
  size_t total, dhk, partial, gemm;
  int split_k;
  int64_t nblk;
};
static GmmpWs gmmp_ws_layout(const gnn_graph_t* g, int fin, int fout, int K) {
  GmmpWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += ws_granule(bytes); return o; };
  w.nblk = ps_dst_blocks(g, fout);
  w.dhk = take(sizeof(float) * (size_t)g->n * K * fout);
  w.partial = take(sizeof(float) * (size_t)(w.nblk + 1 + sum_partials_scratch_rows((int)w.nblk)) * kPsValsProj);
  w.split_k = gemm_pick_split_k(fin, K * fout, g->n);
  w.gemm = take(w.split_k > 1 ? sizeof(float) * (size_t)w.split_k * fin * K * fout : 0);
  w.total = off;
  return w;
}

static gnn_status_t gmmp_check(const gnn_graph_t* g, int fin, int fout, int K, int R, const char* who) {
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "%s: graph is null", who);
  GNN_REQUIRE(fin > 0 && fout > 0 && K > 0 && R > 0, GNN_ERR_INVALID_ARG, "%s: sizes must be positive", who);
  GNN_REQUIRE(fout % 4 == 0 && fout <= 256, GNN_ERR_UNSUPPORTED,
              "%s: fout = %d must be a multiple of 4, at most 256", who, fout);
  GNN_REQUIRE(K <= kPsK && R <= kPsR, GNN_ERR_UNSUPPORTED, "%s: at most %d kernels and %d dimensions", who, kPsK,
              kPsR);
  return GNN_OK;
}

// calls fn with the lane count of a row group as a compile-time constant
template <typename Fn>
static gnn_status_t for_lanes(int lanes, Fn fn) {
  switch (lanes) {
    case 4: return fn(std::integral_constant<int, 4>{});
    case 8: return fn(std::integral_constant<int, 8>{});
    case 16: return fn(std::integral_constant<int, 16>{});
    case 32: return fn(std::integral_constant<int, 32>{});
    default: return fn(std::integral_constant<int, 64>{});
  }
}

}  // namespace gnn

using namespace gnn;

extern "C" size_t gnn_gmmp_workspace_bytes(const gnn_graph_t* g, int fin, int fout, int k) {
  if (!g || fin <= 0 || fout <= 0 || k <= 0 || fout % 4 != 0 || fout > 256) return 0;
  return gmmp_ws_layout(g, fin, fout, k).total;
}

extern "C" gnn_status_t gnn_gmmp_fwd(const gnn_graph_t* g, int fin, int fout, int k, int r, const float* x,
                                     const float* w_fc, const float* pseudo, const float* mu,
                                     const float* inv_sigma, float* hk, float* out, void* stream) {
  clear_error();
  GNN_TRY(gmmp_check(g, fin, fout, k, r, "gnn_gmmp_fwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w_fc && mu && inv_sigma && hk && out && (pseudo || g->nnz == 0), GNN_ERR_INVALID_ARG,
              "gnn_gmmp_fwd: null pointer");
  GNN_REQUIRE(aligned16(hk) && aligned16(out), GNN_ERR_INVALID_ARG, "gnn_gmmp_fwd: hk, out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  GNN_TRY(gemm_f32(g->n, k * fout, fin, x, fin, false, w_fc, k * fout, false, hk, k * fout, 1, nullptr, st));
  const PsParams pm{k, r, fout};
  ProfScope p("gmmp_fwd_fused", st);
  if (const int G = nr_lanes(k, fout)) {
    return for_lanes(G, [&](auto lanes) -> gnn_status_t {
      constexpr int GL = decltype(lanes)::value == 8 ? 8 : 16;
      RowLaunch rl;
      const unsigned grid = nr_grid<GL>(g, 0, rl);
      if (grid != 0) {
        k_gmmp_fwd_nr<GL, false><<<grid, kPsBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, pseudo,
                                                           ProjArgs{}, mu, inv_sigma, pm, out);
        GNN_LAUNCH_CHECK();
      }
      return GNN_OK;
    });
  }
  return for_lanes(ps_lanes(fout), [&](auto lanes) -> gnn_status_t {
    constexpr int L = decltype(lanes)::value;
    RowLaunch rl;
    const unsigned grid = ps_grid<L>(g, 0, rl);
    if (grid != 0) {
      k_gmmp_fwd<L><<<grid, kPsBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, pseudo, mu, inv_sigma,
                                              pm, out);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  });
}

extern "C" gnn_status_t gnn_gmmp_bwd(const gnn_graph_t* g, int fin, int fout, int k, int r, const float* x,
                                     const float* w_fc, const float* pseudo, const float* mu,
                                     const float* inv_sigma, const float* hk, const float* gout, float* gx,
                                     float* gw_fc, float* gmu, float* ginv_sigma, float* gpseudo,
                                     const float* pseudo_t, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(gmmp_check(g, fin, fout, k, r, "gnn_gmmp_bwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w_fc && mu && inv_sigma && hk && gout && gw_fc && gmu && ginv_sigma && (pseudo || g->nnz == 0),
              GNN_ERR_INVALID_ARG, "gnn_gmmp_bwd: null pointer");
  GNN_REQUIRE(aligned16(hk) && aligned16(gout), GNN_ERR_INVALID_ARG,
              "gnn_gmmp_bwd: hk, gout must be 16-byte aligned");
  const GmmpWs W = gmmp_ws_layout(g, fin, fout, k);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= W.total, GNN_ERR_WORKSPACE,
              "gnn_gmmp_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, W.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_gmmp_bwd: workspace must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  float* dhk = reinterpret_cast<float*>(base + W.dhk);
  float* partial = reinterpret_cast<float*>(base + W.partial);
  float* part = reinterpret_cast<float*>(base + W.gemm);
  const PsParams pm{k, r, fout};
  const int KF = k * fout;
  {
    ProfScope p("gmmp_bwd_dst", st);
    unsigned grid = 0;
    const int G = nr_lanes(k, fout);
    GNN_TRY(for_lanes(G ? G : ps_lanes(fout), [&](auto lanes) -> gnn_status_t {
      constexpr int L = decltype(lanes)::value;
      constexpr int GL = L == 8 ? 8 : 16;
      RowLaunch rl;
      grid = G ? nr_grid<GL>(g, 0, rl) : ps_grid<L>(g, 0, rl);
      if (grid == 0) return GNN_OK;
      if (G)
        k_gmmp_bwd_dst_nr<GL, false><<<grid, kPsBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, pseudo,
                                                               ProjArgs{}, mu, inv_sigma, gout, pm, partial,
                                                               gpseudo);
      else
        k_gmmp_bwd_dst<L><<<grid, kPsBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, pseudo, mu,
                                                    inv_sigma, gout, pm, partial, gpseudo);
      GNN_LAUNCH_CHECK();
      return GNN_OK;
    }));
    float* totals = partial + (int64_t)grid * kPsVals;
    GNN_TRY(sum_partials_two_level(kPsVals, (int)grid, partial, totals + kPsVals, totals, st));
    k_gmmp_param_split<<<1, 64, 0, st>>>(k, r, totals, gmu, ginv_sigma);
    GNN_LAUNCH_CHECK();
  }
  {
    ProfScope p("gmmp_bwd_src", st);
    const int G = nr_lanes(k, fout);
    GNN_TRY(for_lanes(G ? G : ps_lanes(fout), [&](auto lanes) -> gnn_status_t {
      constexpr int L = decltype(lanes)::value;
      constexpr int GL = L == 8 ? 8 : 16;
      RowLaunch rl;
      const unsigned grid = G ? nr_grid<GL>(g, 1, rl) : ps_grid<L>(g, 1, rl);
      if (grid == 0) return GNN_OK;
      if (G)
        k_gmmp_bwd_src_nr<GL, false><<<grid, kPsBlock, 0, st>>>(rl, g->order[1], g->indptr_t, g->indices_t,
                                                               g->eid_t, pseudo, pseudo_t, ProjArgs{}, mu,
                                                               inv_sigma, gout, pm, dhk);
      else
        k_gmmp_bwd_src<L><<<grid, kPsBlock, 0, st>>>(rl, g->order[1], g->indptr_t, g->indices_t, g->eid_t, pseudo,
                                                    pseudo_t, mu, inv_sigma, gout, pm, dhk);
      GNN_LAUNCH_CHECK();
      return GNN_OK;
    }));
  }
  GNN_TRY(gemm_f32(fin, KF, g->n, x, fin, true, dhk, KF, false, gw_fc, KF, W.split_k, part, st));
  if (gx) GNN_TRY(gemm_f32(g->n, fin, KF, dhk, KF, false, w_fc, KF, true, gx, fin, 1, nullptr, st));
  return GNN_OK;
}

// workgroups of the projection's backward pass (= partial slots): four rows per workgroup, at most 2048
static int proj_blocks(int64_t n) {
  int64_t b = cdiv(n > 0 ? n : 1, kPsBlock / 64);
  return (int)(b > 2048 ? 2048 : b);
}

extern "C" size_t gnn_pseudo_proj_workspace_bytes(const gnn_graph_t* g) {
  if (!g) return 0;
  const int64_t blocks = proj_blocks(g->n);
  return ws_granule(sizeof(float) * (size_t)(blocks + 1 + sum_partials_scratch_rows((int)blocks)) * 3 * kPsR);
}

extern "C" gnn_status_t gnn_pseudo_proj_fwd(const gnn_graph_t* g, int r, const float* c, const float* proj_w,
                                            const float* proj_b, float* pseudo, float* pseudo_t, void* stream) {
  clear_error();
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "gnn_pseudo_proj_fwd: graph is null");
  GNN_REQUIRE(r > 0 && r <= kPsR, GNN_ERR_UNSUPPORTED, "gnn_pseudo_proj_fwd: r = %d outside 1..%d", r, kPsR);
  if (g->n == 0 || g->nnz == 0) return GNN_OK;
  GNN_REQUIRE(c && proj_w && proj_b && pseudo, GNN_ERR_INVALID_ARG, "gnn_pseudo_proj_fwd: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope p("pseudo_proj_fwd", st);
  const unsigned grid = (unsigned)cdiv((int64_t)g->n * 64, 256);
  k_pseudo_proj_fwd<<<grid, 256, 0, st>>>(g->n, g->indptr, g->indices, c, r, proj_w, proj_b, 0, pseudo);
  GNN_LAUNCH_CHECK();
  if (pseudo_t != nullptr) {
    k_pseudo_proj_fwd<<<grid, 256, 0, st>>>(g->n, g->indptr_t, g->indices_t, c, r, proj_w, proj_b, 1, pseudo_t);
    GNN_LAUNCH_CHECK();
  }
  return GNN_OK;
}

extern "C" gnn_status_t gnn_pseudo_proj_bwd(const gnn_graph_t* g, int r, const float* c, const float* pseudo,
                                            const float* gpseudo, float* gproj_w, float* gproj_b, void* ws,
                                            size_t ws_bytes, void* stream) {
  clear_error();
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "gnn_pseudo_proj_bwd: graph is null");
  GNN_REQUIRE(r > 0 && r <= kPsR, GNN_ERR_UNSUPPORTED, "gnn_pseudo_proj_bwd: r = %d outside 1..%d", r, kPsR);
  GNN_REQUIRE(gproj_w && gproj_b, GNN_ERR_INVALID_ARG, "gnn_pseudo_proj_bwd: null pointer");
  GNN_REQUIRE(ws != nullptr && ws_bytes >= gnn_pseudo_proj_workspace_bytes(g), GNN_ERR_WORKSPACE,
              "gnn_pseudo_proj_bwd: workspace of %zu bytes given, %zu needed", ws_bytes,
              gnn_pseudo_proj_workspace_bytes(g));
  GNN_REQUIRE(g->nnz == 0 || (c && pseudo && gpseudo), GNN_ERR_INVALID_ARG, "gnn_pseudo_proj_bwd: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope p("pseudo_proj_bwd", st);
  const int blocks = proj_blocks(g->n);
  float* partial = static_cast<float*>(ws);
  k_pseudo_proj_bwd<<<blocks, kPsBlock, 0, st>>>(g->n, g->indptr, g->indices, c, r, pseudo, gpseudo, partial);
  GNN_LAUNCH_CHECK();
  float* totals = partial + (int64_t)blocks * 3 * kPsR;
  GNN_TRY(sum_partials_two_level(3 * kPsR, blocks, partial, totals + 3 * kPsR, totals, st));
  k_pseudo_proj_split<<<1, 64, 0, st>>>(r, totals, gproj_w, gproj_b);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

// ---- MoNet layer with the projection of the degree pair fused in ------------------------------
static gnn_status_t monet_check(const gnn_graph_t* g, int fin, int fout, int K, int R, const char* who) {
  GNN_TRY(gmmp_check(g, fin, fout, K, R, who));
  GNN_REQUIRE(K * fout <= 64, GNN_ERR_UNSUPPORTED,
              "%s: k * fout = %d above 64 (wider layers: gnn_pseudo_proj_fwd + gnn_gmmp_fwd)", who, K * fout);
  return GNN_OK;
}

extern "C" size_t gnn_monet_workspace_bytes(const gnn_graph_t* g, int fin, int fout, int k) {
  return gnn_gmmp_workspace_bytes(g, fin, fout, k);
}

extern "C" gnn_status_t gnn_monet_fwd(const gnn_graph_t* g, int fin, int fout, int k, int r, const float* x,
                                      const float* w_fc, const float* c, const float* proj_w,
                                      const float* proj_b, const float* mu, const float* inv_sigma, float* hk,
                                      float* out, void* stream) {
  clear_error();
  GNN_TRY(monet_check(g, fin, fout, k, r, "gnn_monet_fwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w_fc && c && proj_w && proj_b && mu && inv_sigma && hk && out, GNN_ERR_INVALID_ARG,
              "gnn_monet_fwd: null pointer");
  GNN_REQUIRE(aligned16(hk) && aligned16(out), GNN_ERR_INVALID_ARG, "gnn_monet_fwd: hk, out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  GNN_TRY(gemm_f32(g->n, k * fout, fin, x, fin, false, w_fc, k * fout, false, hk, k * fout, 1, nullptr, st));
  const PsParams pm{k, r, fout};
  const ProjArgs pa{c, proj_w, proj_b};
  ProfScope p("monet_fwd_fused", st);
  return for_lanes(k * fout <= 32 ? 8 : 16, [&](auto lanes) -> gnn_status_t {
    constexpr int GL = decltype(lanes)::value == 8 ? 8 : 16;
    RowLaunch rl;
    const unsigned grid = nr_grid<GL>(g, 0, rl);
    if (grid != 0) {
      k_gmmp_fwd_nr<GL, true><<<grid, kPsBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, nullptr, pa, mu,
                                                        inv_sigma, pm, out);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  });
}

extern "C" gnn_status_t gnn_monet_bwd(const gnn_graph_t* g, int fin, int fout, int k, int r, const float* x,
                                      const float* w_fc, const float* c, const float* proj_w,
                                      const float* proj_b, const float* mu, const float* inv_sigma,
                                      const float* hk, const float* gout, float* gx, float* gw_fc, float* gmu,
                                      float* ginv_sigma, float* gproj_w, float* gproj_b, void* ws,
                                      size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(monet_check(g, fin, fout, k, r, "gnn_monet_bwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w_fc && c && proj_w && proj_b && mu && inv_sigma && hk && gout && gw_fc && gmu && ginv_sigma &&
                  gproj_w && gproj_b,
              GNN_ERR_INVALID_ARG, "gnn_monet_bwd: null pointer");
  GNN_REQUIRE(aligned16(hk) && aligned16(gout), GNN_ERR_INVALID_ARG,
              "gnn_monet_bwd: hk, gout must be 16-byte aligned");
  const GmmpWs W = gmmp_ws_layout(g, fin, fout, k);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= W.total, GNN_ERR_WORKSPACE,
              "gnn_monet_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, W.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_monet_bwd: workspace must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  float* dhk = reinterpret_cast<float*>(base + W.dhk);
  float* partial = reinterpret_cast<float*>(base + W.partial);
  float* part = reinterpret_cast<float*>(base + W.gemm);
  const PsParams pm{k, r, fout};
  const ProjArgs pa{c, proj_w, proj_b};
  const int KF = k * fout;
  const int G = KF <= 32 ? 8 : 16;
  {
    ProfScope p("monet_bwd_dst", st);
    unsigned grid = 0;
    GNN_TRY(for_lanes(G, [&](auto lanes) -> gnn_status_t {
      constexpr int GL = decltype(lanes)::value == 8 ? 8 : 16;
      RowLaunch rl;
      grid = nr_grid<GL>(g, 0, rl);
      if (grid == 0) return GNN_OK;
      k_gmmp_bwd_dst_nr<GL, true><<<grid, kPsBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, nullptr, pa,
                                                            mu, inv_sigma, gout, pm, partial, nullptr);
      GNN_LAUNCH_CHECK();
      return GNN_OK;
    }));
    float* totals = partial + (int64_t)grid * kPsValsProj;
    GNN_TRY(sum_partials_two_level(kPsValsProj, (int)grid, partial, totals + kPsValsProj, totals, st));
    k_gmmp_param_split<<<1, 64, 0, st>>>(k, r, totals, gmu, ginv_sigma);
    GNN_LAUNCH_CHECK();
    k_pseudo_proj_split<<<1, 64, 0, st>>>(r, totals + kPsVals, gproj_w, gproj_b);
    GNN_LAUNCH_CHECK();
  }
  {
    ProfScope p("monet_bwd_src", st);
    GNN_TRY(for_lanes(G, [&](auto lanes) -> gnn_status_t {
      constexpr int GL = decltype(lanes)::value == 8 ? 8 : 16;
      RowLaunch rl;
      const unsigned grid = nr_grid<GL>(g, 1, rl);
      if (grid == 0) return GNN_OK;
      k_gmmp_bwd_src_nr<GL, true><<<grid, kPsBlock, 0, st>>>(rl, g->order[1], g->indptr_t, g->indices_t, g->eid_t,
                                                            nullptr, nullptr, pa, mu, inv_sigma, gout, pm, dhk);
      GNN_LAUNCH_CHECK();
      return GNN_OK;
    }));
  }
  GNN_TRY(gemm_f32(fin, KF, g->n, x, fin, true, dhk, KF, false, gw_fc, KF, W.split_k, part, st));
  if (gx) GNN_TRY(gemm_f32(g->n, fin, KF, dhk, KF, false, w_fc, KF, true, gx, fin, 1, nullptr, st));
  return GNN_OK;
}
