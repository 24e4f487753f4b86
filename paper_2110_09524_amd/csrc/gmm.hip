// MoNet / GMMConv layer (App. A.2 "GMMConv").  MoNet has no leading Scatter, so no
// reorganization is needed (Sec. 7.2 "MoNet"); the Gaussian weights (ApplyEdge)
// and the Aggregate are fused into one destination-walking kernel, and the weights
// are recomputed in the backward pass instead of being stored (Sec. 7.3).
//
// Notation: m_e = (c[u], c[v]), t_jd = (m_d - mu[j,d]) inv_sigma[j,d],
// w_j(e) = exp(-1/2 (t_j0^2 + t_j1^2)), out[v] = (1/K) sum_e sum_j w_j(e) hk[u,j,:].
//
// Backward.  dw_j(e) = (1/K) <gout[v], hk[u,j,:]> would need one dot product per
// edge and kernel; by the distributive law the dot product is taken after the
// neighbourhood sum instead.  Per destination v and kernel j the kernel aggregates
//   A_j = sum_e w_j hk[u,j,:],  R_j = sum_e w_j (c[u]-mu_j0) hk[u,j,:],
//   S_j = sum_e w_j (c[u]-mu_j0)^2 hk[u,j,:]
// and then, with tA = <gout[v], A_j> etc. (the second coordinate c[v] is constant
// along a destination row):
//   gmu[j,0]  += tR is_j0^2 / K             gmu[j,1]  += tA (c[v]-mu_j1) is_j1^2 / K
//   gis[j,0]  += -tS is_j0 / K              gis[j,1]  += -tA (c[v]-mu_j1)^2 is_j1 / K
// summed over destinations in a fixed two-stage order.  The source side
//   dhk[u,j,:] = (1/K) sum over out-edges w_j(e) gout[v,:]
// walks the CSC transpose (no atomics).
#include "common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kGmmBlock = 256;
constexpr int kMaxK = 8;

struct GmmParams {
  int K, F;
};

__device__ __forceinline__ float gauss_w(float cu, float cv, float mu0, float mu1, float is0, float is1) {
  const float t0 = (cu - mu0) * is0, t1 = (cv - mu1) * is1;
  return __expf(-0.5f * (t0 * t0 + t1 * t1));
}

constexpr int kGmmKB = 4;  // kernels handled per pass over a row's edges
constexpr int kGmmU = 2;   // edges whose rows are in flight together in the row phase

// Both destination-walking kernels work on chunks of L edges in two phases.  Chunk phase:
// lane li owns edge c0 + li, gathers c[u] and evaluates the Gaussian weights of up to kGmmKB
// kernels (one exp per edge and kernel, not one per lane); edges past the end of the row
// become vertex 0 with weight 0, so the row phase needs no per-edge conditionals.  Row phase:
// lanes own columns; kGmmU edges x kGmmKB kernel rows are loaded before they are used.

// ---- a9: fused forward -----------------------------------------------------------------
template <int L, int NV>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_fwd(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ hk, const float* __restrict__ c,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma, GmmParams pm,
    float* __restrict__ out) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kGmmBlock / kWave);
  constexpr int KB = kGmmKB, U = kGmmU;
  constexpr int NC = 4 * NV;
  constexpr int GS = (1 + KB) * L;  // LDS floats per group: idx | w[KB][L]
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float coop_buf[GPB * L * NC];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + L;

  const int K = pm.K, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  const int32_t v = order[r];
  const int32_t beg = indptr[v], end = indptr[v + 1];
  const float cv = c[v];

  bool slot_ok[NV];
  float4 acc[NV], part[NV];  // two-level summation: `part` collects a few chunks, then folds into `acc`
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    slot_ok[j] = 4 * (li + j * L) < F;
    acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    part[j] = acc[j];
  }
  for (int k0 = 0; k0 < K; k0 += KB) {
    float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const bool ok = k0 + q < K;
      mu0[q] = ok ? mu[2 * (k0 + q)] : 0.f;
      mu1[q] = ok ? mu[2 * (k0 + q) + 1] : 0.f;
      is0[q] = ok ? inv_sigma[2 * (k0 + q)] : 0.f;
      is1[q] = ok ? inv_sigma[2 * (k0 + q) + 1] : 0.f;
    }
    constexpr int kFold = L >= 32 ? 1 : 32 / L;  // `part` is folded into `acc` every ~32 edges
    int chunk_no = 0;
    for (int32_t c0 = beg + gi * L; c0 < end; c0 += ngrp * L) {
      const bool e_ok = c0 + li < end;
      const int32_t u = e_ok ? indices[c0 + li] : 0;
      const float cu = c[u];
      l_idx[li] = u;
#pragma unroll
      for (int q = 0; q < KB; ++q)
        l_w[q * L + li] = (e_ok && k0 + q < K) ? gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) * inv_k : 0.f;
      wave_lds_fence();
      const int cnt = min(L, end - c0);
      for (int t0 = 0; t0 < cnt; t0 += U) {
        int uu[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
          uu[t] = l_idx[t0 + t];
          if (L == 64) uu[t] = __builtin_amdgcn_readfirstlane(uu[t]);
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          if (!slot_ok[j]) continue;
          float4 rowv[U][KB];
#pragma unroll
          for (int t = 0; t < U; ++t)
#pragma unroll
            for (int q = 0; q < KB; ++q)
              if (k0 + q < K) rowv[t][q] = ld4(hk + (int64_t)uu[t] * KF + (k0 + q) * F + 4 * (li + j * L));
#pragma unroll
          for (int t = 0; t < U; ++t)
#pragma unroll
            for (int q = 0; q < KB; ++q)
              if (k0 + q < K) fma4(part[j], l_w[q * L + t0 + t], rowv[t][q]);
        }
      }
      if ((++chunk_no % kFold) == 0) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          add4(acc[j], part[j]);
          part[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
      wave_lds_fence();
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      add4(acc[j], part[j]);
      part[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  if (rr.coop) {
    float vv[NC];
#pragma unroll
    for (int j = 0; j < NV; ++j) pack4(vv + 4 * j, acc[j]);
    coop_sum<L, NC, GPB>(coop_buf, vv, grp, li);
    if (grp != 0) return;
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = unpack4(vv + 4 * j);
  }
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j]) st4(out + (int64_t)v * F + 4 * (li + j * L), acc[j]);
}

// ---- a9, edge-balanced mapping (Sec. 5) ---------------------------------------------------
// A group owns kGmmEbEdges consecutive positions of the edge array instead of a row: it finds
// the row of its first edge by bisection of indptr and walks row by row inside its run.  For
// each row piece the lanes first evaluate the Gaussian weights (lanes = edges), then aggregate
// (lanes = columns).  A row that lies inside the run is stored, a row that continues into other
// runs is added atomically onto an output zeroed before (rows of more than two pieces depend
// on arrival order in the last bits).  At most kGmmKB kernels.
constexpr int kGmmEbEdges = 32;

__global__ void k_gmm_zero_f4(int64_t quads, float* __restrict__ p) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < quads) st4(p + 4 * i, make_float4(0.f, 0.f, 0.f, 0.f));
}

template <int L, int NV>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_fwd_eb(
    int32_t n, int32_t nnz, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
    const float* __restrict__ hk, const float* __restrict__ c, const float* __restrict__ mu,
    const float* __restrict__ inv_sigma, GmmParams pm, float* __restrict__ out) {
  constexpr int GPB = kGmmBlock / L;
  constexpr int KB = kGmmKB, U = kGmmU, RUN = kGmmEbEdges;
  constexpr int GS = (1 + KB) * (RUN + U);  // idx | w[KB], each with U entries of padding
  __shared__ __align__(16) float lds[GPB * GS];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t run = (int64_t)blockIdx.x * GPB + grp;
  if (run * RUN >= nnz) return;
  const int32_t e0 = (int32_t)(run * RUN);
  const int32_t e1 = min(e0 + RUN, nnz);
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + (RUN + U);
  const int K = pm.K, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;

  for (int i = li; i < RUN + U; i += L) {
    l_idx[i] = e0 + i < e1 ? indices[e0 + i] : 0;  // padding gathers row 0 with weight 0
#pragma unroll
    for (int q = 0; q < KB; ++q) l_w[q * (RUN + U) + i] = 0.f;
  }
  float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
  for (int q = 0; q < KB; ++q) {
    const bool ok = q < K;
    mu0[q] = ok ? mu[2 * q] : 0.f;
    mu1[q] = ok ? mu[2 * q + 1] : 0.f;
    is0[q] = ok ? inv_sigma[2 * q] : 0.f;
    is1[q] = ok ? inv_sigma[2 * q + 1] : 0.f;
  }
  // row of the first edge: indptr[lo] <= e0 < indptr[hi] throughout
  int32_t lo = 0, hi = n;
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (indptr[mid] <= e0) lo = mid; else hi = mid;
  }
  int32_t v = lo, row_beg = indptr[v], row_end = indptr[v + 1];
  wave_lds_fence();

  bool slot_ok[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) slot_ok[j] = 4 * (li + j * L) < F;

  int32_t e = e0;
  while (e < e1) {
    const int32_t seg_end = min(row_end, e1);
    const float cv = c[v];
    // chunk phase: the weights of this row piece (edges outside it keep weight 0 from the start
    // or get it back below)
    for (int32_t t = e + li; t < seg_end; t += L) {
      const float cu = c[l_idx[t - e0]];
#pragma unroll
      for (int q = 0; q < KB; ++q)
        if (q < K) l_w[q * (RUN + U) + (t - e0)] = gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) * inv_k;
    }
    wave_lds_fence();
    float4 acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t t0 = e; t0 < seg_end; t0 += U) {
      int uu[U];
      float ok[U];
#pragma unroll
      for (int t = 0; t < U; ++t) {
        uu[t] = l_idx[t0 - e0 + t];
        if (L == 64) uu[t] = __builtin_amdgcn_readfirstlane(uu[t]);
        ok[t] = t0 + t < seg_end ? 1.f : 0.f;  // entries past the piece belong to the next row
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        if (!slot_ok[j]) continue;
        float4 rowv[U][KB];
#pragma unroll
        for (int t = 0; t < U; ++t)
#pragma unroll
          for (int q = 0; q < KB; ++q)
            if (q < K) rowv[t][q] = ld4(hk + (int64_t)uu[t] * KF + q * F + 4 * (li + j * L));
#pragma unroll
        for (int t = 0; t < U; ++t)
#pragma unroll
          for (int q = 0; q < KB; ++q)
            if (q < K) fma4(acc[j], ok[t] * l_w[q * (RUN + U) + (t0 - e0 + t)], rowv[t][q]);
      }
    }
    const bool whole = row_beg >= e0 && row_end <= e1;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (!slot_ok[j]) continue;
      float* o = out + (int64_t)v * F + 4 * (li + j * L);
      if (whole) {
        st4(o, acc[j]);
      } else {
        unsafeAtomicAdd(o, acc[j].x);
        unsafeAtomicAdd(o + 1, acc[j].y);
        unsafeAtomicAdd(o + 2, acc[j].z);
        unsafeAtomicAdd(o + 3, acc[j].w);
      }
    }
    e = seg_end;
    if (e < e1) {  // the next row that has edges starts at e
      do {
        ++v;
        row_beg = row_end;
        row_end = indptr[v + 1];
      } while (row_end == row_beg);
    }
  }
}

// ---- aggregate first, project afterwards (fin < K * fout) -----------------------------------
// The projection is linear, so it commutes with the weighted sums (the observation behind Sec. 4,
// applied in the other direction):
//   out[v] = (1/K) sum_j ( sum_e w_j(e) x[u] ) W_j = (1/K) sum_j agg_j[v] W_j .
// When the input row is narrower than the K projected rows, an edge then gathers fin floats once
// instead of K * fout, and the projection becomes one dense product on vertices,
// out = agg [n, K*fin] . W' [K*fin, fout].  The destination side of backward changes the same way:
// <gout[v], hk[u,j,:]> = <G_j[v], x[u]> with G = gout W'^T, so it gathers x as well.
template <int L>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_fwd_x(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ x, const float* __restrict__ c,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma, int K, int fin,
    float* __restrict__ agg /* [n, K*fin] */) {
  constexpr int GPB = kGmmBlock / L;
  constexpr int KB = kGmmKB, U = 4;
  constexpr int GS = (1 + KB) * L;
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float coop_buf[GPB * L * 4 * KB];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + L;
  const float inv_k = 1.f / (float)K;
  const int32_t v = order[r];
  const int32_t beg = indptr[v], end = indptr[v + 1];
  const float cv = c[v];
  const bool col_ok = 4 * li < fin;
  for (int k0 = 0; k0 < K; k0 += KB) {
    float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const bool ok = k0 + q < K;
      mu0[q] = ok ? mu[2 * (k0 + q)] : 0.f;
      mu1[q] = ok ? mu[2 * (k0 + q) + 1] : 0.f;
      is0[q] = ok ? inv_sigma[2 * (k0 + q)] : 0.f;
      is1[q] = ok ? inv_sigma[2 * (k0 + q) + 1] : 0.f;
    }
    float4 acc[KB], part[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      part[q] = acc[q];
    }
    constexpr int kFold = L >= 32 ? 1 : 32 / L;  // two-level summation, as in k_gmm_fwd
    int chunk_no = 0;
    for (int32_t c0 = beg + gi * L; c0 < end; c0 += ngrp * L) {
      const bool e_ok = c0 + li < end;
      const int32_t u = e_ok ? indices[c0 + li] : 0;
      const float cu = c[u];
      l_idx[li] = u;
#pragma unroll
      for (int q = 0; q < KB; ++q)
        l_w[q * L + li] = (e_ok && k0 + q < K) ? gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) * inv_k : 0.f;
      wave_lds_fence();
      const int cnt = min(L, end - c0);
      if (col_ok) {
        for (int t0 = 0; t0 < cnt; t0 += U) {
          float4 rowv[U];
#pragma unroll
          for (int t = 0; t < U; ++t) {
            int uu = l_idx[min(t0 + t, L - 1)];  // past the chunk: a valid vertex with weight 0 or an unused slot
            if (L == 64) uu = __builtin_amdgcn_readfirstlane(uu);
            rowv[t] = ld4(x + (int64_t)uu * fin + 4 * li);
          }
#pragma unroll
          for (int t = 0; t < U; ++t) {
            if (t0 + t < L) {
#pragma unroll
              for (int q = 0; q < KB; ++q) fma4(part[q], l_w[q * L + t0 + t], rowv[t]);
            }
          }
        }
      }
      if ((++chunk_no % kFold) == 0) {
#pragma unroll
        for (int q = 0; q < KB; ++q) {
          add4(acc[q], part[q]);
          part[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
      wave_lds_fence();
    }
#pragma unroll
    for (int q = 0; q < KB; ++q) add4(acc[q], part[q]);
    if (rr.coop) {  // every group of the workgroup shares the row and runs the same passes
      float vv[4 * KB];
#pragma unroll
      for (int q = 0; q < KB; ++q) pack4(vv + 4 * q, acc[q]);
      coop_sum<L, 4 * KB, GPB>(coop_buf, vv, grp, li);
#pragma unroll
      for (int q = 0; q < KB; ++q) acc[q] = unpack4(vv + 4 * q);
    }
    if (col_ok && (!rr.coop || grp == 0)) {
#pragma unroll
      for (int q = 0; q < KB; ++q)
        if (k0 + q < K) st4(agg + ((int64_t)v * K + k0 + q) * fin + 4 * li, acc[q]);
    }
  }
}

// destination side of backward on gathered x rows; G [n, K*fin] = gout W'^T.  Partials as k_gmm_bwd_dst.
template <int L>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_bwd_dst_x(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ x, const float* __restrict__ c,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma, const float* __restrict__ G, int K,
    int fin, float* __restrict__ partial) {
  constexpr int GPB = kGmmBlock / L;
  constexpr int KB = kGmmKB, U = 4;
  constexpr int GS = (1 + 3 * KB) * L;
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float blk[GPB][kMaxK][4];
  __shared__ float coop_buf[GPB * L * 3];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  const bool active = pick_row<GPB>(rl, grp, rr, r, gi, ngrp);
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + L;
  float* l_wr = l_w + KB * L;
  float* l_ws = l_wr + KB * L;
  const float inv_k = 1.f / (float)K;
  for (int i = li; i < kMaxK * 4; i += L) blk[grp][i >> 2][i & 3] = 0.f;
  if (active) {
    const int32_t v = order[r];
    const int32_t beg = indptr[v], end = indptr[v + 1];
    const float cv = c[v];
    const bool col_ok = 4 * li < fin;
    for (int k0 = 0; k0 < K; k0 += KB) {
      float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        const bool ok = k0 + q < K;
        mu0[q] = ok ? mu[2 * (k0 + q)] : 0.f;
        mu1[q] = ok ? mu[2 * (k0 + q) + 1] : 0.f;
        is0[q] = ok ? inv_sigma[2 * (k0 + q)] : 0.f;
        is1[q] = ok ? inv_sigma[2 * (k0 + q) + 1] : 0.f;
      }
      float4 aA[KB], aR[KB], aS[KB];
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        aA[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        aR[q] = aA[q];
        aS[q] = aA[q];
      }
      for (int32_t c0 = beg + gi * L; c0 < end; c0 += ngrp * L) {
        const bool e_ok = c0 + li < end;
        const int32_t u = e_ok ? indices[c0 + li] : 0;
        const float cu = c[u];
        l_idx[li] = u;
#pragma unroll
        for (int q = 0; q < KB; ++q) {
          const float w = (e_ok && k0 + q < K) ? gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) : 0.f;
          const float d0 = cu - mu0[q];
          l_w[q * L + li] = w;
          l_wr[q * L + li] = w * d0;
          l_ws[q * L + li] = w * d0 * d0;
        }
        wave_lds_fence();
        const int cnt = min(L, end - c0);
        if (col_ok) {
          for (int t0 = 0; t0 < cnt; t0 += U) {
            float4 rowv[U];
#pragma unroll
            for (int t = 0; t < U; ++t) {
              int uu = l_idx[min(t0 + t, L - 1)];
              if (L == 64) uu = __builtin_amdgcn_readfirstlane(uu);
              rowv[t] = ld4(x + (int64_t)uu * fin + 4 * li);
            }
#pragma unroll
            for (int t = 0; t < U; ++t) {
              if (t0 + t < L) {
#pragma unroll
                for (int q = 0; q < KB; ++q) {
                  fma4(aA[q], l_w[q * L + t0 + t], rowv[t]);
                  fma4(aR[q], l_wr[q * L + t0 + t], rowv[t]);
                  fma4(aS[q], l_ws[q * L + t0 + t], rowv[t]);
                }
              }
            }
          }
        }
        wave_lds_fence();
      }
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        if (k0 + q >= K) continue;
        float tA = 0.f, tR = 0.f, tS = 0.f;
        if (col_ok) {
          const float4 g4 = ld4(G + ((int64_t)v * K + k0 + q) * fin + 4 * li);
          tA = dot4(g4, aA[q]);
          tR = dot4(g4, aR[q]);
          tS = dot4(g4, aS[q]);
        }
        tA = group_sum_from<L>(tA, 1);
        tR = group_sum_from<L>(tR, 1);
        tS = group_sum_from<L>(tS, 1);
        if (rr.coop) {
          float vv[3] = {tA, tR, tS};
          coop_sum<L, 3, GPB>(coop_buf, vv, grp, li);
          tA = vv[0]; tR = vv[1]; tS = vv[2];
        }
        if (li == 0 && (!rr.coop || grp == 0)) {
          const float d1 = cv - mu1[q];
          blk[grp][k0 + q][0] = tR * is0[q] * is0[q] * inv_k;
          blk[grp][k0 + q][1] = tA * d1 * is1[q] * is1[q] * inv_k;
          blk[grp][k0 + q][2] = -tS * is0[q] * inv_k;
          blk[grp][k0 + q][3] = -tA * d1 * d1 * is1[q] * inv_k;
        }
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < kMaxK * 4) {
    const int k = threadIdx.x >> 2, q = threadIdx.x & 3;
    float s = 0.f;
    for (int g2 = 0; g2 < GPB; ++g2) s += blk[g2][k][q];  // fixed order
    partial[((int64_t)blockIdx.x * kMaxK + k) * 4 + q] = s;
  }
}

// W'[(k*fin + i), f] = w_fc[i, k*F + f]
__global__ void k_gmm_wt(int fin, int K, int F, const float* __restrict__ w_fc, float* __restrict__ wt) {
  const int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (t >= (int64_t)fin * K * F) return;
  const int f = (int)(t % F);
  const int64_t ki = t / F;
  const int i = (int)(ki % fin), k = (int)(ki / fin);
  wt[t] = w_fc[(int64_t)i * K * F + (int64_t)k * F + f];
}

// ---- a10, destination side: gradients of mu and inv_sigma (CSR walk) ------------------
// partial[block][j][4] = this block's share of (gmu_j0, gmu_j1, gis_j0, gis_j1)
template <int L, int NV>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_bwd_dst(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ hk, const float* __restrict__ c,
    const float* __restrict__ mu, const float* __restrict__ inv_sigma, const float* __restrict__ gout,
    GmmParams pm, float* __restrict__ partial) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kGmmBlock / kWave);
  constexpr int KB = kGmmKB, U = kGmmU;
  constexpr int GS = (1 + 3 * KB) * L;  // LDS floats per group: idx | w[KB][L] | wr[KB][L] | ws[KB][L]
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float blk[GPB][kMaxK][4];
  __shared__ float coop_buf[GPB * L * 3];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  const bool active = pick_row<GPB>(rl, grp, rr, r, gi, ngrp);  // coop: the same for the whole workgroup
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + L;
  float* l_wr = l_w + KB * L;
  float* l_ws = l_wr + KB * L;

  const int K = pm.K, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  if (li < kMaxK) {
    blk[grp][li][0] = 0.f; blk[grp][li][1] = 0.f; blk[grp][li][2] = 0.f; blk[grp][li][3] = 0.f;
  }
  if (L < kMaxK) {  // L == 4: lanes 0..3 also clear kernels 4..7
    if (li + 4 < kMaxK) {
      blk[grp][li + 4][0] = 0.f; blk[grp][li + 4][1] = 0.f; blk[grp][li + 4][2] = 0.f; blk[grp][li + 4][3] = 0.f;
    }
  }
  if (active) {
    const int32_t v = order[r];
    const int32_t beg = indptr[v], end = indptr[v + 1];
    const float cv = c[v];
    bool slot_ok[NV];
    float4 g4[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      slot_ok[j] = 4 * (li + j * L) < F;
      g4[j] = slot_ok[j] ? ld4(gout + (int64_t)v * F + 4 * (li + j * L)) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int k0 = 0; k0 < K; k0 += KB) {
      float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        const bool ok = k0 + q < K;
        mu0[q] = ok ? mu[2 * (k0 + q)] : 0.f;
        mu1[q] = ok ? mu[2 * (k0 + q) + 1] : 0.f;
        is0[q] = ok ? inv_sigma[2 * (k0 + q)] : 0.f;
        is1[q] = ok ? inv_sigma[2 * (k0 + q) + 1] : 0.f;
      }
      // a row that is not shared by the workgroup has fewer than kCoopChunks chunks, a shared
      // one is cut into GPB interleaved parts: either way one running sum sees few terms
      float4 aA[KB][NV], aR[KB][NV], aS[KB][NV];
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          aA[q][j] = make_float4(0.f, 0.f, 0.f, 0.f);
          aR[q][j] = aA[q][j];
          aS[q][j] = aA[q][j];
        }
      for (int32_t c0 = beg + gi * L; c0 < end; c0 += ngrp * L) {
        const bool e_ok = c0 + li < end;
        const int32_t u = e_ok ? indices[c0 + li] : 0;
        const float cu = c[u];
        l_idx[li] = u;
#pragma unroll
        for (int q = 0; q < KB; ++q) {
          const float w = (e_ok && k0 + q < K) ? gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) : 0.f;
          const float d0 = cu - mu0[q];
          l_w[q * L + li] = w;
          l_wr[q * L + li] = w * d0;
          l_ws[q * L + li] = w * d0 * d0;
        }
        wave_lds_fence();
        const int cnt = min(L, end - c0);
        for (int t0 = 0; t0 < cnt; t0 += U) {
          int uu[U];
#pragma unroll
          for (int t = 0; t < U; ++t) {
            uu[t] = l_idx[t0 + t];
            if (L == 64) uu[t] = __builtin_amdgcn_readfirstlane(uu[t]);
          }
#pragma unroll
          for (int j = 0; j < NV; ++j) {
            if (!slot_ok[j]) continue;
            float4 rowv[U][KB];
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
              for (int q = 0; q < KB; ++q)
                if (k0 + q < K) rowv[t][q] = ld4(hk + (int64_t)uu[t] * KF + (k0 + q) * F + 4 * (li + j * L));
#pragma unroll
            for (int t = 0; t < U; ++t)
#pragma unroll
              for (int q = 0; q < KB; ++q)
                if (k0 + q < K) {
                  fma4(aA[q][j], l_w[q * L + t0 + t], rowv[t][q]);
                  fma4(aR[q][j], l_wr[q * L + t0 + t], rowv[t][q]);
                  fma4(aS[q][j], l_ws[q * L + t0 + t], rowv[t][q]);
                }
          }
        }
        wave_lds_fence();
      }
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        if (k0 + q >= K) continue;
        float tA = 0.f, tR = 0.f, tS = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          tA += dot4(g4[j], aA[q][j]);
          tR += dot4(g4[j], aR[q][j]);
          tS += dot4(g4[j], aS[q][j]);
        }
        tA = group_sum_from<L>(tA, 1);
        tR = group_sum_from<L>(tR, 1);
        tS = group_sum_from<L>(tS, 1);
        if (rr.coop) {
          float vv[3] = {tA, tR, tS};
          coop_sum<L, 3, GPB>(coop_buf, vv, grp, li);
          tA = vv[0]; tR = vv[1]; tS = vv[2];
        }
        if (li == 0 && (!rr.coop || grp == 0)) {
          const float d1 = cv - mu1[q];
          blk[grp][k0 + q][0] = tR * is0[q] * is0[q] * inv_k;
          blk[grp][k0 + q][1] = tA * d1 * is1[q] * is1[q] * inv_k;
          blk[grp][k0 + q][2] = -tS * is0[q] * inv_k;
          blk[grp][k0 + q][3] = -tA * d1 * d1 * is1[q] * inv_k;
        }
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < kMaxK * 4) {
    const int k = threadIdx.x >> 2, q = threadIdx.x & 3;
    float s = 0.f;
    for (int gi = 0; gi < GPB; ++gi) s += blk[gi][k][q];  // fixed order
    partial[((int64_t)blockIdx.x * kMaxK + k) * 4 + q] = s;
  }
}

// totals[j][4] -> gmu[j, 0..1], gis[j, 0..1]
__global__ void k_gmm_param_split(int K, const float* __restrict__ totals, float* __restrict__ gmu,
                                  float* __restrict__ gis) {
  const int t = threadIdx.x;  // (k, q)
  if (t >= K * 4) return;
  const int k = t >> 2, q = t & 3;
  if (q < 2) gmu[2 * k + q] = totals[t]; else gis[2 * k + (q - 2)] = totals[t];
}

// ---- a10, source side: dhk[u,j,:] = (1/K) sum over out-edges w_j(e) gout[v,:] ----------
template <int L, int NV>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_bwd_src(
    RowLaunch rl, const int32_t* __restrict__ order_t, const int32_t* __restrict__ indptr_t,
    const int32_t* __restrict__ indices_t, const float* __restrict__ c, const float* __restrict__ mu,
    const float* __restrict__ inv_sigma, const float* __restrict__ gout, GmmParams pm,
    float* __restrict__ dhk) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kGmmBlock / kWave);
  constexpr int KB = kGmmKB;  // kernels accumulated per pass over the out-edges
  constexpr int U = 4;        // gathered rows in flight per lane
  constexpr int NC = 4 * KB * NV;
  constexpr int GS = (1 + KB) * L;  // LDS floats per group: idx | w[KB][L]
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float coop_buf[GPB * L * NC];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + L;

  const int K = pm.K, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  const int32_t u = order_t[r];
  const int32_t beg = indptr_t[u], end = indptr_t[u + 1];
  const float cu = c[u];
  bool slot_ok[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) slot_ok[j] = 4 * (li + j * L) < F;

  for (int k0 = 0; k0 < K; k0 += KB) {
    float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const bool ok = k0 + q < K;
      mu0[q] = ok ? mu[2 * (k0 + q)] : 0.f;
      mu1[q] = ok ? mu[2 * (k0 + q) + 1] : 0.f;
      is0[q] = ok ? inv_sigma[2 * (k0 + q)] : 0.f;
      is1[q] = ok ? inv_sigma[2 * (k0 + q) + 1] : 0.f;
    }
    float4 acc[KB][NV];
#pragma unroll
    for (int q = 0; q < KB; ++q)
#pragma unroll
      for (int j = 0; j < NV; ++j) acc[q][j] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t c0 = beg + gi * L; c0 < end; c0 += ngrp * L) {
      // chunk phase: lane li owns out-edge c0 + li; edges past the end become vertex 0, weight 0
      const bool e_ok = c0 + li < end;
      const int32_t v = e_ok ? indices_t[c0 + li] : 0;
      const float cv = c[v];
      l_idx[li] = v;
#pragma unroll
      for (int q = 0; q < KB; ++q)
        l_w[q * L + li] = (e_ok && k0 + q < K) ? gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) * inv_k : 0.f;
      wave_lds_fence();
      float4 part[KB][NV];  // this chunk's share (two-level summation)
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j) part[q][j] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int cnt = min(L, end - c0);
      for (int t0 = 0; t0 < cnt; t0 += U) {
        int vv[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
          vv[t] = l_idx[t0 + t];
          if (L == 64) vv[t] = __builtin_amdgcn_readfirstlane(vv[t]);
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          if (!slot_ok[j]) continue;
          float4 rowv[U];
#pragma unroll
          for (int t = 0; t < U; ++t) rowv[t] = ld4(gout + (int64_t)vv[t] * F + 4 * (li + j * L));
#pragma unroll
          for (int t = 0; t < U; ++t)
#pragma unroll
            for (int q = 0; q < KB; ++q) fma4(part[q][j], l_w[q * L + t0 + t], rowv[t]);
        }
      }
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j) add4(acc[q][j], part[q][j]);
      wave_lds_fence();
    }
    if (rr.coop) {
      float vv[NC];
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j) pack4(vv + 4 * (q * NV + j), acc[q][j]);
      coop_sum<L, NC, GPB>(coop_buf, vv, grp, li);
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j) acc[q][j] = unpack4(vv + 4 * (q * NV + j));
    }
    if (!rr.coop || grp == 0)
#pragma unroll
    for (int q = 0; q < KB; ++q)
      if (k0 + q < K)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) st4(dhk + (int64_t)u * KF + (k0 + q) * F + 4 * (li + j * L), acc[q][j]);
  }
}

// ---- a10, edge-balanced mapping of both halves of the backward pass (Sec. 5) --------------
// As k_gmm_fwd_eb: a group owns kGmmEbEdges consecutive positions of an edge array and walks the
// row pieces inside its run.  At most kGmmKB kernels.
//
// Source side (edge array of the CSC transpose): dhk[u,j,:] = (1/K) sum over out-edges
// w_j(e) gout[v,:]; an edge gathers gout[v] once for all kernels.  Pieces of rows that span
// several runs are added atomically onto a dhk zeroed before.
template <int L, int NV>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_bwd_src_eb(
    int32_t n, int32_t nnz, const int32_t* __restrict__ indptr_t, const int32_t* __restrict__ indices_t,
    const float* __restrict__ c, const float* __restrict__ mu, const float* __restrict__ inv_sigma,
    const float* __restrict__ gout, GmmParams pm, float* __restrict__ dhk) {
  constexpr int GPB = kGmmBlock / L;
  constexpr int KB = kGmmKB, U = 4, RUN = kGmmEbEdges;
  constexpr int GS = (1 + KB) * (RUN + U);  // idx | w[KB], each with U entries of padding
  __shared__ __align__(16) float lds[GPB * GS];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t run = (int64_t)blockIdx.x * GPB + grp;
  if (run * RUN >= nnz) return;
  const int32_t e0 = (int32_t)(run * RUN);
  const int32_t e1 = min(e0 + RUN, nnz);
  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_w = lds + grp * GS + (RUN + U);
  const int K = pm.K, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;

  for (int i = li; i < RUN + U; i += L) {
    l_idx[i] = e0 + i < e1 ? indices_t[e0 + i] : 0;  // padding gathers row 0 with weight 0
#pragma unroll
    for (int q = 0; q < KB; ++q) l_w[q * (RUN + U) + i] = 0.f;
  }
  float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
  for (int q = 0; q < KB; ++q) {
    const bool ok = q < K;
    mu0[q] = ok ? mu[2 * q] : 0.f;
    mu1[q] = ok ? mu[2 * q + 1] : 0.f;
    is0[q] = ok ? inv_sigma[2 * q] : 0.f;
    is1[q] = ok ? inv_sigma[2 * q + 1] : 0.f;
  }
  int32_t lo = 0, hi = n;  // row of the first edge: indptr_t[lo] <= e0 < indptr_t[hi] throughout
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (indptr_t[mid] <= e0) lo = mid; else hi = mid;
  }
  int32_t u = lo, row_beg = indptr_t[u], row_end = indptr_t[u + 1];
  wave_lds_fence();

  bool slot_ok[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) slot_ok[j] = 4 * (li + j * L) < F;

  int32_t e = e0;
  while (e < e1) {
    const int32_t seg_end = min(row_end, e1);
    const float cu = c[u];
    for (int32_t t = e + li; t < seg_end; t += L) {
      const float cv = c[l_idx[t - e0]];
#pragma unroll
      for (int q = 0; q < KB; ++q)
        if (q < K) l_w[q * (RUN + U) + (t - e0)] = gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]) * inv_k;
    }
    wave_lds_fence();
    float4 acc[KB][NV];
#pragma unroll
    for (int q = 0; q < KB; ++q)
#pragma unroll
      for (int j = 0; j < NV; ++j) acc[q][j] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t t0 = e; t0 < seg_end; t0 += U) {
      int vv[U];
      float ok[U];
#pragma unroll
      for (int t = 0; t < U; ++t) {
        vv[t] = l_idx[t0 - e0 + t];
        if (L == 64) vv[t] = __builtin_amdgcn_readfirstlane(vv[t]);
        ok[t] = t0 + t < seg_end ? 1.f : 0.f;  // entries past the piece belong to the next row
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        if (!slot_ok[j]) continue;
        float4 rowv[U];
#pragma unroll
        for (int t = 0; t < U; ++t) rowv[t] = ld4(gout + (int64_t)vv[t] * F + 4 * (li + j * L));
#pragma unroll
        for (int t = 0; t < U; ++t)
#pragma unroll
          for (int q = 0; q < KB; ++q)
            if (q < K) fma4(acc[q][j], ok[t] * l_w[q * (RUN + U) + (t0 - e0 + t)], rowv[t]);
      }
    }
    const bool whole = row_beg >= e0 && row_end <= e1;
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      if (q >= K) continue;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        if (!slot_ok[j]) continue;
        float* o = dhk + (int64_t)u * KF + q * F + 4 * (li + j * L);
        if (whole) {
          st4(o, acc[q][j]);
        } else {
          unsafeAtomicAdd(o, acc[q][j].x);
          unsafeAtomicAdd(o + 1, acc[q][j].y);
          unsafeAtomicAdd(o + 2, acc[q][j].z);
          unsafeAtomicAdd(o + 3, acc[q][j].w);
        }
      }
    }
    e = seg_end;
    if (e < e1) {  // the next row that has edges starts at e
      do {
        ++u;
        row_beg = row_end;
        row_end = indptr_t[u + 1];
      } while (row_end == row_beg);
    }
  }
}

// Destination side (CSR edge array): the sums A_j, R_j, S_j of a row piece are dotted with gout[v]
// right away (everything is linear in the per-edge terms, so a row's pieces need not meet) and
// the piece's share of (gmu_j0, gmu_j1, gis_j0, gis_j1) is added to the group's totals, pieces in
// edge order; groups, then workgroups are summed in a fixed order as in the vertex-balanced
// kernel: no atomics, bit-reproducible.  partial[block][j][4] as k_gmm_bwd_dst.
template <int L, int NV>
__global__ __launch_bounds__(kGmmBlock) void k_gmm_bwd_dst_eb(
    int32_t n, int32_t nnz, const int32_t* __restrict__ indptr, const int32_t* __restrict__ indices,
    const float* __restrict__ hk, const float* __restrict__ c, const float* __restrict__ mu,
    const float* __restrict__ inv_sigma, const float* __restrict__ gout, GmmParams pm,
    float* __restrict__ partial) {
  constexpr int GPB = kGmmBlock / L;
  constexpr int KB = kGmmKB, U = kGmmU, RUN = kGmmEbEdges;
  constexpr int GS = (1 + 3 * KB) * (RUN + U);  // idx | w[KB] | w d0 [KB] | w d0^2 [KB], each padded by U
  __shared__ __align__(16) float lds[GPB * GS];
  __shared__ float blk[GPB][kMaxK][4];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t run = (int64_t)blockIdx.x * GPB + grp;
  const int K = pm.K, F = pm.F, KF = K * F;
  const float inv_k = 1.f / (float)K;
  for (int i = li; i < kMaxK * 4; i += L) blk[grp][i >> 2][i & 3] = 0.f;
  if (run * RUN < nnz) {
    const int32_t e0 = (int32_t)(run * RUN);
    const int32_t e1 = min(e0 + RUN, nnz);
    int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
    float* l_w = lds + grp * GS + (RUN + U);
    float* l_wr = l_w + KB * (RUN + U);
    float* l_ws = l_wr + KB * (RUN + U);
    for (int i = li; i < RUN + U; i += L) {
      l_idx[i] = e0 + i < e1 ? indices[e0 + i] : 0;
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        l_w[q * (RUN + U) + i] = 0.f;
        l_wr[q * (RUN + U) + i] = 0.f;
        l_ws[q * (RUN + U) + i] = 0.f;
      }
    }
    float mu0[KB], mu1[KB], is0[KB], is1[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const bool ok = q < K;
      mu0[q] = ok ? mu[2 * q] : 0.f;
      mu1[q] = ok ? mu[2 * q + 1] : 0.f;
      is0[q] = ok ? inv_sigma[2 * q] : 0.f;
      is1[q] = ok ? inv_sigma[2 * q + 1] : 0.f;
    }
    int32_t lo = 0, hi = n;
    while (hi - lo > 1) {
      const int32_t mid = (lo + hi) >> 1;
      if (indptr[mid] <= e0) lo = mid; else hi = mid;
    }
    int32_t v = lo, row_end = indptr[v + 1];
    wave_lds_fence();
    bool slot_ok[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) slot_ok[j] = 4 * (li + j * L) < F;
    float tot[KB][4];  // the group's totals (all lanes carry them; lane 0 stores)
#pragma unroll
    for (int q = 0; q < KB; ++q) tot[q][0] = tot[q][1] = tot[q][2] = tot[q][3] = 0.f;

    int32_t e = e0;
    while (e < e1) {
      const int32_t seg_end = min(row_end, e1);
      const float cv = c[v];
      float4 g4[NV];
#pragma unroll
      for (int j = 0; j < NV; ++j)
        g4[j] = slot_ok[j] ? ld4(gout + (int64_t)v * F + 4 * (li + j * L)) : make_float4(0.f, 0.f, 0.f, 0.f);
      for (int32_t t = e + li; t < seg_end; t += L) {
        const float cu = c[l_idx[t - e0]];
#pragma unroll
        for (int q = 0; q < KB; ++q)
          if (q < K) {
            const float w = gauss_w(cu, cv, mu0[q], mu1[q], is0[q], is1[q]);
            const float d0 = cu - mu0[q];
            l_w[q * (RUN + U) + (t - e0)] = w;
            l_wr[q * (RUN + U) + (t - e0)] = w * d0;
            l_ws[q * (RUN + U) + (t - e0)] = w * d0 * d0;
          }
      }
      wave_lds_fence();
      float4 aA[KB][NV], aR[KB][NV], aS[KB][NV];
#pragma unroll
      for (int q = 0; q < KB; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          aA[q][j] = make_float4(0.f, 0.f, 0.f, 0.f);
          aR[q][j] = aA[q][j];
          aS[q][j] = aA[q][j];
        }
      for (int32_t t0 = e; t0 < seg_end; t0 += U) {
        int uu[U];
        float ok[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
          uu[t] = l_idx[t0 - e0 + t];
          if (L == 64) uu[t] = __builtin_amdgcn_readfirstlane(uu[t]);
          ok[t] = t0 + t < seg_end ? 1.f : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          if (!slot_ok[j]) continue;
          float4 rowv[U][KB];
#pragma unroll
          for (int t = 0; t < U; ++t)
#pragma unroll
            for (int q = 0; q < KB; ++q)
              if (q < K) rowv[t][q] = ld4(hk + (int64_t)uu[t] * KF + q * F + 4 * (li + j * L));
#pragma unroll
          for (int t = 0; t < U; ++t)
#pragma unroll
            for (int q = 0; q < KB; ++q)
              if (q < K) {
                const int at = q * (RUN + U) + (t0 - e0 + t);
                fma4(aA[q][j], ok[t] * l_w[at], rowv[t][q]);
                fma4(aR[q][j], ok[t] * l_wr[at], rowv[t][q]);
                fma4(aS[q][j], ok[t] * l_ws[at], rowv[t][q]);
              }
        }
      }
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        if (q >= K) continue;
        float tA = 0.f, tR = 0.f, tS = 0.f;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          tA += dot4(g4[j], aA[q][j]);
          tR += dot4(g4[j], aR[q][j]);
          tS += dot4(g4[j], aS[q][j]);
        }
        tA = group_sum_from<L>(tA, 1);
        tR = group_sum_from<L>(tR, 1);
        tS = group_sum_from<L>(tS, 1);
        const float d1 = cv - mu1[q];
        tot[q][0] += tR * is0[q] * is0[q] * inv_k;
        tot[q][1] += tA * d1 * is1[q] * is1[q] * inv_k;
        tot[q][2] += -tS * is0[q] * inv_k;
        tot[q][3] += -tA * d1 * d1 * is1[q] * inv_k;
      }
      e = seg_end;
      if (e < e1) {
        do {
          ++v;
          row_end = indptr[v + 1];
        } while (row_end == e);
      }
    }
    if (li == 0) {
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        blk[grp][q][0] = tot[q][0]; blk[grp][q][1] = tot[q][1];
        blk[grp][q][2] = tot[q][2]; blk[grp][q][3] = tot[q][3];
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < kMaxK * 4) {
    const int k = threadIdx.x >> 2, q = threadIdx.x & 3;
    float s = 0.f;
    for (int gi = 0; gi < GPB; ++gi) s += blk[gi][k][q];  // fixed order
    partial[((int64_t)blockIdx.x * kMaxK + k) * 4 + q] = s;
  }
}

template <int L, int NV>
struct GmmFwdLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* hk, const float* c, const float* mu,
                          const float* is, GmmParams pm, float* out, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kGmmBlock / kWave);
    ProfScope p("gmm_fwd_fused", st);
    const RowSplit sp = split_rows(g, 0, L, GPB);
    // hub rows (one workgroup each) and the rest in one launch
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_gmm_fwd<L, NV><<<grid, kGmmBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, c, mu, is, pm,
                                                   out);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct GmmFwdEbLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* hk, const float* c, const float* mu,
                          const float* is, GmmParams pm, float* out, hipStream_t st) {
    constexpr int GPB = kGmmBlock / L;
    ProfScope p("gmm_fwd_fused", st);
    const int64_t quads = (int64_t)g->n * (pm.F / 4);
    k_gmm_zero_f4<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, out);
    GNN_LAUNCH_CHECK();
    const int64_t runs = cdiv(g->nnz, kGmmEbEdges);
    if (runs != 0) {
      k_gmm_fwd_eb<L, NV><<<(unsigned)cdiv(runs, GPB), kGmmBlock, 0, st>>>(
          g->n, (int32_t)g->nnz, g->indptr, g->indices, hk, c, mu, is, pm, out);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct GmmFwdXLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* x, const float* c, const float* mu,
                          const float* is, int K, int fin, float* agg, hipStream_t st) {
    constexpr int GPB = kGmmBlock / L;
    ProfScope p("gmm_fwd_fused", st);
    const RowSplit sp = split_rows(g, 0, L, GPB);
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_gmm_fwd_x<L><<<grid, kGmmBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, x, c, mu, is, K, fin, agg);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct GmmBwdDstXLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* x, const float* c, const float* mu,
                          const float* is, const float* G, int K, int fin, float* partial, float* gmu,
                          float* gis, hipStream_t st) {
    constexpr int GPB = kGmmBlock / L;
    ProfScope p("gmm_bwd_dst", st);
    const RowSplit sp = split_rows(g, 0, L, GPB);
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_gmm_bwd_dst_x<L><<<grid, kGmmBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, x, c, mu, is, G, K,
                                                    fin, partial);
      GNN_LAUNCH_CHECK();
    }
    float* totals = partial + (int64_t)grid * kMaxK * 4;
    GNN_TRY(sum_partials_two_level(kMaxK * 4, (int)grid, partial, totals + kMaxK * 4, totals, st));
    k_gmm_param_split<<<1, 64, 0, st>>>(K, totals, gmu, gis);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};

// number of workgroups (= partial slots) the destination-side kernel uses
template <int L>
static int64_t gmm_dst_blocks(const gnn_graph_t* g) {
  constexpr int GPB = (kWave / L) * (kGmmBlock / kWave);
  const RowSplit sp = split_rows(g, 0, L, GPB);
  return (int64_t)sp.hub_grid + sp.rest_grid;
}

template <int L, int NV>
struct GmmBwdDstLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* hk, const float* c, const float* mu,
                          const float* is, const float* gout, GmmParams pm, float* partial,
                          float* gmu, float* gis, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kGmmBlock / kWave);
    ProfScope p("gmm_bwd_dst", st);
    const RowSplit sp = split_rows(g, 0, L, GPB);
    // hub rows (one workgroup each) and the rest in one launch; one partial slot per workgroup
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_gmm_bwd_dst<L, NV><<<grid, kGmmBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, hk, c, mu, is,
                                                       gout, pm, partial);
      GNN_LAUNCH_CHECK();
    }
    // after the block slots: one slot for the totals, then the second-level scratch
    float* totals = partial + (int64_t)grid * kMaxK * 4;
    GNN_TRY(sum_partials_two_level(kMaxK * 4, (int)grid, partial, totals + kMaxK * 4, totals, st));
    k_gmm_param_split<<<1, 64, 0, st>>>(pm.K, totals, gmu, gis);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};

template <int L, int NV>
struct GmmBwdSrcLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* c, const float* mu, const float* is,
                          const float* gout, GmmParams pm, float* dhk, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kGmmBlock / kWave);
    ProfScope p("gmm_bwd_src", st);
    const RowSplit sp = split_rows(g, 1, L, GPB);
    // hub rows (one workgroup each) and the rest in one launch
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_gmm_bwd_src<L, NV><<<grid, kGmmBlock, 0, st>>>(rl, g->order[1], g->indptr_t, g->indices_t, c, mu, is,
                                                       gout, pm, dhk);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct GmmBwdDstEbLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* hk, const float* c, const float* mu,
                          const float* is, const float* gout, GmmParams pm, float* partial,
                          float* gmu, float* gis, hipStream_t st) {
    constexpr int GPB = kGmmBlock / L;
    ProfScope p("gmm_bwd_dst", st);
    const unsigned grid = (unsigned)cdiv(cdiv(g->nnz, kGmmEbEdges), GPB);
    if (grid != 0) {
      k_gmm_bwd_dst_eb<L, NV><<<grid, kGmmBlock, 0, st>>>(g->n, (int32_t)g->nnz, g->indptr, g->indices, hk, c, mu,
                                                          is, gout, pm, partial);
      GNN_LAUNCH_CHECK();
    }
    float* totals = partial + (int64_t)grid * kMaxK * 4;
    GNN_TRY(sum_partials_two_level(kMaxK * 4, (int)grid, partial, totals + kMaxK * 4, totals, st));
    k_gmm_param_split<<<1, 64, 0, st>>>(pm.K, totals, gmu, gis);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};

template <int L, int NV>
struct GmmBwdSrcEbLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* c, const float* mu, const float* is,
                          const float* gout, GmmParams pm, float* dhk, hipStream_t st) {
    constexpr int GPB = kGmmBlock / L;
    ProfScope p("gmm_bwd_src", st);
    const int64_t quads = (int64_t)g->n * (pm.K * pm.F / 4);
    k_gmm_zero_f4<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, dhk);
    GNN_LAUNCH_CHECK();
    const int64_t runs = cdiv(g->nnz, kGmmEbEdges);
    if (runs != 0) {
      k_gmm_bwd_src_eb<L, NV><<<(unsigned)cdiv(runs, GPB), kGmmBlock, 0, st>>>(
          g->n, (int32_t)g->nnz, g->indptr_t, g->indices_t, c, mu, is, gout, pm, dhk);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

// fout <= 256 keeps NV == 1
template <template <int, int> class Launcher, typename... Args>
static gnn_status_t gmm_dispatch(GroupShape gs, Args... args) {
  switch (gs.L) {
    case 4: return Launcher<4, 1>::run(args...);
    case 8: return Launcher<8, 1>::run(args...);
    case 16: return Launcher<16, 1>::run(args...);
    case 32: return Launcher<32, 1>::run(args...);
    case 64: return Launcher<64, 1>::run(args...);
  }
  set_error("unsupported row-group shape L=%d", gs.L);
  return GNN_ERR_UNSUPPORTED;
}

// mapping of the forward aggregation: 0 vertex-balanced, 1 edge-balanced (at most kGmmKB kernels),
// 2 what gnn_gmm_tune found faster on this graph (vertex-balanced on a graph never tuned)
static bool gmm_use_edge_balanced(const gnn_graph_t* g, int K) {
  if (K > kGmmKB) return false;
  const int64_t mode = config_get(kCfgGmmMapping);
  if (mode == 1) return true;
  return mode == 2 && g->gmm_edge_balanced == 1;
}

// the same for the two halves of the backward pass (side 0: destination, 1: source); gnn_gmm_tune_bwd
// records what it measured
static bool gmm_bwd_use_edge_balanced(const gnn_graph_t* g, int K, int side) {
  if (K > kGmmKB) return false;
  const int64_t mode = config_get(kCfgGmmMapping);
  if (mode == 1) return true;
  return mode == 2 && g->gmm_bwd_edge_balanced[side] == 1;
}

static gnn_status_t gmm_aggregate(const gnn_graph_t* g, bool edge_balanced, const float* hk, const float* c,
                                  const float* mu, const float* is, GmmParams pm, float* out, hipStream_t st) {
  if (edge_balanced) return gmm_dispatch<GmmFwdEbLauncher>(pick_group(pm.F), g, hk, c, mu, is, pm, out, st);
  return gmm_dispatch<GmmFwdLauncher>(pick_group(pm.F), g, hk, c, mu, is, pm, out, st);
}

// aggregate first when an input row is narrower than the K projected rows (and fits one float4 per lane)
static bool gmm_aggregate_first(int fin, int fout, int K) {
  return fin % 4 == 0 && fin <= 256 && fin < K * fout;
}

struct GmmWs {
  size_t total, dhk, partial, gemm, agg, wt;
  int split_k;
  int64_t nblk;
};

static int64_t gmm_dst_blocks_for(const gnn_graph_t* g, int width) {
  switch (pick_group(width).L) {
    case 4: return gmm_dst_blocks<4>(g);
    case 8: return gmm_dst_blocks<8>(g);
    case 16: return gmm_dst_blocks<16>(g);
    case 32: return gmm_dst_blocks<32>(g);
    default: return gmm_dst_blocks<64>(g);
  }
}

static GmmWs gmm_ws_layout(const gnn_graph_t* g, int fin, int fout, int K) {
  const int64_t n = g->n;
  GmmWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += ws_granule(bytes); return o; };
  const bool xg = gmm_aggregate_first(fin, fout, K);
  w.nblk = gmm_dst_blocks_for(g, fout);
  if (xg) {
    const int64_t nb = gmm_dst_blocks_for(g, fin);
    if (nb > w.nblk) w.nblk = nb;
  }
  if (K <= kGmmKB) {  // the edge-balanced destination side: one slot per workgroup of runs
    const int64_t nb = cdiv(cdiv(g->nnz, kGmmEbEdges), kGmmBlock / pick_group(fout).L);
    if (nb > w.nblk) w.nblk = nb;
  }
  w.dhk = take(sizeof(float) * (size_t)n * K * fout);
  // block slots + one slot for the totals + second-level scratch
  w.partial = take(sizeof(float) * (size_t)(w.nblk + 1 + sum_partials_scratch_rows((int)w.nblk)) * kMaxK * 4);
  w.split_k = gemm_pick_split_k(fin, K * fout, n);
  w.gemm = take(w.split_k > 1 ? sizeof(float) * (size_t)w.split_k * fin * K * fout : 0);
  w.agg = take(xg ? sizeof(float) * (size_t)n * K * fin : 0);  // forward: aggregated inputs; backward: gout W'^T
  w.wt = take(xg ? sizeof(float) * (size_t)K * fin * fout : 0);
  w.total = off;
  return w;
}

static gnn_status_t gmm_check(const gnn_graph_t* g, int fin, int fout, int K, const char* who) {
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "%s: graph is null", who);
  GNN_REQUIRE(fin > 0 && fout > 0 && K > 0, GNN_ERR_INVALID_ARG, "%s: sizes must be positive", who);
  GNN_REQUIRE(fout % 4 == 0 && fout <= 256, GNN_ERR_UNSUPPORTED,
              "%s: fout = %d must be a multiple of 4, at most 256", who, fout);
  GNN_REQUIRE(K <= kMaxK, GNN_ERR_UNSUPPORTED, "%s: k = %d exceeds %d", who, K, kMaxK);
  return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" size_t gnn_gmm_workspace_bytes(const gnn_graph_t* g, int fin, int fout, int k) {
  if (!g || fin <= 0 || fout <= 0 || k <= 0) return 0;
  return gmm_ws_layout(g, fin, fout, k).total;
}

extern "C" gnn_status_t gnn_gmm_fwd(const gnn_graph_t* g, int fin, int fout, int k, const float* x,
                                    const float* w_fc, const float* c, const float* mu,
                                    const float* inv_sigma, float* hk, float* out, void* ws,
                                    size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(gmm_check(g, fin, fout, k, "gnn_gmm_fwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w_fc && c && mu && inv_sigma && hk && out, GNN_ERR_INVALID_ARG,
              "gnn_gmm_fwd: null pointer");
  GNN_REQUIRE(aligned16(hk) && aligned16(out), GNN_ERR_INVALID_ARG,
              "gnn_gmm_fwd: hk, out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  GmmParams pm{k, fout};
  const bool eb = gmm_use_edge_balanced(g, k);
  if (!eb && gmm_aggregate_first(fin, fout, k) && ws != nullptr && aligned16(ws)) {
    const GmmWs W = gmm_ws_layout(g, fin, fout, k);
    if (ws_bytes >= W.total) {
      // aggregate the input rows per kernel, then project: out = agg W'
      char* base = static_cast<char*>(ws);
      float* agg = reinterpret_cast<float*>(base + W.agg);
      float* wt = reinterpret_cast<float*>(base + W.wt);
      {
        ProfScope p("gmm_weight_layout", st);
        const int64_t cnt = (int64_t)fin * k * fout;
        k_gmm_wt<<<(unsigned)cdiv(cnt, 256), 256, 0, st>>>(fin, k, fout, w_fc, wt);
        GNN_LAUNCH_CHECK();
      }
      GNN_TRY((gmm_dispatch<GmmFwdXLauncher>(pick_group(fin), g, x, c, mu, inv_sigma, k, fin, agg, st)));
      return gemm_f32(g->n, fout, (int64_t)k * fin, agg, (int64_t)k * fin, false, wt, fout, false, out, fout, 1,
                      nullptr, st);
    }
  }
  // project first: hk = x w_fc, then the fused weights + aggregate over the projected rows
  GNN_TRY(gemm_f32(g->n, k * fout, fin, x, fin, false, w_fc, k * fout, false, hk, k * fout, 1, nullptr, st));
  return gmm_aggregate(g, eb, hk, c, mu, inv_sigma, pm, out, st);
}

extern "C" gnn_status_t gnn_gmm_tune(gnn_graph_t* g, int fout, int k, const float* hk, const float* c,
                                     const float* mu, const float* inv_sigma, float* out, void* stream,
                                     float* ms_out) {
  clear_error();
  GNN_TRY(gmm_check(g, 1, fout, k, "gnn_gmm_tune"));
  float ms[2] = {0.f, 0.f};
  if (g->n != 0 && g->nnz != 0 && k <= kGmmKB) {
    GNN_REQUIRE(hk && c && mu && inv_sigma && out, GNN_ERR_INVALID_ARG, "gnn_gmm_tune: null pointer");
    GNN_REQUIRE(aligned16(hk) && aligned16(out), GNN_ERR_INVALID_ARG,
                "gnn_gmm_tune: hk, out must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t a = nullptr, b = nullptr;
    GNN_HIP(hipEventCreate(&a));
    if (hipEventCreate(&b) != hipSuccess) {
      (void)hipEventDestroy(a);
      set_error("gnn_gmm_tune: hipEventCreate failed");
      return GNN_ERR_HIP;
    }
    constexpr int kReps = 3;
    GmmParams pm{k, fout};
    gnn_status_t status = GNN_OK;
    for (int eb = 0; eb < 2 && status == GNN_OK; ++eb) {
      status = gmm_aggregate(g, eb != 0, hk, c, mu, inv_sigma, pm, out, st);  // warm-up
      if (status == GNN_OK && hipEventRecord(a, st) != hipSuccess) status = GNN_ERR_HIP;
      for (int r = 0; r < kReps && status == GNN_OK; ++r)
        status = gmm_aggregate(g, eb != 0, hk, c, mu, inv_sigma, pm, out, st);
      if (status == GNN_OK && (hipEventRecord(b, st) != hipSuccess || hipEventSynchronize(b) != hipSuccess))
        status = GNN_ERR_HIP;
      float t = 0.f;
      if (status == GNN_OK && hipEventElapsedTime(&t, a, b) != hipSuccess) status = GNN_ERR_HIP;
      ms[eb] = t / kReps;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (status != GNN_OK) {
      if (status == GNN_ERR_HIP && gnn_last_error()[0] == 0) set_error("gnn_gmm_tune: a HIP event call failed");
      return status;
    }
    g->gmm_edge_balanced = ms[1] < ms[0] ? 1 : 0;
  }
  if (ms_out) {
    ms_out[0] = ms[0];
    ms_out[1] = ms[1];
  }
  return GNN_OK;
}

// times `reps` runs of fn after one warm-up; status and milliseconds per run
template <typename Fn>
static gnn_status_t time_passes(hipStream_t st, int reps, Fn fn, float* ms) {
  hipEvent_t a = nullptr, b = nullptr;
  GNN_HIP(hipEventCreate(&a));
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    set_error("hipEventCreate failed");
    return GNN_ERR_HIP;
  }
  gnn_status_t status = fn();  // warm-up
  if (status == GNN_OK && hipEventRecord(a, st) != hipSuccess) status = GNN_ERR_HIP;
  for (int r = 0; r < reps && status == GNN_OK; ++r) status = fn();
  if (status == GNN_OK && (hipEventRecord(b, st) != hipSuccess || hipEventSynchronize(b) != hipSuccess))
    status = GNN_ERR_HIP;
  float t = 0.f;
  if (status == GNN_OK && hipEventElapsedTime(&t, a, b) != hipSuccess) status = GNN_ERR_HIP;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (status == GNN_ERR_HIP && gnn_last_error()[0] == 0) set_error("a HIP event call failed");
  *ms = t / (float)reps;
  return status;
}

extern "C" gnn_status_t gnn_gmm_tune_bwd(gnn_graph_t* g, int fin, int fout, int k, const float* hk,
                                         const float* c, const float* mu, const float* inv_sigma,
                                         const float* gout, void* ws, size_t ws_bytes, void* stream,
                                         float* ms_out) {
  clear_error();
  GNN_TRY(gmm_check(g, fin, fout, k, "gnn_gmm_tune_bwd"));
  float ms[4] = {0.f, 0.f, 0.f, 0.f};
  if (g->n != 0 && g->nnz != 0 && k <= kGmmKB) {
    GNN_REQUIRE(hk && c && mu && inv_sigma && gout, GNN_ERR_INVALID_ARG, "gnn_gmm_tune_bwd: null pointer");
    GNN_REQUIRE(aligned16(hk) && aligned16(gout), GNN_ERR_INVALID_ARG,
                "gnn_gmm_tune_bwd: hk, gout must be 16-byte aligned");
    const GmmWs L = gmm_ws_layout(g, fin, fout, k);
    GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
                "gnn_gmm_tune_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
    GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_gmm_tune_bwd: workspace must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    float* dhk = reinterpret_cast<float*>(base + L.dhk);
    float* partial = reinterpret_cast<float*>(base + L.partial);
    float* gmu = dhk;  // the destination side's results are not kept: they land in the dhk area (4 k floats)
    float* gis = dhk + 2 * k;
    GmmParams pm{k, fout};
    const GroupShape gs = pick_group(fout);
    constexpr int kReps = 3;
    GNN_TRY(time_passes(st, kReps, [&] { return gmm_dispatch<GmmBwdDstLauncher>(gs, g, hk, c, mu, inv_sigma, gout, pm, partial, gmu, gis, st); }, &ms[0]));
    GNN_TRY(time_passes(st, kReps, [&] { return gmm_dispatch<GmmBwdDstEbLauncher>(gs, g, hk, c, mu, inv_sigma, gout, pm, partial, gmu, gis, st); }, &ms[1]));
    GNN_TRY(time_passes(st, kReps, [&] { return gmm_dispatch<GmmBwdSrcLauncher>(gs, g, c, mu, inv_sigma, gout, pm, dhk, st); }, &ms[2]));
    GNN_TRY(time_passes(st, kReps, [&] { return gmm_dispatch<GmmBwdSrcEbLauncher>(gs, g, c, mu, inv_sigma, gout, pm, dhk, st); }, &ms[3]));
    g->gmm_bwd_edge_balanced[0] = ms[1] < ms[0] ? 1 : 0;
    g->gmm_bwd_edge_balanced[1] = ms[3] < ms[2] ? 1 : 0;
  }
  if (ms_out)
    for (int i = 0; i < 4; ++i) ms_out[i] = ms[i];
  return GNN_OK;
}

extern "C" gnn_status_t gnn_gmm_bwd(const gnn_graph_t* g, int fin, int fout, int k, const float* x,
                                    const float* w_fc, const float* c, const float* mu,
                                    const float* inv_sigma, const float* hk, const float* gout,
                                    float* gx, float* gw_fc, float* gmu, float* ginv_sigma, void* ws,
                                    size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(gmm_check(g, fin, fout, k, "gnn_gmm_bwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w_fc && c && mu && inv_sigma && hk && gout && gw_fc && gmu && ginv_sigma,
              GNN_ERR_INVALID_ARG, "gnn_gmm_bwd: null pointer");
  GNN_REQUIRE(aligned16(hk) && aligned16(gout), GNN_ERR_INVALID_ARG,
              "gnn_gmm_bwd: hk, gout must be 16-byte aligned");
  const GmmWs L = gmm_ws_layout(g, fin, fout, k);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "gnn_gmm_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_gmm_bwd: workspace must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  float* dhk = reinterpret_cast<float*>(base + L.dhk);
  float* partial = reinterpret_cast<float*>(base + L.partial);
  float* part = reinterpret_cast<float*>(base + L.gemm);
  const int64_t n = g->n;
  const int KF = k * fout;
  GmmParams pm{k, fout};
  const GroupShape gs = pick_group(fout);
  // the tuner compares the destination side with the project-first kernel: where the layer would
  // gather the narrower input rows instead, only an explicit gmm_mapping = 1 switches
  const bool eb_dst = gmm_bwd_use_edge_balanced(g, k, 0) &&
                      (config_get(kCfgGmmMapping) == 1 || !gmm_aggregate_first(fin, fout, k));
  const bool eb_src = gmm_bwd_use_edge_balanced(g, k, 1);
  if (eb_dst) {
    const float* hk_use = hk;
    if (gmm_aggregate_first(fin, fout, k)) {
      // the forward call may have aggregated first and left hk unwritten: project again, into the
      // dhk area, which the source side fills only afterwards
      GNN_TRY(gemm_f32(n, KF, fin, x, fin, false, w_fc, KF, false, dhk, KF, 1, nullptr, st));
      hk_use = dhk;
    }
    GNN_TRY(gmm_dispatch<GmmBwdDstEbLauncher>(gs, g, hk_use, c, mu, inv_sigma, gout, pm, partial, gmu, ginv_sigma, st));
  } else if (gmm_aggregate_first(fin, fout, k)) {
    // <gout[v], hk[u,j,:]> = <G_j[v], x[u]>, G = gout W'^T: the destination side gathers x rows
    float* G = reinterpret_cast<float*>(base + L.agg);
    float* wt = reinterpret_cast<float*>(base + L.wt);
    {
      ProfScope p("gmm_weight_layout", st);
      const int64_t cnt = (int64_t)fin * k * fout;
      k_gmm_wt<<<(unsigned)cdiv(cnt, 256), 256, 0, st>>>(fin, k, fout, w_fc, wt);
      GNN_LAUNCH_CHECK();
    }
    GNN_TRY(gemm_f32(n, k * fin, fout, gout, fout, false, wt, fout, true, G, (int64_t)k * fin, 1, nullptr, st));
    GNN_TRY((gmm_dispatch<GmmBwdDstXLauncher>(pick_group(fin), g, x, c, mu, inv_sigma, (const float*)G, k, fin,
                                              partial, gmu, ginv_sigma, st)));
  } else {
    GNN_TRY(gmm_dispatch<GmmBwdDstLauncher>(gs, g, hk, c, mu, inv_sigma, gout, pm, partial, gmu, ginv_sigma, st));
  }
  if (eb_src) GNN_TRY(gmm_dispatch<GmmBwdSrcEbLauncher>(gs, g, c, mu, inv_sigma, gout, pm, dhk, st));
  else GNN_TRY(gmm_dispatch<GmmBwdSrcLauncher>(gs, g, c, mu, inv_sigma, gout, pm, dhk, st));
  GNN_TRY(gemm_f32(fin, KF, n, x, fin, true, dhk, KF, false, gw_fc, KF, L.split_k, part, st));
  if (gx) GNN_TRY(gemm_f32(n, fin, KF, dhk, KF, false, w_fc, KF, true, gx, fin, 1, nullptr, st));
  return GNN_OK;
}
