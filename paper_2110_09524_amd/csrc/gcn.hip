// GCN layer with separable static edge weights e_uv = c_src[u] c_dst[v] (App. A.2 "GCN";
// the symmetric normalisation, mean and plain-sum aggregation are of this form).
//
// Reorganization (Sec. 4): multiplying by the edge weight is linear, so both factors move
// from the edges onto the vertices,
//     out[v] = c_dst[v] * sum over in-edges of  (c_src ⊙ (x w))[u],
// and the fused Scatter-ApplyEdge-Gather is an unweighted gather-sum of rows: no per-edge
// scalar is read at all.  Backward is the same sum over the CSC transpose (no atomics):
//     dz[u] = c_src[u] * sum over out-edges of (c_dst ⊙ gout)[v],  gw = x^T dz,  gx = dz w^T.
// Nothing per-edge is stored; the saved state is zs = c_src ⊙ (x w).
//
// Large graphs use the same column-blocked, XCD-sliced traversal as the GAT kernels: 8
// column slices (workgroup id mod 8, one per XCD), blocks of `block_cols` gathered vertices,
// one launch per block, running sums read-add-written between launches.
//
// Two thread mappings of the single-launch sum (Sec. 5, the vertex-balanced and the
// edge-balanced mapping of a fused Gather): k_rowsum gives a group one row, k_rowsum_eb gives
// a group a fixed run of consecutive edges and joins the pieces of a row that spans several
// runs with atomic adds.  gnn_gcn_tune times both on a graph and the layer calls then use the
// faster one per side (the profile-driven choice of the mapping).
#include <atomic>
#include <cstdio>

#include "common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kGcnBlock = 256;
constexpr int kGcnSlices = 8;
constexpr int kGcnRows = 4;  // consecutive rows of the degree order per group (software-pipelined)

// out[v,:] = c[v] * in[v,:]   (in == out allowed)
__global__ void k_scale_rows(int64_t quads, int q_per_row, const float* __restrict__ c,
                             const float* in, float* out) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= quads) return;
  const float s = c[i / q_per_row];
  const float4 v = ld4(in + 4 * i);
  st4(out + 4 * i, make_float4(s * v.x, s * v.y, s * v.z, s * v.w));
}

// ---- single launch: out[row,:] = scale[row] * sum over the row's gathered vertices of feat ----
// W: every edge carries a static weight (wgt, in the order of cols); scale may then be null
template <int L, int NV, bool W = false>
__global__ __launch_bounds__(kGcnBlock) void k_rowsum(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ ptr,
    const int32_t* __restrict__ cols, const float* __restrict__ feat, int F,
    const float* __restrict__ scale, float* __restrict__ out, const float* __restrict__ wgt = nullptr) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kGcnBlock / kWave);
  constexpr int NC = 4 * NV;
  constexpr int U = 4;
  __shared__ int lds[GPB * L];
  __shared__ float lds_w[W ? GPB * L : 1];
  __shared__ float coop_buf[GPB * L * NC];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  int* l_idx = lds + grp * L;
  float* l_w = lds_w + (W ? grp * L : 0);
  const int32_t v = order[r];
  const int32_t beg = ptr[v], end = ptr[v + 1];

  bool slot_ok[NV];
  float4 acc[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    slot_ok[j] = 4 * (li + j * L) < F;
    acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  for (int32_t c0 = beg + gi * L; c0 < end; c0 += ngrp * L) {
    l_idx[li] = c0 + li < end ? cols[c0 + li] : 0;
    if (W) l_w[li] = c0 + li < end ? wgt[c0 + li] : 0.f;
    wave_lds_fence();
    float4 part[NV];  // this chunk's share (two-level summation)
#pragma unroll
    for (int j = 0; j < NV; ++j) part[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int cnt = min(L, end - c0);
    for (int t0 = 0; t0 < cnt; t0 += U) {
      int uu[U];
      float ww[U];
#pragma unroll
      for (int t = 0; t < U; ++t) {
        uu[t] = l_idx[t0 + t];
        if (L == 64) uu[t] = __builtin_amdgcn_readfirstlane(uu[t]);
        ww[t] = W ? l_w[t0 + t] : (t0 + t < cnt ? 1.f : 0.f);  // padding adds 0 * row 0
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        if (!slot_ok[j]) continue;
        float4 rowv[U];
#pragma unroll
        for (int t = 0; t < U; ++t) rowv[t] = ld4(feat + (int64_t)uu[t] * F + 4 * (li + j * L));
#pragma unroll
        for (int t = 0; t < U; ++t) fma4(part[j], ww[t], rowv[t]);
      }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) add4(acc[j], part[j]);
    wave_lds_fence();
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
  const float s = scale ? scale[v] : 1.f;
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j])
      st4(out + (int64_t)v * F + 4 * (li + j * L), make_float4(s * acc[j].x, s * acc[j].y, s * acc[j].z, s * acc[j].w));
}

// ---- edge-balanced mapping of the same sum ------------------------------------------------
// A group owns kEbEdges consecutive positions of the edge array, whatever rows they belong to
// (every group does the same amount of gathering, however skewed the degrees are).  It finds
// the row of its first edge by bisection of ptr, then walks row by row.  A row that lies
// entirely inside the run is stored; a row that continues into other runs is added atomically
// onto an output that a fill kernel zeroed before (rows without edges stay zero).  Two pieces
// add up the same in either order; rows of more than two pieces (degree > kEbEdges) depend on
// the arrival order in the last bits.
constexpr int kEbEdges = 64;

__global__ void k_zero_f4(int64_t quads, float* __restrict__ p) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < quads) st4(p + 4 * i, make_float4(0.f, 0.f, 0.f, 0.f));
}

// W: every edge carries a static weight (wgt, in the order of cols); scale may then be null
template <int L, int NV, bool W = false>
__global__ __launch_bounds__(kGcnBlock) void k_rowsum_eb(
    int32_t n, int32_t nnz, const int32_t* __restrict__ ptr, const int32_t* __restrict__ cols,
    const float* __restrict__ feat, int F, const float* __restrict__ scale, float* __restrict__ out,
    const float* __restrict__ wgt = nullptr) {
  constexpr int GPB = kGcnBlock / L;
  constexpr int U = 4;
  constexpr int GS = (W ? 2 : 1) * (kEbEdges + U);  // the run's gathered vertices (and weights), each with U entries of padding
  __shared__ int lds[GPB * GS];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t run = (int64_t)blockIdx.x * GPB + grp;
  if (run * kEbEdges >= nnz) return;
  const int32_t e0 = (int32_t)(run * kEbEdges);
  const int32_t e1 = min(e0 + kEbEdges, nnz);
  int* l_idx = lds + grp * GS;
  float* l_wt = reinterpret_cast<float*>(l_idx + kEbEdges + U);
  for (int i = li; i < kEbEdges + U; i += L) {
    l_idx[i] = e0 + i < e1 ? cols[e0 + i] : 0;  // padding gathers row 0, weight 0
    if (W) l_wt[i] = e0 + i < e1 ? wgt[e0 + i] : 0.f;
  }

  // row of the first edge: ptr[lo] <= e0 < ptr[hi] throughout (ptr[0] = 0, ptr[n] = nnz)
  int32_t lo = 0, hi = n;
  while (hi - lo > 1) {
    const int32_t mid = (lo + hi) >> 1;
    if (ptr[mid] <= e0) lo = mid; else hi = mid;
  }
  int32_t v = lo, row_beg = ptr[v], row_end = ptr[v + 1];
  wave_lds_fence();

  bool slot_ok[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) slot_ok[j] = 4 * (li + j * L) < F;

  int32_t e = e0;
  while (e < e1) {
    const int32_t seg_end = min(row_end, e1);
    float4 acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int32_t t0 = e; t0 < seg_end; t0 += U) {
      int uu[U];
#pragma unroll
      for (int t = 0; t < U; ++t) {
        uu[t] = l_idx[t0 - e0 + t];
        if (L == 64) uu[t] = __builtin_amdgcn_readfirstlane(uu[t]);
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        if (!slot_ok[j]) continue;
        float4 rowv[U];
#pragma unroll
        for (int t = 0; t < U; ++t) rowv[t] = ld4(feat + (int64_t)uu[t] * F + 4 * (li + j * L));
#pragma unroll
        for (int t = 0; t < U; ++t)
          fma4(acc[j], t0 + t < seg_end ? (W ? l_wt[t0 - e0 + t] : 1.f) : 0.f, rowv[t]);
      }
    }
    const float s = scale != nullptr ? scale[v] : 1.f;
    const bool whole = row_beg >= e0 && row_end <= e1;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (!slot_ok[j]) continue;
      float* o = out + (int64_t)v * F + 4 * (li + j * L);
      const float4 r = make_float4(s * acc[j].x, s * acc[j].y, s * acc[j].z, s * acc[j].w);
      if (whole) {
        st4(o, r);
      } else {
        unsafeAtomicAdd(o, r.x);
        unsafeAtomicAdd(o + 1, r.y);
        unsafeAtomicAdd(o + 2, r.z);
        unsafeAtomicAdd(o + 3, r.w);
      }
    }
    e = seg_end;
    if (e < e1) {  // the next row that has edges (it starts at e)
      do {
        ++v;
        row_beg = row_end;
        row_end = ptr[v + 1];
      } while (row_end == row_beg);
    }
  }
}

// ---- one column block of the same sum (running sums in acc_buf) -----------------------
// W: every edge carries a static weight, bw in the order of bcol (a second coalesced stream)
template <int SL, bool SKIP, bool W = false>
__global__ __launch_bounds__(kGcnBlock) void k_rowsum_blk(
    int32_t n_rows, const int32_t* __restrict__ order, const int2* __restrict__ bseg_b,
    const int32_t* __restrict__ bcol, const float* __restrict__ feat, int32_t col_begin, int F,
    int first, int ns /* column slices: 8, 4, 2 or 1 */, float* __restrict__ acc_buf,
    int nseg /* adjacent column blocks of this launch (1 .. kMaxMerge): segment j of the row at
                position r of the degree order is bseg_b[j * n_rows + r] */,
    const float* __restrict__ bw = nullptr) {
  constexpr int GPB = kGcnBlock / SL;
  constexpr int R = kGcnRows;
  constexpr int U = SL < 8 ? 4 : 8;
  constexpr int GS = SL + R + 2 * R * kMaxMerge + (W ? SL : 0);  // LDS ints per group: idx | rows | (beg, end) per row and block | weights
  static_assert(GS % 4 == 0, "group scratch must stay 16-byte aligned");
  static_assert(SL >= R, "one lane per pipelined row loads its metadata");
  __shared__ __align__(16) int lds[GPB * GS];
  const int lane = threadIdx.x & 63;
  const int li = lane & (SL - 1);
  const int grp = threadIdx.x / SL;
  const int slice = blockIdx.x % ns;
  const int64_t r0 = ((int64_t)(blockIdx.x / ns) * GPB + grp) * R;
  if (r0 >= n_rows) return;
  int* l_idx = lds + grp * GS;
  int* l_row = l_idx + SL;
  int2* l_seg = reinterpret_cast<int2*>(l_row + R);  // [R][kMaxMerge]
  float* l_w = reinterpret_cast<float*>(l_idx + SL + R + 2 * R * kMaxMerge);
  const int col = slice * 4 * SL + 4 * li;

  if (li < R) {
    const int64_t r = r0 + li;
    int32_t row = -1;
    bool any = false;
    if (r < n_rows) row = order[r];
    for (int j = 0; j < nseg; ++j) {
      int2 seg = make_int2(0, 0);
      if (r < n_rows) seg = bseg_b[(int64_t)j * n_rows + r];
      any = any || seg.x != seg.y;
      l_seg[li * kMaxMerge + j] = seg;
    }
    if (!first && !any) row = -1;  // nothing to add to this row in these blocks
    l_row[li] = row;
  }
  wave_lds_fence();

  struct Row {
    int32_t row, beg, end, c_first;
    float w_first;
    float4 acc;
  };
  auto fetch = [&](int k, Row& s) {
    s.row = l_row[k];
    const int2 seg0 = l_seg[k * kMaxMerge];
    s.beg = seg0.x;
    s.end = seg0.y;
    s.c_first = col_begin;
    s.w_first = 0.f;
    s.acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s.row < 0) return;
    if (s.beg + li < s.end) {
      s.c_first = bcol[s.beg + li];
      if (W) s.w_first = bw[s.beg + li];
    }
    if (!first) s.acc = ld4_stream(acc_buf + (int64_t)s.row * F + col);
  };

  Row cur, nxt;
  fetch(0, cur);
  for (int k = 0; k < R; ++k) {
    if (k + 1 < R) fetch(k + 1, nxt);
    if (cur.row >= 0) {
      float4 acc = cur.acc;
      int32_t beg = cur.beg, end = cur.end, c_next = cur.c_first;
      float w_next = cur.w_first;
      for (int sgi = 0; sgi < nseg; ++sgi) {
      // the bounds and the first indices of the row's segment in the next block are in flight
      // while this one is processed
      int32_t beg_n = 0, end_n = 0, c_first_n = col_begin;
      float w_first_n = 0.f;
      if (sgi + 1 < nseg) {
        const int2 sn = l_seg[k * kMaxMerge + sgi + 1];
        beg_n = sn.x;
        end_n = sn.y;
        if (beg_n + li < end_n) {
          c_first_n = bcol[beg_n + li];
          if (W) w_first_n = bw[beg_n + li];
        }
      }
      for (int32_t c0 = beg; c0 < end; c0 += SL) {
        // lanes past the end point at the block's first vertex (valid, cache-resident) and
        // their rows are multiplied by 0; with SKIP, quadruples of gathered rows that lie
        // entirely past the end are skipped (a padded load costs the texture path as much as a
        // real one).  The branches cost the overlap of the second half's loads with the first
        // half's sums: rows cut into four or more slices gain 2 % overall, rows cut into two lose
        // 24 % (measured), so SKIP is instantiated only for the former.
        const int32_t c = c0 + li < end ? c_next : col_begin;
        const float wv = c0 + li < end ? w_next : 0.f;
        if (c0 + SL + li < end) {
          c_next = bcol[c0 + SL + li];
          if (W) w_next = bw[c0 + SL + li];
        }
        l_idx[li] = c;
        if (W) l_w[li] = wv;
        wave_lds_fence();
        const int cnt = min(SL, end - c0);
        float4 part = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int t0 = 0; t0 < SL; t0 += U) {
          int idv[U];
#pragma unroll
          for (int q = 0; q < U / 4; ++q) {
            const int4 i4 = *reinterpret_cast<const int4*>(l_idx + t0 + 4 * q);
            idv[4 * q] = i4.x; idv[4 * q + 1] = i4.y; idv[4 * q + 2] = i4.z; idv[4 * q + 3] = i4.w;
          }
          float4 rowv[U];
#pragma unroll
          for (int t4 = 0; t4 < U; t4 += 4)
            if (!SKIP || t0 + t4 < cnt) {
#pragma unroll
              for (int t = t4; t < t4 + 4; ++t) rowv[t] = ld4(feat + (int64_t)idv[t] * F + col);
            }
#pragma unroll
          for (int t4 = 0; t4 < U; t4 += 4)
            if (!SKIP || t0 + t4 < cnt) {
#pragma unroll
              for (int t = t4; t < t4 + 4; ++t) fma4(part, W ? l_w[t0 + t] : (t0 + t < cnt ? 1.f : 0.f), rowv[t]);
            }
        }
        add4(acc, part);
        wave_lds_fence();
      }
      beg = beg_n;
      end = end_n;
      c_next = c_first_n;
      w_next = w_first_n;
      }
      st4_stream(acc_buf + (int64_t)cur.row * F + col, acc);
    }
    cur = nxt;
  }
}

// ---- all column blocks in one persistent launch: the running sums stay in LDS ------------
// The launches above pay for cache residency with one read-add-write of the [n, F] running sums
// per block.  Here one workgroup per CU runs for the whole pass and keeps the sums of up to
// kResSlots (row, slice) pairs in LDS.  It takes all of them through column block 0, then all of
// them through block 1, and so on ("phases"); after the last block it writes the rows out once
// and takes its next rows ("generation").  Every workgroup owns the same number of rows per
// generation, dealt from the degree order one position at a time in alternating direction, so
// all workgroups carry nearly the same load in every phase and walk the blocks in step by
// themselves; the workgroups of an XCD meet once per generation (phase_step_done, a bounded
// wait), so an L2 serves gathers from one block at a time.  Inside a workgroup the groups draw
// rows from an LDS counter, longest rows first, which levels the segments' lengths.  A row's
// sums run in block order and its edges in list order, so the result is bit-identical to the
// launch-per-block path whoever draws what.
constexpr int kResThreads = 1024;
constexpr int kResRows = 8;  // rows per group and generation (on average: the groups draw them)

template <int SL>
constexpr int kResSlots = (kResThreads / SL) * kResRows;
// LDS ints of a workgroup: sums | (beg, end) of two phases | row ids | per group idx (and weights) | two counters
template <int SL, bool W>
constexpr int kResLdsInts = 4 * SL * kResSlots<SL> + 2 * 2 * kResSlots<SL> + kResSlots<SL> +
                            (kResThreads / SL) * (W ? 2 : 1) * SL + 4;

template <int SL, bool W>
__global__ __launch_bounds__(kResThreads) void k_rowsum_res(
    int32_t n_rows, const int32_t* __restrict__ order, const int2* __restrict__ bseg /* [nblk][n_rows] */,
    const int32_t* __restrict__ bcol, const float* __restrict__ feat, int32_t block_cols, int nblk, int F,
    int ns, const float* __restrict__ scale /* nullable: factor per row */, float* __restrict__ out,
    const float* __restrict__ bw, int32_t* __restrict__ clock /* nullable: step counters, zeroed */,
    int spin_limit, int sync_every) {
  constexpr int GPB = kResThreads / SL;
  constexpr int R = kResRows;
  constexpr int NSLOT = kResSlots<SL>;
  constexpr int U = SL < 8 ? 4 : 8;
  static_assert(NSLOT <= kResThreads, "one thread per slot loads its segment bounds");
  extern __shared__ __align__(16) int lds_res[];
  const int lane = threadIdx.x & 63;
  const int li = threadIdx.x & (SL - 1);
  const int grp = threadIdx.x / SL;
  const int slice = blockIdx.x % ns;
  const int64_t nwg = gridDim.x / ns;         // workgroups that serve this slice
  const int64_t wg = blockIdx.x / ns;
  const int64_t ngroups = nwg * GPB;
  float4* l_acc = reinterpret_cast<float4*>(lds_res);            // [NSLOT][SL]
  int2* l_seg = reinterpret_cast<int2*>(lds_res + 4 * SL * NSLOT);  // [2][NSLOT]
  int* l_row = lds_res + 4 * SL * NSLOT + 4 * NSLOT;             // [NSLOT]
  int* l_idx = l_row + NSLOT + grp * (W ? 2 : 1) * SL;
  float* l_w = reinterpret_cast<float*>(l_idx + SL);
  int* l_cnt = l_row + NSLOT + GPB * (W ? 2 : 1) * SL;           // [2]
  // a row narrower than its slice: the lanes past its end gather its first columns again (same
  // cache line) and store nothing
  const bool col_ok = slice * 4 * SL + 4 * li < F;
  const int col = col_ok ? slice * 4 * SL + 4 * li : 0;

  const int64_t rows_per_group = (n_rows + ngroups - 1) / ngroups;
  const int ngen = (int)((rows_per_group + R - 1) / R);
  // workgroups go to the XCDs round-robin: those with the same id mod 8 share an L2
  PhaseClock pc{clock ? clock + (blockIdx.x % kXcds) * kClockStride : nullptr, (int)(gridDim.x / kXcds), spin_limit,
                false, sync_every > 0 ? sync_every : nblk};

  struct Item {
    int32_t beg, end, c_first;
    float w_first;
  };

  for (int gen = 0; gen < ngen; ++gen) {
    const int64_t j0 = gen * rows_per_group / ngen, j1 = (gen + 1) * rows_per_group / ngen;
    const int nslots = (int)(j1 - j0) * GPB;  // slot q: row at position (j0 * GPB + q) * nwg + wg (or + nwg - 1 - wg)
    __syncthreads();                          // the previous generation's rows are written out
    int64_t pos = -1;                         // thread q < nslots: position of slot q's row in the degree order
    if ((int)threadIdx.x < nslots) {
      // consecutive positions of the degree order go to consecutive workgroups, in alternating
      // direction from one round to the next, so every workgroup gets the same mix of degrees
      const int64_t r = (j0 * GPB + threadIdx.x) * nwg + ((threadIdx.x & 1) ? nwg - 1 - wg : wg);
      if (r < n_rows) pos = r;
      l_row[threadIdx.x] = pos >= 0 ? order[pos] : -1;
      l_seg[threadIdx.x] = pos >= 0 ? bseg[pos] : make_int2(0, 0);
    }
    for (int i = threadIdx.x; i < nslots * SL; i += kResThreads) l_acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (threadIdx.x == 0) l_cnt[0] = 0;
    __syncthreads();  // the tables are in place

    // a group's next slot of phase p, from that phase's counter
    auto grab = [&](int p) {
      int q = 0;
      if (li == 0) q = atomicAdd(l_cnt + (p & 1), 1);
      return __shfl(q, lane & ~(SL - 1), 64);
    };
    // what a slot needs before its edge loop in phase p: bounds and first indices
    auto fetch = [&](int p, int q) {
      Item it{0, 0, p * block_cols, 0.f};
      if (q >= nslots) return it;
      const int2 sg = l_seg[(p & 1) * NSLOT + q];
      it.beg = sg.x;
      it.end = sg.y;
      if (it.beg + li < it.end) {
        it.c_first = bcol[it.beg + li];
        if (W) it.w_first = bw[it.beg + li];
      }
      return it;
    };
    int q = grab(0);
    Item cur = fetch(0, q);

    for (int p = 0; p < nblk; ++p) {
      const int32_t col_begin = p * block_cols;
      // the next phase's bounds travel while this one is worked on
      int2 seg_next = make_int2(0, 0);
      if (p + 1 < nblk && pos >= 0) seg_next = bseg[(int64_t)(p + 1) * n_rows + pos];
      if (threadIdx.x == 0) l_cnt[(p + 1) & 1] = 0;

      while (q < nslots) {
        const int qn = grab(p);
        const Item nxt = fetch(p, qn);
        const int32_t beg = cur.beg, end = cur.end;
        if (beg < end) {
          float4 acc = l_acc[q * SL + li];
          int32_t c_next = cur.c_first;
          float w_next = cur.w_first;
          for (int32_t c0 = beg; c0 < end; c0 += SL) {
            const int32_t c = c0 + li < end ? c_next : col_begin;
            const float wv = c0 + li < end ? w_next : 0.f;
            if (c0 + SL + li < end) {
              c_next = bcol[c0 + SL + li];
              if (W) w_next = bw[c0 + SL + li];
            }
            l_idx[li] = c;
            if (W) l_w[li] = wv;
            wave_lds_fence();
            const int cn = min(SL, end - c0);
            float4 part = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int t0 = 0; t0 < SL; t0 += U) {
              int idv[U];
#pragma unroll
              for (int qq = 0; qq < U / 4; ++qq) {
                const int4 i4 = *reinterpret_cast<const int4*>(l_idx + t0 + 4 * qq);
                idv[4 * qq] = i4.x; idv[4 * qq + 1] = i4.y; idv[4 * qq + 2] = i4.z; idv[4 * qq + 3] = i4.w;
              }
              float4 rowv[U];
#pragma unroll
              for (int t4 = 0; t4 < U; t4 += 4)
                if (t0 + t4 < cn) {
#pragma unroll
                  for (int t = t4; t < t4 + 4; ++t) rowv[t] = ld4(feat + (int64_t)idv[t] * F + col);
                }
#pragma unroll
              for (int t4 = 0; t4 < U; t4 += 4)
                if (t0 + t4 < cn) {
#pragma unroll
                  for (int t = t4; t < t4 + 4; ++t) fma4(part, W ? l_w[t0 + t] : (t0 + t < cn ? 1.f : 0.f), rowv[t]);
                }
            }
            add4(acc, part);
            wave_lds_fence();
          }
          l_acc[q * SL + li] = acc;
        }
        q = qn;
        cur = nxt;
      }
      if ((int)threadIdx.x < nslots) l_seg[((p + 1) & 1) * NSLOT + threadIdx.x] = seg_next;
      __syncthreads();  // the workgroup is done with this block; the next phase's bounds are in LDS
      if (p + 1 < nblk) {  // first slot of the next phase: its loads travel during the wait below
        q = grab(p + 1);
        cur = fetch(p + 1, q);
      }
      phase_step_done(pc, gen * nblk + p);
      __syncthreads();  // every workgroup of the XCD is done with this block (or the wait ran out)
    }
    for (int q = grp; q < nslots; q += GPB) {
      const int32_t row = l_row[q];
      if (row < 0 || !col_ok) continue;
      float4 acc = l_acc[q * SL + li];
      if (scale != nullptr) scale4(acc, scale[row]);
      st4_stream(out + (int64_t)row * F + col, acc);
    }
  }
}

// A row of F floats is cut into `ns` slices of SL float4.  Slices of 256 bytes where the row has
// 2, 4 or 8 of them (measured at 1 KB rows: 17.8 -> 17.2 ms per layer against 8 slices of 128
// bytes, 22.9 ms with two of 512); wider rows have 8 slices, one per XCD.  With fewer than 8,
// workgroup id mod `ns` picks the slice, so XCD k and XCD k + ns share columns and split the rows.
static bool gcn_slicing(int F, int& SL, int& ns) {
  // rows of at most 64 floats: one slice, persistent kernel only (a launch per block would move
  // as many bytes of running sums as of gathered rows)
  if (F <= 64 && F % 4 == 0 && config_get(kCfgResidentSums)) {
    SL = 16;
    ns = 1;
    return true;
  }
  if (F % 32 != 0) return false;
  const int q = F / 32;
  if (q == 4 || q == 8 || q == 16) {
    SL = 16;
    ns = q / 2;
    return true;
  }
  if (q >= kGcnSlices) {
    SL = q;
    ns = kGcnSlices;
    return q == 32;
  }
  return false;  // narrower rows stay with the single-launch kernel
}

static bool gcn_blocked_applies(const gnn_graph_t* g, int F) {
  if (!g->blocked_pays() || config_get(kCfgForceSimple)) return false;
  int SL, ns;
  return gcn_slicing(F, SL, ns);
}

template <int SL>
static gnn_status_t launch_rowsum_blocks(const gnn_graph_t* g, int side, const char* name, const float* feat,
                                         int F, float* acc, hipStream_t st, const float* bw = nullptr) {
  const int rows_per_wg = (kGcnBlock / SL) * kGcnRows;
  const int ns = F / (4 * SL);
  const unsigned grid = (unsigned)(cdiv(g->n, rows_per_wg) * ns);
  const std::vector<int32_t>& groups = g->h_group[side][0];
  GNN_REQUIRE(groups.size() >= 2 && groups.front() == 0 && groups.back() == g->nblk, GNN_ERR_UNSUPPORTED,
              "gcn blocked: the plan has no launch groups");
  for (size_t gi = 0; gi + 1 < groups.size(); ++gi) {
    const int b = groups[gi], nseg = groups[gi + 1] - b;
    GNN_REQUIRE(nseg >= 1 && nseg <= kMaxMerge, GNN_ERR_UNSUPPORTED, "gcn blocked: bad launch group");
    const int2* bseg_b = reinterpret_cast<const int2*>(g->bseg[side]) + (int64_t)b * g->n;
    ProfScope p(name, st);  // one timed bracket per launch
    if (bw != nullptr && ns >= 4)
      k_rowsum_blk<SL, true, true><<<grid, kGcnBlock, 0, st>>>(g->n, g->order[side], bseg_b, g->bcol[side], feat,
                                                              b * g->block_cols, F, b == 0, ns, acc, nseg, bw);
    else if (bw != nullptr)
      k_rowsum_blk<SL, false, true><<<grid, kGcnBlock, 0, st>>>(g->n, g->order[side], bseg_b, g->bcol[side], feat,
                                                               b * g->block_cols, F, b == 0, ns, acc, nseg, bw);
    else if (ns >= 4)
      k_rowsum_blk<SL, true><<<grid, kGcnBlock, 0, st>>>(g->n, g->order[side], bseg_b, g->bcol[side], feat,
                                                        b * g->block_cols, F, b == 0, ns, acc, nseg);
    else
      k_rowsum_blk<SL, false><<<grid, kGcnBlock, 0, st>>>(g->n, g->order[side], bseg_b, g->bcol[side], feat,
                                                         b * g->block_cols, F, b == 0, ns, acc, nseg);
    GNN_LAUNCH_CHECK();
  }
  return GNN_OK;
}

__global__ void k_zero_clock(int32_t* __restrict__ clock) { clock[threadIdx.x] = 0; }

// LDS of the persistent kernel; more than 64 KB of dynamic LDS needs the attribute once per instantiation
constexpr size_t kResLdsLimit = 152 * 1024;
template <int SL, bool W>
static gnn_status_t launch_rowsum_resident(const gnn_graph_t* g, int side, const char* name, const float* feat,
                                           int F, const float* scale, float* out, hipStream_t st,
                                           const float* bw) {
  const int ns = F <= 4 * SL ? 1 : F / (4 * SL);
  const size_t lds = sizeof(int) * (size_t)kResLdsInts<SL, W>;
  GNN_REQUIRE(lds <= kResLdsLimit, GNN_ERR_UNSUPPORTED, "gcn resident: %zu bytes of LDS", lds);
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_acquire)) {
    GNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_rowsum_res<SL, W>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kResLdsLimit));
    attr_set.store(true, std::memory_order_release);
  }
  // one workgroup per CU, a multiple of the slice count so that every XCD serves one slice
  const unsigned grid = (unsigned)(device_cu_count() / kXcds * kXcds);
  ProfScope p(name, st);
  int32_t* clock = g->phase_clock;
  if (clock != nullptr) {
    k_zero_clock<<<1, kXcds * kClockStride, 0, st>>>(clock);
    GNN_LAUNCH_CHECK();
  }
  k_rowsum_res<SL, W><<<grid, kResThreads, lds, st>>>(g->n, g->order[side], reinterpret_cast<const int2*>(g->bseg[side]),
                                                     g->bcol[side], feat, g->block_cols, g->nblk, F, ns, scale, out, bw,
                                                     clock, (int)config_get(kCfgResidentSpin), (int)config_get(kCfgResidentSyncEvery));
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

template <int L, int NV>
struct RowsumLauncher {
  static gnn_status_t run(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                          const float* scale, float* out, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kGcnBlock / kWave);
    ProfScope p(name, st);
    const RowSplit sp = split_rows(g, side, L, GPB);
    const int32_t* ptr = side == 0 ? g->indptr : g->indptr_t;
    const int32_t* cols = side == 0 ? g->indices : g->indices_t;
    // hub rows (one workgroup each) and the rest in one launch
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_rowsum<L, NV><<<grid, kGcnBlock, 0, st>>>(rl, g->order[side], ptr, cols, feat, F, scale, out);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

// the same sum with a static weight per edge (wgt in the order of the side's edge array)
template <int L, int NV>
struct RowsumWeightedLauncher {
  static gnn_status_t run(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                          const float* wgt, float* out, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kGcnBlock / kWave);
    ProfScope p(name, st);
    const RowSplit sp = split_rows(g, side, L, GPB);
    const int32_t* ptr = side == 0 ? g->indptr : g->indptr_t;
    const int32_t* cols = side == 0 ? g->indices : g->indices_t;
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_rowsum<L, NV, true><<<grid, kGcnBlock, 0, st>>>(rl, g->order[side], ptr, cols, feat, F, nullptr, out, wgt);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct RowsumEbLauncher {
  static gnn_status_t run(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                          const float* scale, float* out, hipStream_t st) {
    constexpr int GPB = kGcnBlock / L;
    ProfScope p(name, st);
    const int64_t quads = (int64_t)g->n * (F / 4);
    k_zero_f4<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, out);
    GNN_LAUNCH_CHECK();
    const int64_t runs = cdiv(g->nnz, kEbEdges);
    if (runs != 0) {
      k_rowsum_eb<L, NV><<<(unsigned)cdiv(runs, GPB), kGcnBlock, 0, st>>>(
          g->n, (int32_t)g->nnz, side == 0 ? g->indptr : g->indptr_t, side == 0 ? g->indices : g->indices_t,
          feat, F, scale, out);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct RowsumWeightedEbLauncher {
  static gnn_status_t run(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                          const float* wgt, float* out, hipStream_t st) {
    constexpr int GPB = kGcnBlock / L;
    ProfScope p(name, st);
    const int64_t quads = (int64_t)g->n * (F / 4);
    k_zero_f4<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, out);
    GNN_LAUNCH_CHECK();
    const int64_t runs = cdiv(g->nnz, kEbEdges);
    if (runs != 0) {
      k_rowsum_eb<L, NV, true><<<(unsigned)cdiv(runs, GPB), kGcnBlock, 0, st>>>(
          g->n, (int32_t)g->nnz, side == 0 ? g->indptr : g->indptr_t, side == 0 ? g->indices : g->indices_t,
          feat, F, nullptr, out, wgt);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <template <int, int> class Launcher>
static gnn_status_t dispatch_rowsum(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                                    const float* scale, float* out, hipStream_t st) {
  const GroupShape gs = pick_group(F);
  switch (gs.L) {
    case 4: return Launcher<4, 1>::run(g, side, name, feat, F, scale, out, st);
    case 8: return Launcher<8, 1>::run(g, side, name, feat, F, scale, out, st);
    case 16: return Launcher<16, 1>::run(g, side, name, feat, F, scale, out, st);
    case 32: return Launcher<32, 1>::run(g, side, name, feat, F, scale, out, st);
    case 64:
      switch (gs.NV) {
        case 1: return Launcher<64, 1>::run(g, side, name, feat, F, scale, out, st);
        case 2: return Launcher<64, 2>::run(g, side, name, feat, F, scale, out, st);
        case 3: return Launcher<64, 3>::run(g, side, name, feat, F, scale, out, st);
        case 4: return Launcher<64, 4>::run(g, side, name, feat, F, scale, out, st);
      }
  }
  set_error("unsupported row-group shape L=%d NV=%d", gs.L, gs.NV);
  return GNN_ERR_UNSUPPORTED;
}

// mapping: 0 vertex-balanced, 1 edge-balanced, 2 what gnn_gcn_tune found faster on this graph
// (vertex-balanced on a graph that was never tuned)
static bool use_edge_balanced(const gnn_graph_t* g, int side) {
  const int64_t mode = config_get(kCfgGcnMapping);
  if (mode == 1) return true;
  return mode == 2 && g->gcn_edge_balanced[side] == 1;
}

// vertex-balanced: column-blocked launches on large graphs, else one launch
static gnn_status_t gcn_aggregate_vertex(const gnn_graph_t* g, int side, const char* name, const float* feat,
                                         int F, const float* scale, float* out, hipStream_t st) {
  if (gcn_blocked_applies(g, F)) {
    int SL = 0, ns = 0;
    gcn_slicing(F, SL, ns);
    if (config_get(kCfgResidentSums) && SL == 16)
      return launch_rowsum_resident<16, false>(g, side, name, feat, F, scale, out, st, nullptr);
    switch (SL) {
      case 8: GNN_TRY(launch_rowsum_blocks<8>(g, side, name, feat, F, out, st)); break;
      case 16: GNN_TRY(launch_rowsum_blocks<16>(g, side, name, feat, F, out, st)); break;
      default: GNN_TRY(launch_rowsum_blocks<32>(g, side, name, feat, F, out, st)); break;
    }
    ProfScope p("gcn_scale_rows", st);
    const int64_t quads = (int64_t)g->n * (F / 4);
    k_scale_rows<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, F / 4, scale, out, out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
  return dispatch_rowsum<RowsumLauncher>(g, side, name, feat, F, scale, out, st);
}

// out[row,:] = scale[row] * sum of feat over the row's neighbours on `side` (0: in-edges, 1: out-edges)
static gnn_status_t gcn_aggregate(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                                  const float* scale, float* out, hipStream_t st) {
  if (use_edge_balanced(g, side)) return dispatch_rowsum<RowsumEbLauncher>(g, side, name, feat, F, scale, out, st);
  return gcn_aggregate_vertex(g, side, name, feat, F, scale, out, st);
}

// out[row,:] = sum over the row's edges on `side` of weight * feat[neighbour,:]  (vertex-balanced:
// column-blocked launches on large graphs, else one launch)
static gnn_status_t gcn_aggregate_weighted(const gnn_graph_t* g, const gnn_edge_weights* ew, int side,
                                           const char* name, const float* feat, int F, float* out,
                                           hipStream_t st) {
  // edge-balanced only on request (gcn_mapping = 1): gnn_gcn_tune times the unweighted sums
  if (config_get(kCfgGcnMapping) == 1)
    return dispatch_rowsum<RowsumWeightedEbLauncher>(g, side, name, feat, F, ew->w_side[side], out, st);
  if (gcn_blocked_applies(g, F) && ew->w_blk[side] != nullptr) {
    int SL = 0, ns = 0;
    gcn_slicing(F, SL, ns);
    if (config_get(kCfgResidentSums) && SL == 16)
      return launch_rowsum_resident<16, true>(g, side, name, feat, F, nullptr, out, st, ew->w_blk[side]);
    switch (SL) {
      case 8: return launch_rowsum_blocks<8>(g, side, name, feat, F, out, st, ew->w_blk[side]);
      case 16: return launch_rowsum_blocks<16>(g, side, name, feat, F, out, st, ew->w_blk[side]);
      default: return launch_rowsum_blocks<32>(g, side, name, feat, F, out, st, ew->w_blk[side]);
    }
  }
  return dispatch_rowsum<RowsumWeightedLauncher>(g, side, name, feat, F, ew->w_side[side], out, st);
}

struct GcnWs {
  size_t total, gs, dz, gemm;
  int split_k;
};

static GcnWs gcn_ws_layout(int64_t n, int fin, int fout) {
  GcnWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += ws_granule(bytes); return o; };
  w.gs = take(sizeof(float) * (size_t)n * fout);
  w.dz = take(sizeof(float) * (size_t)n * fout);
  w.split_k = gemm_pick_split_k(fin, fout, n);
  w.gemm = take(w.split_k > 1 ? sizeof(float) * (size_t)w.split_k * fin * fout : 0);
  w.total = off;
  return w;
}

static gnn_status_t gcn_check(const gnn_graph_t* g, int fin, int fout, const char* who) {
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "%s: graph is null", who);
  GNN_REQUIRE(fin > 0 && fout > 0, GNN_ERR_INVALID_ARG, "%s: sizes must be positive", who);
  GNN_REQUIRE(fout % 4 == 0 && fout <= 1024, GNN_ERR_UNSUPPORTED,
              "%s: fout = %d must be a multiple of 4, at most 1024", who, fout);
  return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" size_t gnn_gcn_workspace_bytes(const gnn_graph_t* g, int fin, int fout) {
  if (!g || fin <= 0 || fout <= 0) return 0;
  return gcn_ws_layout(g->n, fin, fout).total;
}

extern "C" gnn_status_t gnn_gcn_fwd(const gnn_graph_t* g, int fin, int fout, const float* x, const float* w,
                                    const float* c_src, const float* c_dst, float* zs, float* out,
                                    void* stream) {
  clear_error();
  GNN_TRY(gcn_check(g, fin, fout, "gnn_gcn_fwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && c_src && c_dst && zs && out, GNN_ERR_INVALID_ARG, "gnn_gcn_fwd: null pointer");
  GNN_REQUIRE(aligned16(zs) && aligned16(out), GNN_ERR_INVALID_ARG,
              "gnn_gcn_fwd: zs, out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  // projection before propagation, then the source half of the edge weight on vertices
  GNN_TRY(gemm_f32(g->n, fout, fin, x, fin, false, w, fout, false, zs, fout, 1, nullptr, st));
  {
    ProfScope p("gcn_scale_rows", st);
    const int64_t quads = (int64_t)g->n * (fout / 4);
    k_scale_rows<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, fout / 4, c_src, zs, zs);
    GNN_LAUNCH_CHECK();
  }
  return gcn_aggregate(g, 0, "gcn_fwd_fused", zs, fout, c_dst, out, st);
}

extern "C" gnn_status_t gnn_gcn_bwd(const gnn_graph_t* g, int fin, int fout, const float* x, const float* w,
                                    const float* c_src, const float* c_dst, const float* gout, float* gx,
                                    float* gw, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(gcn_check(g, fin, fout, "gnn_gcn_bwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && c_src && c_dst && gout && gw, GNN_ERR_INVALID_ARG, "gnn_gcn_bwd: null pointer");
  GNN_REQUIRE(aligned16(gout), GNN_ERR_INVALID_ARG, "gnn_gcn_bwd: gout must be 16-byte aligned");
  const GcnWs L = gcn_ws_layout(g->n, fin, fout);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "gnn_gcn_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_gcn_bwd: workspace must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  float* gs = reinterpret_cast<float*>(base + L.gs);
  float* dz = reinterpret_cast<float*>(base + L.dz);
  float* part = reinterpret_cast<float*>(base + L.gemm);
  {
    ProfScope p("gcn_scale_rows", st);
    const int64_t quads = (int64_t)g->n * (fout / 4);
    k_scale_rows<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, fout / 4, c_dst, gout, gs);
    GNN_LAUNCH_CHECK();
  }
  GNN_TRY(gcn_aggregate(g, 1, "gcn_bwd_src", gs, fout, c_src, dz, st));
  GNN_TRY(gemm_f32(fin, fout, g->n, x, fin, true, dz, fout, false, gw, fout, L.split_k, part, st));
  if (gx) GNN_TRY(gemm_f32(g->n, fin, fout, dz, fout, false, w, fout, true, gx, fin, 1, nullptr, st));
  return GNN_OK;
}

static gnn_status_t gcn_edge_check(const gnn_graph_t* g, const gnn_edge_weights* ew, const char* who) {
  GNN_REQUIRE(ew != nullptr, GNN_ERR_INVALID_ARG, "%s: edge weights are null", who);
  GNN_REQUIRE(ew->graph == g && ew->nnz == g->nnz, GNN_ERR_INVALID_ARG,
              "%s: the edge weights were made for another graph", who);
  return GNN_OK;
}

extern "C" gnn_status_t gnn_gcn_edge_fwd(const gnn_graph_t* g, const gnn_edge_weights_t* ew, int fin, int fout,
                                         const float* x, const float* w, float* z, float* out, void* stream) {
  clear_error();
  GNN_TRY(gcn_check(g, fin, fout, "gnn_gcn_edge_fwd"));
  GNN_TRY(gcn_edge_check(g, ew, "gnn_gcn_edge_fwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && z && out, GNN_ERR_INVALID_ARG, "gnn_gcn_edge_fwd: null pointer");
  GNN_REQUIRE(aligned16(z) && aligned16(out), GNN_ERR_INVALID_ARG,
              "gnn_gcn_edge_fwd: z, out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  GNN_TRY(gemm_f32(g->n, fout, fin, x, fin, false, w, fout, false, z, fout, 1, nullptr, st));
  return gcn_aggregate_weighted(g, ew, 0, "gcn_fwd_fused", z, fout, out, st);
}

extern "C" gnn_status_t gnn_gcn_edge_bwd(const gnn_graph_t* g, const gnn_edge_weights_t* ew, int fin, int fout,
                                         const float* x, const float* w, const float* gout, float* gx,
                                         float* gw, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(gcn_check(g, fin, fout, "gnn_gcn_edge_bwd"));
  GNN_TRY(gcn_edge_check(g, ew, "gnn_gcn_edge_bwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && gout && gw, GNN_ERR_INVALID_ARG, "gnn_gcn_edge_bwd: null pointer");
  GNN_REQUIRE(aligned16(gout), GNN_ERR_INVALID_ARG, "gnn_gcn_edge_bwd: gout must be 16-byte aligned");
  const GcnWs L = gcn_ws_layout(g->n, fin, fout);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "gnn_gcn_edge_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_gcn_edge_bwd: workspace must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  float* dz = reinterpret_cast<float*>(base + L.dz);
  float* part = reinterpret_cast<float*>(base + L.gemm);
  // dz[u] = sum over out-edges of e_uv gout[v]: the same weighted sum over the transpose
  GNN_TRY(gcn_aggregate_weighted(g, ew, 1, "gcn_bwd_src", gout, fout, dz, st));
  GNN_TRY(gemm_f32(fin, fout, g->n, x, fin, true, dz, fout, false, gw, fout, L.split_k, part, st));
  if (gx) GNN_TRY(gemm_f32(g->n, fin, fout, dz, fout, false, w, fout, true, gx, fin, 1, nullptr, st));
  return GNN_OK;
}

__global__ void k_fill_f32(int64_t count, float value, float* __restrict__ p) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < count) p[i] = value;
}

extern "C" gnn_status_t gnn_gcn_tune(gnn_graph_t* g, int fout, void* ws, size_t ws_bytes, void* stream,
                                     float* ms_out) {
  clear_error();
  GNN_TRY(gcn_check(g, 1, fout, "gnn_gcn_tune"));
  const GcnWs L = gcn_ws_layout(g->n, 1, fout);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "gnn_gcn_tune: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_gcn_tune: workspace must be 16-byte aligned");
  float ms[4] = {0.f, 0.f, 0.f, 0.f};
  if (g->n != 0 && g->nnz != 0) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(ws);
    float* feat = reinterpret_cast<float*>(base + L.gs);  // all ones; its first n entries double as the scale
    float* out = reinterpret_cast<float*>(base + L.dz);
    const int64_t count = (int64_t)g->n * fout;
    k_fill_f32<<<(unsigned)cdiv(count, 256), 256, 0, st>>>(count, 1.f, feat);
    GNN_LAUNCH_CHECK();
    hipEvent_t a = nullptr, b = nullptr;
    GNN_HIP(hipEventCreate(&a));
    if (hipEventCreate(&b) != hipSuccess) {
      (void)hipEventDestroy(a);
      set_error("gnn_gcn_tune: hipEventCreate failed");
      return GNN_ERR_HIP;
    }
    constexpr int kReps = 3;
    gnn_status_t status = GNN_OK;
    for (int side = 0; side < 2 && status == GNN_OK; ++side) {
      for (int eb = 0; eb < 2 && status == GNN_OK; ++eb) {
        auto once = [&]() {
          return eb ? dispatch_rowsum<RowsumEbLauncher>(g, side, "gcn_tune", feat, fout, feat, out, st)
                    : gcn_aggregate_vertex(g, side, "gcn_tune", feat, fout, feat, out, st);
        };
        status = once();  // warm-up
        if (status == GNN_OK && hipEventRecord(a, st) != hipSuccess) status = GNN_ERR_HIP;
        for (int r = 0; r < kReps && status == GNN_OK; ++r) status = once();
        if (status == GNN_OK && (hipEventRecord(b, st) != hipSuccess || hipEventSynchronize(b) != hipSuccess))
          status = GNN_ERR_HIP;
        float t = 0.f;
        if (status == GNN_OK && hipEventElapsedTime(&t, a, b) != hipSuccess) status = GNN_ERR_HIP;
        ms[2 * side + eb] = t / kReps;
      }
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (status != GNN_OK) {
      if (status == GNN_ERR_HIP && gnn_last_error()[0] == 0) set_error("gnn_gcn_tune: a HIP event call failed");
      return status;
    }
    for (int side = 0; side < 2; ++side) g->gcn_edge_balanced[side] = ms[2 * side + 1] < ms[2 * side] ? 1 : 0;
  }
  if (ms_out)
    for (int i = 0; i < 4; ++i) ms_out[i] = ms[i];
  return GNN_OK;
}

// Which instantiation of the column-blocked sum a pass launches for this graph and width under the
// current configuration, spelled as a profiler prints it; "" when other kernels run.
extern "C" gnn_status_t gnn_gcn_blocked_kernel_name(const gnn_graph_t* g, int fout, int weighted, char* buf,
                                                    size_t len) {
  clear_error();
  GNN_REQUIRE(g != nullptr && buf != nullptr && len > 0, GNN_ERR_INVALID_ARG,
              "gnn_gcn_blocked_kernel_name: null argument");
  buf[0] = 0;
  if (fout <= 0 || !gcn_blocked_applies(g, fout) || config_get(kCfgGcnMapping) == 1) return GNN_OK;
  int SL = 0, ns = 0;
  gcn_slicing(fout, SL, ns);
  if (config_get(kCfgResidentSums) && SL == 16 && g->phase_clock != nullptr)
    std::snprintf(buf, len, "k_rowsum_res<16, %s>", weighted ? "true" : "false");
  else
    std::snprintf(buf, len, "k_rowsum_blk<%d, %s, %s>", SL, ns >= 4 ? "true" : "false", weighted ? "true" : "false");
  return GNN_OK;
}
