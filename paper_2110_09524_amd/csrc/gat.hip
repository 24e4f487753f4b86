// GAT layer: attention halves, the fused score -> edge-softmax -> aggregate
// kernel, and the recomputing backward kernels.
//
// Forward (App. A.2 "GAT", fused operator M0..H^(l+1); Sec. 5 example): one row
// group per destination, online softmax over chunks of its in-edges, the
// projected source rows gathered with 16-byte loads.  Saved: max m and
// denominator d per (vertex, head) only (Sec. 6 example).
//
// Backward (Sec. 6; operator rules of App. B).  With alpha_e the softmax value,
// g_e = LeakyReLU'(el[u]+er[v]) and D[v,h] = <gout[v,h,:], out[v,h,:]>, the score
// gradient of edge e is  dp_e = alpha_e g_e (<gout[v,h,:], z[u,h,:]> - D[v,h]).
// Instead of one dot product per edge, the dot product is postponed past the
// neighbourhood sum (the same distributive-law argument as Sec. 4):
//   der[v,h] = sum_in  dp_e = <gout[v,h,:], sum_in alpha_e g_e z[u,h,:]> - D[v,h] sum_in alpha_e g_e
//   del[u,h] = sum_out dp_e = <z[u,h,:], sum_out alpha_e g_e gout[v,h,:]> - sum_out alpha_e g_e D[v,h]
// so both backward kernels are weighted row aggregations like the forward one:
// the destination-side kernel walks the CSR, the source-side kernel walks the
// CSC transpose (no atomics), and alpha_e is recomputed from el, er, m, d.
#include "common.h"
#include <hip/hip_fp16.h>

#include <mutex>

#include "gat_common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kBlock = 256;  // 4 wavefronts
#ifndef GNN_GAT_UNROLL
#define GNN_GAT_UNROLL 4
#endif
constexpr int kU = GNN_GAT_UNROLL;  // gathered rows in flight per lane

// ---- a2: attention halves  el = <z, a_l>, er = <z, a_r> per (vertex, head) -----
__global__ void k_gat_attn_halves(int64_t n, int H, int F, const float* __restrict__ z,
                                  const float* __restrict__ a_l, const float* __restrict__ a_r,
                                  float* __restrict__ el, float* __restrict__ er) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;  // (vertex, head)
  if (i >= n * H) return;
  int h = (int)(i % H);
  const float* zr = z + i * F;  // z[v, h, :] : i*F = (v*H + h)*F
  const float* al = a_l + (int64_t)h * F;
  const float* ar = a_r + (int64_t)h * F;
  float sl = 0.f, sr = 0.f;
  for (int f = 0; f < F; f += 4) {
    float4 zz = ld4(zr + f);
    sl += dot4(zz, ld4(al + f));
    sr += dot4(zz, ld4(ar + f));
  }
  el[i] = sl;
  er[i] = sr;
}


// LDS layout per group: idx[L] | p[L] | p2[L] | misc[L] | red[2*L*NV]
template <int L, int NV>
struct GroupLds {
  static constexpr int kFloats = 4 * L + 2 * L * NV;
};

// ---- a3: fused forward ----------------------------------------------------------
// WT: also produce t[v] = sum_e alpha_e g_e z[u] and sg[v,h] = sum_e alpha_e g_e, the two
// destination-side sums of the backward pass.  They ride on the same gathered rows, and
// they are O(|V|) vertex state, which is cheaper to stash than to recompute (Sec. 6:
// recompute only when computation / memory is O(1); here it is |E|/|V|).
template <int L, int NV, bool WT, int ES>
__global__ __launch_bounds__(kBlock) void k_gat_fwd(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ z, const float* __restrict__ el,
    const float* __restrict__ er, GatDims dm, float* __restrict__ out, float* __restrict__ m_out,
    float* __restrict__ d_out, float* __restrict__ t_out, float* __restrict__ sg_out) {
  // A row group has GL = L * ES lanes: L column lanes (float4 slots), replicated ES times.  The
  // chunk phase spreads all GL lanes over (edge, head) pairs; in the row phase replica s takes
  // the chunk's edges s, s + ES, ... and the replicas' sums are added at the end of the row.
  // Narrow rows with many heads (8 heads x 8 columns: L = 16) would otherwise see two edges
  // per chunk and walk a row in many short, latency-bound steps.
  constexpr int GL = L * ES;
  constexpr int G = kWave / GL;
  constexpr int GPB = G * (kBlock / kWave);
  constexpr int NC = (WT ? 8 : 4) * NV + 2;  // floats per lane folded across cooperating groups
  static_assert(GL <= kWave && (ES == 1 || NV == 1), "replicas only for rows of at most 64 float4 slots");
  __shared__ float lds[GPB * GroupLds<GL, NV>::kFloats];
  __shared__ float coop_buf[GPB * GL * NC];
  __shared__ float coop_m[GPB * GL];

  const int lane = threadIdx.x & 63;
  const int li = lane & (GL - 1);
  const int grp = threadIdx.x / GL;  // group inside the block
  const int cl = li & (L - 1);       // column lane
  const int rep = li / L;            // replica: which of the chunk's edges this lane adds up
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;  // whole group (coop: whole workgroup) leaves together
  float* g_lds = lds + grp * GroupLds<GL, NV>::kFloats;
  int* l_idx = reinterpret_cast<int*>(g_lds);
  float* l_p = g_lds + GL;
  float* l_p2 = g_lds + 2 * GL;
  float* l_sc = g_lds + 3 * GL;

  const int H = dm.H, HF = dm.HF;
  const int Hp = 1 << dm.log2Hp;
  const int epc = GL >> dm.log2Hp;  // edges per chunk
  const int e_loc = li >> dm.log2Hp;
  const int h = li & (Hp - 1);
  const bool head_ok = h < H;

  const int32_t v = order[r];
  const int32_t beg = indptr[v], end = indptr[v + 1];
  const float er_vh = head_ok ? er[(int64_t)v * H + h] : 0.f;

  int hs[NV];
  bool slot_ok[NV];
  float4 acc[NV], acc2[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int col = 4 * (cl + j * L);
    slot_ok[j] = col < HF;
    hs[j] = slot_ok[j] ? col / dm.F : 0;
    acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    acc2[j] = acc[j];
  }

  float m_run = -INFINITY, d_run = 0.f, d2_run = 0.f;
  for (int32_t c0 = beg + gi * epc; c0 < end; c0 += ngrp * epc) {
    // chunk phase: lane = (edge e_loc of the chunk, head h)
    const int32_t e = c0 + e_loc;
    const bool e_ok = e < end;
    const int32_t u = e_ok ? indices[e] : 0;
    float s = -INFINITY, raw = 0.f;
    if (e_ok && head_ok) {
      raw = el[(int64_t)u * H + h] + er_vh;
      s = leaky(raw, dm.slope);
    }
    const float cmax = group_max_from<GL>(s, Hp);
    const float m_new = fmaxf(m_run, cmax);
    const float p = (e_ok && head_ok) ? __expf(s - m_new) : 0.f;
    const float sc = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
    d_run = d_run * sc + p;
    m_run = m_new;
    if (h == 0) l_idx[e_loc] = u;
    l_p[li] = p;
    if (WT) {
      const float p2 = raw > 0.f ? p : dm.slope * p;  // weight times LeakyReLU'
      d2_run = d2_run * sc + p2;
      l_p2[li] = p2;
    }
    if (e_loc == 0) l_sc[h] = sc;
    wave_lds_fence();
    // row phase: lane = float4 column slots; the chunk is summed on its own first
    float4 part[NV], part2[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      part[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      part2[j] = part[j];
    }
    const int cnt = min(epc, end - c0);
    int t = rep;
    for (; t + (kU - 1) * ES < cnt; t += kU * ES) {
      int uu[kU];
      float4 row[kU][NV];
#pragma unroll
      for (int q = 0; q < kU; ++q) {
        uu[q] = l_idx[t + q * ES];
        if (L == 64) uu[q] = __builtin_amdgcn_readfirstlane(uu[q]);
      }
#pragma unroll
      for (int q = 0; q < kU; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) row[q][j] = ld4(z + (int64_t)uu[q] * HF + 4 * (cl + j * L));
#pragma unroll
      for (int q = 0; q < kU; ++q)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) {
            const int pi = ((t + q * ES) << dm.log2Hp) + hs[j];
            fma4(part[j], l_p[pi], row[q][j]);
            if (WT) fma4(part2[j], l_p2[pi], row[q][j]);
          }
    }
    for (; t < cnt; t += ES) {
      int uu = l_idx[t];
      if (L == 64) uu = __builtin_amdgcn_readfirstlane(uu);
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (slot_ok[j]) {
          const float4 row1 = ld4(z + (int64_t)uu * HF + 4 * (cl + j * L));
          const int pi = (t << dm.log2Hp) + hs[j];
          fma4(part[j], l_p[pi], row1);
          if (WT) fma4(part2[j], l_p2[pi], row1);
        }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {  // rescale to the new max, add the chunk
      const float scj = l_sc[hs[j]];
      fold4(acc[j], scj, part[j]);
      if (WT) fold4(acc2[j], scj, part2[j]);
    }
    wave_lds_fence();
  }

  if (rr.coop) {
    // groups ran their own online softmax: bring them to the common maximum, then add
    if (e_loc == 0) coop_m[grp * Hp + h] = m_run;
    __syncthreads();
    float m_all = -INFINITY;
    for (int g2 = 0; g2 < GPB; ++g2) m_all = fmaxf(m_all, coop_m[g2 * Hp + h]);
    const float sc_own = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_all);
    float v[NC];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      float mj_all = -INFINITY;
      for (int g2 = 0; g2 < GPB; ++g2) mj_all = fmaxf(mj_all, coop_m[g2 * Hp + hs[j]]);
      const float mj = coop_m[grp * Hp + hs[j]];
      const float scj = (mj == -INFINITY) ? 0.f : __expf(mj - mj_all);
      scale4(acc[j], scj);
      pack4(v + 4 * j, acc[j]);
      if (WT) {
        scale4(acc2[j], scj);
        pack4(v + 4 * NV + 4 * j, acc2[j]);
      }
    }
    v[NC - 2] = d_run * sc_own;
    v[NC - 1] = d2_run * sc_own;
    coop_sum<GL, NC, GPB>(coop_buf, v, grp, li);
    if (grp != 0) return;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      acc[j] = unpack4(v + 4 * j);
      if (WT) acc2[j] = unpack4(v + 4 * NV + 4 * j);
    }
    d_run = v[NC - 2];
    d2_run = v[NC - 1];
    m_run = m_all;
  }
  if (ES > 1) {  // add the replicas' sums; afterwards every replica holds the row's totals
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      for (int off = L; off < GL; off <<= 1) {
        acc[j].x += __shfl_xor(acc[j].x, off, 64);
        acc[j].y += __shfl_xor(acc[j].y, off, 64);
        acc[j].z += __shfl_xor(acc[j].z, off, 64);
        acc[j].w += __shfl_xor(acc[j].w, off, 64);
        if (WT) {
          acc2[j].x += __shfl_xor(acc2[j].x, off, 64);
          acc2[j].y += __shfl_xor(acc2[j].y, off, 64);
          acc2[j].z += __shfl_xor(acc2[j].z, off, 64);
          acc2[j].w += __shfl_xor(acc2[j].w, off, 64);
        }
      }
    }
  }
  // denominators: sum the per-lane partials of each head, then hand them to the column lanes
  float dd = group_sum_from<GL>(d_run, Hp);
  const bool empty = beg == end;
  if (empty) { dd = 1.f; m_run = 0.f; }
  if (e_loc == 0) l_sc[h] = dd;
  wave_lds_fence();
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j] && rep == 0) {
      float inv = 1.f / l_sc[hs[j]];
      scale4(acc[j], inv);
      st4(out + (int64_t)v * HF + 4 * (cl + j * L), acc[j]);
      if (WT) {
        scale4(acc2[j], inv);
        st4(t_out + (int64_t)v * HF + 4 * (cl + j * L), acc2[j]);
      }
    }
  if (WT) {
    const float dd2 = group_sum_from<GL>(d2_run, Hp);
    if (e_loc == 0 && head_ok) sg_out[(int64_t)v * H + h] = empty ? 0.f : dd2 / dd;
  }
  if (e_loc == 0 && head_ok) {
    m_out[(int64_t)v * H + h] = m_run;
    d_out[(int64_t)v * H + h] = dd;
  }
}

// per-head sum of per-slot partials: lane (e_loc == 0, h) adds the slots of head h
template <int L, int NV>
__device__ __forceinline__ float head_sum(const float* red, int h, int F) {
  float s = 0.f;
  const int q0 = h * F / 4, q1 = (h + 1) * F / 4;
  for (int q = q0; q < q1; ++q) s += red[(q / L) * L + (q % L)];  // slot q = (lane q%L, j = q/L)
  return s;
}

// ---- a4: backward, destination side (CSR walk) -----------------------------------
// writes der[v,h], and vstate[v,h] = (er, m, 1/d, D) for the source-side kernel
template <int L, int NV>
__global__ __launch_bounds__(kBlock) void k_gat_bwd_dst(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ z, const float* __restrict__ el,
    const float* __restrict__ er, const float* __restrict__ m_in, const float* __restrict__ d_in,
    const float* __restrict__ out, const float* __restrict__ gout, GatDims dm,
    float* __restrict__ der, float4* __restrict__ vstate) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kBlock / kWave);
  constexpr int NC = 4 * NV + 1;
  __shared__ float lds[GPB * GroupLds<L, NV>::kFloats];
  __shared__ float coop_buf[GPB * L * NC];

  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  float* g_lds = lds + grp * GroupLds<L, NV>::kFloats;
  int* l_idx = reinterpret_cast<int*>(g_lds);
  float* l_p = g_lds + L;
  float* l_sc = g_lds + 3 * L;
  float* l_red = g_lds + 4 * L;

  const int H = dm.H, HF = dm.HF;
  const int Hp = 1 << dm.log2Hp;
  const int epc = L >> dm.log2Hp;
  const int e_loc = li >> dm.log2Hp;
  const int h = li & (Hp - 1);
  const bool head_ok = h < H;

  const int32_t v = order[r];
  const int32_t beg = indptr[v], end = indptr[v + 1];
  float er_vh = 0.f, m_vh = 0.f, invd_vh = 1.f;
  if (head_ok) {
    er_vh = er[(int64_t)v * H + h];
    m_vh = m_in[(int64_t)v * H + h];
    invd_vh = 1.f / d_in[(int64_t)v * H + h];
  }

  int hs[NV];
  bool slot_ok[NV];
  float4 acc[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int col = 4 * (li + j * L);
    slot_ok[j] = col < HF;
    hs[j] = slot_ok[j] ? col / dm.F : 0;
    acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  }

  float sg_run = 0.f;  // partial of sum alpha_e g_e
  for (int32_t c0 = beg + gi * epc; c0 < end; c0 += ngrp * epc) {
    const int32_t e = c0 + e_loc;
    const bool e_ok = e < end;
    const int32_t u = e_ok ? indices[e] : 0;
    float q = 0.f;
    if (e_ok && head_ok) {
      const float raw = el[(int64_t)u * H + h] + er_vh;
      const float alpha = __expf(leaky(raw, dm.slope) - m_vh) * invd_vh;
      q = raw > 0.f ? alpha : dm.slope * alpha;
    }
    sg_run += q;
    if (h == 0) l_idx[e_loc] = u;
    l_p[li] = q;
    wave_lds_fence();
    float4 part[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) part[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int cnt = min(epc, end - c0);
    int t = 0;
    for (; t + kU <= cnt; t += kU) {
      int uu[kU];
      float4 row[kU][NV];
#pragma unroll
      for (int k = 0; k < kU; ++k) {
        uu[k] = l_idx[t + k];
        if (L == 64) uu[k] = __builtin_amdgcn_readfirstlane(uu[k]);
      }
#pragma unroll
      for (int k = 0; k < kU; ++k)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) row[k][j] = ld4(z + (int64_t)uu[k] * HF + 4 * (li + j * L));
#pragma unroll
      for (int k = 0; k < kU; ++k)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) fma4(part[j], l_p[((t + k) << dm.log2Hp) + hs[j]], row[k][j]);
    }
    for (; t < cnt; ++t) {
      int uu = l_idx[t];
      if (L == 64) uu = __builtin_amdgcn_readfirstlane(uu);
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (slot_ok[j])
          fma4(part[j], l_p[(t << dm.log2Hp) + hs[j]], ld4(z + (int64_t)uu * HF + 4 * (li + j * L)));
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) add4(acc[j], part[j]);
    wave_lds_fence();
  }

  if (rr.coop) {
    float v[NC];
#pragma unroll
    for (int j = 0; j < NV; ++j) pack4(v + 4 * j, acc[j]);
    v[NC - 1] = sg_run;
    coop_sum<L, NC, GPB>(coop_buf, v, grp, li);
    if (grp != 0) return;
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = unpack4(v + 4 * j);
    sg_run = v[NC - 1];
  }
  const float sg = group_sum_from<L>(sg_run, Hp);
  // per-slot partial dot products with gout[v], then per-head sums through LDS
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    float p1 = 0.f, pd = 0.f;
    if (slot_ok[j]) {
      const int64_t off = (int64_t)v * HF + 4 * (li + j * L);
      const float4 g4 = ld4(gout + off);
      p1 = dot4(g4, acc[j]);
      pd = dot4(g4, ld4(out + off));
    }
    l_red[j * L + li] = p1;
    l_red[L * NV + j * L + li] = pd;
  }
  wave_lds_fence();
  if (e_loc == 0 && head_ok) {
    const float t1 = head_sum<L, NV>(l_red, h, dm.F);
    const float D = head_sum<L, NV>(l_red + L * NV, h, dm.F);
    der[(int64_t)v * H + h] = t1 - D * sg;
    vstate[(int64_t)v * H + h] = make_float4(er_vh, m_vh, invd_vh, D);
  }
}

// ---- a5: backward, source side (CSC walk, no atomics) ------------------------------
// dz[u] = sum_out alpha_e gout[v] + a_l del[u] + a_r der[u];  writes del[u,h] too
template <int L, int NV, int ES>
__global__ __launch_bounds__(kBlock) void k_gat_bwd_src(
    RowLaunch rl, const int32_t* __restrict__ order_t, const int32_t* __restrict__ indptr_t,
    const int32_t* __restrict__ indices_t, const float* __restrict__ z, const float* __restrict__ el,
    const float4* __restrict__ vstate, const float* __restrict__ der, const float* __restrict__ gout,
    const float* __restrict__ a_l, const float* __restrict__ a_r, GatDims dm,
    float* __restrict__ dz, float* __restrict__ del,
    const float* __restrict__ alpha_t /* nullable: stashed softmax values, CSC order, signed */) {
  // GL = L * ES lanes per row: L column lanes replicated ES times, as in k_gat_fwd
  constexpr int GL = L * ES;
  constexpr int G = kWave / GL;
  constexpr int GPB = G * (kBlock / kWave);
  constexpr int NC = 8 * NV + 1;
  static_assert(GL <= kWave && (ES == 1 || NV == 1), "replicas only for rows of at most 64 float4 slots");
  __shared__ float lds[GPB * GroupLds<GL, NV>::kFloats];
  __shared__ float coop_buf[GPB * GL * NC];

  const int lane = threadIdx.x & 63;
  const int li = lane & (GL - 1);
  const int grp = threadIdx.x / GL;
  const int cl = li & (L - 1);
  const int rep = li / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  float* g_lds = lds + grp * GroupLds<GL, NV>::kFloats;
  int* l_idx = reinterpret_cast<int*>(g_lds);
  float* l_p = g_lds + GL;
  float* l_p2 = g_lds + 2 * GL;
  float* l_sc = g_lds + 3 * GL;
  float* l_red = g_lds + 4 * GL;

  const int H = dm.H, HF = dm.HF;
  const int Hp = 1 << dm.log2Hp;
  const int epc = GL >> dm.log2Hp;
  const int e_loc = li >> dm.log2Hp;
  const int h = li & (Hp - 1);
  const bool head_ok = h < H;

  const int32_t u = order_t[r];
  const int32_t beg = indptr_t[u], end = indptr_t[u + 1];
  const float el_uh = head_ok ? el[(int64_t)u * H + h] : 0.f;

  int hs[NV];
  bool slot_ok[NV];
  float4 acc1[NV], acc2[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int col = 4 * (cl + j * L);
    slot_ok[j] = col < HF;
    hs[j] = slot_ok[j] ? col / dm.F : 0;
    acc1[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    acc2[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  }

  float sd_run = 0.f;  // partial of sum alpha_e g_e D[v,h]
  for (int32_t c0 = beg + gi * epc; c0 < end; c0 += ngrp * epc) {
    const int32_t e = c0 + e_loc;
    const bool e_ok = e < end;
    const int32_t v = e_ok ? indices_t[e] : 0;
    float alpha = 0.f, ag = 0.f;
    if (e_ok && head_ok) {
      const float4 vs = vstate[(int64_t)v * H + h];  // (er, m, 1/d, D)
      if (alpha_t) {  // the "fusion with stashing" arm: nothing per-edge is recomputed
        const float a = alpha_t[(int64_t)e * H + h];
        alpha = fabsf(a);
        ag = signbit(a) ? dm.slope * alpha : alpha;
      } else {
        const float raw = el_uh + vs.x;
        alpha = __expf(leaky(raw, dm.slope) - vs.y) * vs.z;
        ag = raw > 0.f ? alpha : dm.slope * alpha;
      }
      sd_run = fmaf(ag, vs.w, sd_run);
    }
    if (h == 0) l_idx[e_loc] = v;
    l_p[li] = alpha;
    l_p2[li] = ag;
    wave_lds_fence();
    float4 part1[NV], part2[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      part1[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      part2[j] = part1[j];
    }
    const int cnt = min(epc, end - c0);
    int t = rep;
    for (; t + (kU - 1) * ES < cnt; t += kU * ES) {
      int vv[kU];
      float4 row[kU][NV];
#pragma unroll
      for (int k = 0; k < kU; ++k) {
        vv[k] = l_idx[t + k * ES];
        if (L == 64) vv[k] = __builtin_amdgcn_readfirstlane(vv[k]);
      }
#pragma unroll
      for (int k = 0; k < kU; ++k)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) row[k][j] = ld4(gout + (int64_t)vv[k] * HF + 4 * (cl + j * L));
#pragma unroll
      for (int k = 0; k < kU; ++k)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) {
            const int pi = ((t + k * ES) << dm.log2Hp) + hs[j];
            fma4(part1[j], l_p[pi], row[k][j]);
            fma4(part2[j], l_p2[pi], row[k][j]);
          }
    }
    for (; t < cnt; t += ES) {
      int vv = l_idx[t];
      if (L == 64) vv = __builtin_amdgcn_readfirstlane(vv);
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (slot_ok[j]) {
          const float4 row = ld4(gout + (int64_t)vv * HF + 4 * (cl + j * L));
          const int pi = (t << dm.log2Hp) + hs[j];
          fma4(part1[j], l_p[pi], row);
          fma4(part2[j], l_p2[pi], row);
        }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      add4(acc1[j], part1[j]);
      add4(acc2[j], part2[j]);
    }
    wave_lds_fence();
  }

  if (rr.coop) {
    float v[NC];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      pack4(v + 4 * j, acc1[j]);
      pack4(v + 4 * NV + 4 * j, acc2[j]);
    }
    v[NC - 1] = sd_run;
    coop_sum<GL, NC, GPB>(coop_buf, v, grp, li);
    if (grp != 0) return;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      acc1[j] = unpack4(v + 4 * j);
      acc2[j] = unpack4(v + 4 * NV + 4 * j);
    }
    sd_run = v[NC - 1];
  }
  if (ES > 1) {  // add the replicas' sums; afterwards every replica holds the row's totals
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      for (int off = L; off < GL; off <<= 1) {
        acc1[j].x += __shfl_xor(acc1[j].x, off, 64);
        acc1[j].y += __shfl_xor(acc1[j].y, off, 64);
        acc1[j].z += __shfl_xor(acc1[j].z, off, 64);
        acc1[j].w += __shfl_xor(acc1[j].w, off, 64);
        acc2[j].x += __shfl_xor(acc2[j].x, off, 64);
        acc2[j].y += __shfl_xor(acc2[j].y, off, 64);
        acc2[j].z += __shfl_xor(acc2[j].z, off, 64);
        acc2[j].w += __shfl_xor(acc2[j].w, off, 64);
      }
    }
  }
  const float sd = group_sum_from<GL>(sd_run, Hp);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    float p = 0.f;
    if (slot_ok[j]) p = dot4(ld4(z + (int64_t)u * HF + 4 * (cl + j * L)), acc2[j]);
    if (rep == 0) l_red[j * L + cl] = p;   // per-slot partials of <z[u], A2[u]>, read by head_sum
  }
  wave_lds_fence();
  if (e_loc == 0) {
    float dl = 0.f, dr = 0.f;
    if (head_ok) {
      dl = head_sum<L, NV>(l_red, h, dm.F) - sd;
      dr = der[(int64_t)u * H + h];
      del[(int64_t)u * H + h] = dl;
    }
    l_sc[h] = dl;
    l_p[h] = dr;  // reuse as the per-head der broadcast
  }
  wave_lds_fence();
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j] && rep == 0) {
      const int col = 4 * (cl + j * L);
      const float dl = l_sc[hs[j]], dr = l_p[hs[j]];
      float4 o = acc1[j];
      fma4(o, dl, ld4(a_l + col));  // a_l, a_r are [H, F] = HF contiguous floats
      fma4(o, dr, ld4(a_r + col));
      st4(dz + (int64_t)u * HF + col, o);
    }
}

// ---- a6: ga_l[h,f] = sum_u del[u,h] z[u,h,f], ga_r[h,f] = sum_v der[v,h] z[v,h,f] ---
// stage 1: each block reduces a contiguous range of vertices; stage 2 adds the blocks in order.
// Inside a block, HF/4 lanes own the float4 columns of a row and the 256 / (HF/4) row groups
// take the block's rows round-robin; their sums are added in group order (fixed => reproducible).
constexpr int kParamThreads = 256;
__global__ __launch_bounds__(kParamThreads) void k_gat_param_partial(
    int64_t n, int H, int F, int64_t rows_per_block, const float* __restrict__ z,
    const float* __restrict__ del, const float* __restrict__ der, float* __restrict__ partial) {
  __shared__ float4 red[2][kParamThreads];
  const int HF = H * F;
  const int lanes = HF / 4;                      // float4 columns of a row (<= 256)
  const int groups = kParamThreads / lanes;      // row groups in this block (>= 1)
  const int li = threadIdx.x % lanes, grp = threadIdx.x / lanes;
  const int64_t r0 = blockIdx.x * rows_per_block;
  int64_t r1 = r0 + rows_per_block;
  if (r1 > n) r1 = n;
  float4 sl = make_float4(0.f, 0.f, 0.f, 0.f), sr = sl;
  if (grp < groups) {
    const int h = (4 * li) / F;
    for (int64_t r = r0 + grp; r < r1; r += groups) {
      const float4 zz = ld4(z + r * HF + 4 * li);
      fma4(sl, del[r * H + h], zz);
      fma4(sr, der[r * H + h], zz);
    }
  }
  red[0][threadIdx.x] = sl;
  red[1][threadIdx.x] = sr;
  __syncthreads();
  if (threadIdx.x < lanes) {
    float4 tl = red[0][li], tr = red[1][li];
    for (int g = 1; g < groups; ++g) {
      add4(tl, red[0][g * lanes + li]);
      add4(tr, red[1][g * lanes + li]);
    }
    st4(partial + ((int64_t)blockIdx.x * 2 + 0) * HF + 4 * li, tl);
    st4(partial + ((int64_t)blockIdx.x * 2 + 1) * HF + 4 * li, tr);
  }
}

// ---- host side -------------------------------------------------------------------
static int param_blocks(int64_t n) {
  int64_t b = cdiv(n, 64);
  if (b > 1024) b = 1024;
  return b < 1 ? 1 : (int)b;
}

struct GatWs {
  size_t total;
  size_t dz, vstate, der, del, partial, gemm, blk_rows, blk_scal, blk_elt, blk_queue, fwd_gemm, blk_half;
  int split_k, nblk, fwd_split_k;
};

static GatWs gat_ws_layout(const gnn_graph_t* g, int fin, int H, int F) {
  const int64_t n = g->n;
  GatWs w{};
  const int HF = H * F;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += ws_granule(bytes); return o; };
  w.dz = take(sizeof(float) * n * HF);
  w.vstate = take(sizeof(float) * 4 * n * H);
  w.der = take(sizeof(float) * n * H);
  w.del = take(sizeof(float) * n * H);
  w.nblk = param_blocks(n);
  w.partial = take(sizeof(float) * 2 * (size_t)w.nblk * HF);
  w.split_k = gemm_pick_split_k(fin, HF, n);
  w.gemm = take(w.split_k > 1 ? sizeof(float) * (size_t)w.split_k * fin * HF : 0);
  const bool blocked = gat_blocked_applies(g, H, F);
  w.blk_rows = take(blocked ? sizeof(float) * n * HF : 0);  // T, then A2
  w.blk_scal = take(blocked ? sizeof(float) * n * 8 : 0);   // sg, then the slices' shares of del
  w.blk_elt = take(blocked ? sizeof(float) * n * H : 0);    // head-major el
  w.blk_queue = take(blocked ? sizeof(int32_t) * 8 * (size_t)g->nblk : 0);  // row counters of the staged kernels
  // a narrow projection of a mid-sized graph has too few output tiles to fill the chip: split K
  w.fwd_split_k = gemm_pick_split_k(n, HF, fin);
  w.fwd_gemm = take(w.fwd_split_k > 1 ? sizeof(float) * (size_t)w.fwd_split_k * n * HF : 0);
  w.blk_half = take(gat_blocked_half(g, H, F) ? 2 * (size_t)n * HF : 0);  // fp16 copy of the gathered rows
  w.total = off;
  return w;
}

static gnn_status_t check_gat_dims(const gnn_graph_t* g, int fin, int H, int F, const char* who) {
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "%s: graph is null", who);
  GNN_REQUIRE(fin > 0 && H > 0 && F > 0, GNN_ERR_INVALID_ARG, "%s: sizes must be positive", who);
  GNN_REQUIRE(F % 4 == 0, GNN_ERR_UNSUPPORTED, "%s: f = %d is not a multiple of 4", who, F);
  GNN_REQUIRE(H * F <= 1024, GNN_ERR_UNSUPPORTED, "%s: heads*f = %d exceeds 1024", who, H * F);
  GNN_REQUIRE(H <= 64, GNN_ERR_UNSUPPORTED, "%s: heads = %d exceeds 64", who, H);
  GroupShape gs = pick_group(H * F);
  GNN_REQUIRE(next_pow2(H) <= gs.L, GNN_ERR_UNSUPPORTED,
              "%s: %d heads do not fit a %d-lane row group", who, H, gs.L);
  return GNN_OK;
}

template <template <int, int> class Launcher, typename... Args>
static gnn_status_t dispatch_group(GroupShape gs, Args... args) {
  switch (gs.L) {
    case 4: return Launcher<4, 1>::run(args...);
    case 8: return Launcher<8, 1>::run(args...);
    case 16: return Launcher<16, 1>::run(args...);
    case 32: return Launcher<32, 1>::run(args...);
    case 64:
      switch (gs.NV) {
        case 1: return Launcher<64, 1>::run(args...);
        case 2: return Launcher<64, 2>::run(args...);
        case 3: return Launcher<64, 3>::run(args...);
        case 4: return Launcher<64, 4>::run(args...);
      }
  }
  set_error("unsupported row-group shape L=%d NV=%d", gs.L, gs.NV);
  return GNN_ERR_UNSUPPORTED;
}

// Replicas of the column lanes per row group (see k_gat_fwd): doubled while the group still fits
// a wavefront and a chunk would hold fewer than 8 edges; at most 4.
template <int L, int NV>
static int pick_replicas(const GatDims& dm) {
  int es = 1;
  if (NV == 1)
    while (es < 4 && L * es * 2 <= kWave && ((L * es) >> dm.log2Hp) < 8) es *= 2;
  return es;
}

template <int L, int NV>
struct FwdLauncher {
  template <int ES>
  static gnn_status_t launch(const gnn_graph_t* g, const float* z, const float* el, const float* er,
                             GatDims dm, float* out, float* m, float* d, float* t, float* sg,
                             hipStream_t st) {
    if constexpr (L * ES <= kWave && (ES == 1 || NV == 1)) {
      constexpr int GL = L * ES;
      constexpr int GPB = (kWave / GL) * (kBlock / kWave);
      const RowSplit sp = split_rows(g, 0, GL >> dm.log2Hp, GPB);
      // hub rows (one workgroup each) and the rest in one launch
      const unsigned grid = sp.hub_grid + sp.rest_grid;
      const RowLaunch rl{sp.hub.end, g->n};
      if (grid != 0) {
        if (t)
          k_gat_fwd<L, NV, true, ES><<<grid, kBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, z, el,
                                                              er, dm, out, m, d, t, sg);
        else
          k_gat_fwd<L, NV, false, ES><<<grid, kBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, z, el,
                                                               er, dm, out, m, d, nullptr, nullptr);
        GNN_LAUNCH_CHECK();
      }
    }
    return GNN_OK;
  }
  static gnn_status_t run(const gnn_graph_t* g, const float* z, const float* el, const float* er,
                          GatDims dm, float* out, float* m, float* d, float* t, float* sg,
                          hipStream_t st) {
    ProfScope p("gat_fwd_fused", st);
    switch (pick_replicas<L, NV>(dm)) {
      case 4: return launch<4>(g, z, el, er, dm, out, m, d, t, sg, st);
      case 2: return launch<2>(g, z, el, er, dm, out, m, d, t, sg, st);
      default: return launch<1>(g, z, el, er, dm, out, m, d, t, sg, st);
    }
  }
};

// ---- vertex-side closing steps of the backward pass (one row group per vertex) -------
// der[v,h] = <gout[v,h,:], t[v,h,:]> - D[v,h] sg[v,h],  D[v,h] = <gout[v,h,:], out[v,h,:]>,
// vstate[v,h] = (er, m, 1/d, D)
template <int L, int NV>
__global__ __launch_bounds__(kBlock) void k_gat_dst_finish(
    int32_t n_rows, const float* __restrict__ gout, const float* __restrict__ t_in,
    const float* __restrict__ out, const float* __restrict__ sg, const float* __restrict__ er,
    const float* __restrict__ m_in, const float* __restrict__ d_in, GatDims dm, int flags,
    float* __restrict__ der, float4* __restrict__ vstate) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kBlock / kWave);
  // flags: kDstHeadMajor - vstate is [H][n] instead of [n][H]; kDstHalfGout - gout is rounded to
  // fp16 first, as the source-side kernel will see it when it gathers an fp16 copy (D and the
  // per-edge dot products <gout[v], z[u]> then cancel exactly where they should)
  const bool head_major = (flags & kDstHeadMajor) != 0, half_gout = (flags & kDstHalfGout) != 0;
  __shared__ float lds[GPB * 2 * L * NV];
  const int li = threadIdx.x & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t v = (int64_t)blockIdx.x * GPB + grp;
  if (v >= n_rows) return;
  float* l_red = lds + grp * 2 * L * NV;
  const int H = dm.H, HF = dm.HF;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int col = 4 * (li + j * L);
    float p1 = 0.f, pd = 0.f;
    if (col < HF) {
      float4 g4 = ld4(gout + v * HF + col);
      if (half_gout)
        g4 = make_float4(__half2float(__float2half_rn(g4.x)), __half2float(__float2half_rn(g4.y)),
                         __half2float(__float2half_rn(g4.z)), __half2float(__float2half_rn(g4.w)));
      p1 = dot4(g4, ld4(t_in + v * HF + col));
      pd = dot4(g4, ld4(out + v * HF + col));
    }
    l_red[j * L + li] = p1;
    l_red[L * NV + j * L + li] = pd;
  }
  wave_lds_fence();
  if (li < H) {
    const int h = li;
    const float t1 = head_sum<L, NV>(l_red, h, dm.F);
    const float D = head_sum<L, NV>(l_red + L * NV, h, dm.F);
    const int64_t i = v * H + h;
    der[i] = t1 - D * sg[i];
    // head-major ([H][n]) for the column-blocked source kernel, whose XCD slice reads one
    // head only: a block of gathered vertices then spans 16 B per vertex instead of 16*H
    vstate[head_major ? (int64_t)h * n_rows + v : i] = make_float4(er[i], m_in[i], 1.f / d_in[i], D);
  }
}

// del[u,h] = <z[u,h,:], a2[u,h,:]> - sd[u,h];  dz[u,h,:] += a_l[h,:] del[u,h] + a_r[h,:] der[u,h]
template <int L, int NV>
__global__ __launch_bounds__(kBlock) void k_gat_src_finish(
    int32_t n_rows, const float* __restrict__ z, const float* __restrict__ a2,
    const float* __restrict__ sd, const float* __restrict__ der, const float* __restrict__ a_l,
    const float* __restrict__ a_r, GatDims dm, float* __restrict__ dz, float* __restrict__ del) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kBlock / kWave);
  __shared__ float lds[GPB * 3 * L * NV];
  const int li = threadIdx.x & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t u = (int64_t)blockIdx.x * GPB + grp;
  if (u >= n_rows) return;
  float* l_red = lds + grp * 3 * L * NV;
  float* l_dl = l_red + L * NV;
  float* l_dr = l_red + 2 * L * NV;
  const int H = dm.H, HF = dm.HF;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int col = 4 * (li + j * L);
    float p = 0.f;
    if (col < HF) p = dot4(ld4(z + u * HF + col), ld4(a2 + u * HF + col));
    l_red[j * L + li] = p;
  }
  wave_lds_fence();
  if (li < H) {
    const int64_t i = u * H + li;
    const float dl = head_sum<L, NV>(l_red, li, dm.F) - sd[i];
    del[i] = dl;
    l_dl[li] = dl;
    l_dr[li] = der[i];
  }
  wave_lds_fence();
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int col = 4 * (li + j * L);
    if (col < HF) {
      const int h = col / dm.F;
      float4 o = ld4(dz + u * HF + col);
      fma4(o, l_dl[h], ld4(a_l + col));
      fma4(o, l_dr[h], ld4(a_r + col));
      st4(dz + u * HF + col, o);
    }
  }
}

template <int L, int NV>
struct DstFinishLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* gout, const float* t, const float* out,
                          const float* sg, const float* er, const float* m, const float* d, GatDims dm,
                          int head_major, float* der, float4* vstate, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kBlock / kWave);
    ProfScope p("gat_bwd_dst_finish", st);
    k_gat_dst_finish<L, NV><<<(unsigned)cdiv(g->n, GPB), kBlock, 0, st>>>(g->n, gout, t, out, sg, er, m,
                                                                         d, dm, head_major, der, vstate);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};

template <int L, int NV>
struct SrcFinishLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* z, const float* a2, const float* sd,
                          const float* der, const float* a_l, const float* a_r, GatDims dm, float* dz,
                          float* del, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kBlock / kWave);
    ProfScope p("gat_bwd_src_finish", st);
    k_gat_src_finish<L, NV><<<(unsigned)cdiv(g->n, GPB), kBlock, 0, st>>>(g->n, z, a2, sd, der, a_l,
                                                                         a_r, dm, dz, del);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};



template <int L, int NV>
struct BwdDstLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* z, const float* el, const float* er,
                          const float* m, const float* d, const float* out, const float* gout,
                          GatDims dm, float* der, float4* vstate, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kBlock / kWave);
    ProfScope p("gat_bwd_dst", st);
    const RowSplit sp = split_rows(g, 0, L >> dm.log2Hp, GPB);
    // hub rows (one workgroup each) and the rest in one launch
    const unsigned grid = sp.hub_grid + sp.rest_grid;
    const RowLaunch rl{sp.hub.end, g->n};
    if (grid != 0) {
      k_gat_bwd_dst<L, NV><<<grid, kBlock, 0, st>>>(rl, g->order[0], g->indptr, g->indices, z, el, er, m, d,
                                                    out, gout, dm, der, vstate);
      GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
  }
};

template <int L, int NV>
struct BwdSrcLauncher {
  template <int ES>
  static gnn_status_t launch(const gnn_graph_t* g, const float* z, const float* el, const float4* vstate,
                             const float* der, const float* gout, const float* a_l, const float* a_r,
                             GatDims dm, float* dz, float* del, const float* alpha_t, hipStream_t st) {
    if constexpr (L * ES <= kWave && (ES == 1 || NV == 1)) {
      constexpr int GL = L * ES;
      constexpr int GPB = (kWave / GL) * (kBlock / kWave);
      const RowSplit sp = split_rows(g, 1, GL >> dm.log2Hp, GPB);
      // hub rows (one workgroup each) and the rest in one launch
      const unsigned grid = sp.hub_grid + sp.rest_grid;
      const RowLaunch rl{sp.hub.end, g->n};
      if (grid != 0) {
        k_gat_bwd_src<L, NV, ES><<<grid, kBlock, 0, st>>>(rl, g->order[1], g->indptr_t, g->indices_t, z, el,
                                                          vstate, der, gout, a_l, a_r, dm, dz, del, alpha_t);
        GNN_LAUNCH_CHECK();
      }
    }
    return GNN_OK;
  }
  static gnn_status_t run(const gnn_graph_t* g, const float* z, const float* el, const float4* vstate,
                          const float* der, const float* gout, const float* a_l, const float* a_r,
                          GatDims dm, float* dz, float* del, const float* alpha_t, hipStream_t st) {
    ProfScope p("gat_bwd_src", st);
    switch (pick_replicas<L, NV>(dm)) {
      case 4: return launch<4>(g, z, el, vstate, der, gout, a_l, a_r, dm, dz, del, alpha_t, st);
      case 2: return launch<2>(g, z, el, vstate, der, gout, a_l, a_r, dm, dz, del, alpha_t, st);
      default: return launch<1>(g, z, el, vstate, der, gout, a_l, a_r, dm, dz, del, alpha_t, st);
    }
  }
};

gnn_status_t gat_dst_finish(const gnn_graph_t* g, GatDims dm, const float* gout, const float* t,
                            const float* out, const float* sg, const float* er, const float* m,
                            const float* d, int head_major, float* der, float4* vstate,
                            hipStream_t st) {
  return dispatch_group<DstFinishLauncher>(pick_group(dm.HF), g, gout, t, out, sg, er, m, d, dm,
                                           head_major, der, vstate, st);
}
gnn_status_t gat_src_finish(const gnn_graph_t* g, GatDims dm, const float* z, const float* a2,
                            const float* sd, const float* der, const float* a_l, const float* a_r,
                            float* dz, float* del, hipStream_t st) {
  return dispatch_group<SrcFinishLauncher>(pick_group(dm.HF), g, z, a2, sd, der, a_l, a_r, dm, dz, del,
                                           st);
}


// ---- the per-edge stash of the "fusion with stashing" arm (Sec. 7.3, recomputation study) ----
// alpha_t[p, h] for CSC position p: the softmax value of that edge, carrying the sign of the
// raw score (the only other per-edge fact the backward pass needs: LeakyReLU' is 1 or slope).
// One thread per (position, head); the edge's source comes from the plan's position -> CSR
// edge id table.
__global__ void k_gat_stash_alpha(int64_t count, int H, float slope, const int32_t* __restrict__ indices,
                                  const int32_t* __restrict__ indices_t, const int32_t* __restrict__ eid_t,
                                  const float* __restrict__ el, const float* __restrict__ er,
                                  const float* __restrict__ m, const float* __restrict__ d,
                                  float* __restrict__ alpha_t) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= count) return;
  const int64_t p = i / H;
  const int h = (int)(i - p * H);
  const int32_t v = indices_t[p];
  const int32_t u = indices[eid_t[p]];
  const float raw = el[(int64_t)u * H + h] + er[(int64_t)v * H + h];
  const float a = __expf(leaky(raw, slope) - m[(int64_t)v * H + h]) / d[(int64_t)v * H + h];
  alpha_t[i] = raw > 0.f ? a : -a;
}

static gnn_status_t gat_bwd_impl(const char* who, const gnn_graph_t* g, int fin, int heads, int f, float slope,
                                 const float* x, const float* w, const float* a_l, const float* a_r,
                                 const float* z, const float* el, const float* er, const float* m,
                                 const float* d, const float* out, const float* t, const float* sg,
                                 const float* alpha_t, const float* gout, float* gx, float* gw, float* ga_l,
                                 float* ga_r, void* ws, size_t ws_bytes, void* stream);

}  // namespace gnn

using namespace gnn;

extern "C" size_t gnn_gat_workspace_bytes(const gnn_graph_t* g, int fin, int heads, int f) {
  if (!g || fin <= 0 || heads <= 0 || f <= 0) return 0;
  return gat_ws_layout(g, fin, heads, f).total;
}

extern "C" gnn_status_t gnn_gat_fwd(const gnn_graph_t* g, int fin, int heads, int f, float slope,
                                    const float* x, const float* w, const float* a_l, const float* a_r,
                                    float* z, float* el, float* er, float* m, float* d, float* out,
                                    float* t, float* sg, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(check_gat_dims(g, fin, heads, f, "gnn_gat_fwd"));
  GNN_REQUIRE((t == nullptr) == (sg == nullptr), GNN_ERR_INVALID_ARG,
              "gnn_gat_fwd: t and sg must be given together");
  GNN_REQUIRE(t == nullptr || aligned16(t), GNN_ERR_INVALID_ARG, "gnn_gat_fwd: t must be 16-byte aligned");
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && a_l && a_r && z && el && er && m && d && out, GNN_ERR_INVALID_ARG,
              "gnn_gat_fwd: null pointer");
  GNN_REQUIRE(aligned16(z) && aligned16(out) && aligned16(a_l) && aligned16(a_r), GNN_ERR_INVALID_ARG,
              "gnn_gat_fwd: z, out, a_l, a_r must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int HF = heads * f;
  const int64_t n = g->n;
  // a1: projection before propagation (split over K when the workspace offers room for the parts)
  const GatWs L = gat_ws_layout(g, fin, heads, f);
  const bool have_ws = ws != nullptr && ws_bytes >= L.total && aligned16(ws);
  bool halves_done = false;
  if (have_ws && L.fwd_split_k > 1) {
    GNN_TRY(gemm_f32(n, HF, fin, x, fin, false, w, HF, false, z, HF, L.fwd_split_k,
                     reinterpret_cast<float*>(static_cast<char*>(ws) + L.fwd_gemm), st));
  } else if (gemm_attn_epilogue_ok(heads, f) && fin < (1 << 24)) {
    // a1 + a2: the attention halves come out of the projection's accumulators
    GNN_TRY(gemm_f32_attn(n, heads, f, fin, x, w, a_l, a_r, z, el, er, st));
    halves_done = true;
  } else {
    GNN_TRY(gemm_f32(n, HF, fin, x, fin, false, w, HF, false, z, HF, 1, nullptr, st));
  }
  // a2: attention halves (shapes the epilogue does not cover, and split-K projections)
  if (!halves_done) {
    ProfScope p("gat_attn_halves", st);
    k_gat_attn_halves<<<(unsigned)cdiv(n * heads, 256), 256, 0, st>>>(n, heads, f, z, a_l, a_r, el, er);
    GNN_LAUNCH_CHECK();
  }
  // a3: fused score -> softmax -> aggregate
  // The column-blocked kernels need scratch (a head-major copy of el, row counters, and the
  // running softmax statistics, which borrow the dz area the backward call uses later: 128 of
  // its >= 512 bytes per vertex); without a workspace the single-launch kernels run.
  // Rows of 512 bytes and more take them (two 256-byte slices at 512 bytes; measured at Reddit
  // scale, 1 x 128: 7.9 ms against 8.5 ms for the single-launch forward kernel), and single-head
  // rows of up to 256 bytes as one slice of the persistent kernels.
  if (gat_blocked_applies(g, heads, f) && have_ws) {
    char* base = static_cast<char*>(ws);
    return gat_blocked_fwd(g, make_dims(heads, f, slope), z, el, er, m, d, out, t, sg,
                           reinterpret_cast<float*>(base + L.blk_elt),
                           reinterpret_cast<int32_t*>(base + L.blk_queue),
                           reinterpret_cast<float4*>(base + L.dz),
                           gat_blocked_half(g, heads, f) ? base + L.blk_half : nullptr, st);
  }
  return dispatch_group<FwdLauncher>(pick_group(HF), g, (const float*)z, (const float*)el,
                                     (const float*)er, make_dims(heads, f, slope), out, m, d, t, sg, st);
}

extern "C" gnn_status_t gnn_gat_bwd(const gnn_graph_t* g, int fin, int heads, int f, float slope,
                                    const float* x, const float* w, const float* a_l, const float* a_r,
                                    const float* z, const float* el, const float* er, const float* m,
                                    const float* d, const float* out, const float* t, const float* sg,
                                    const float* gout, float* gx, float* gw, float* ga_l, float* ga_r,
                                    void* ws, size_t ws_bytes, void* stream) {
  return gat_bwd_impl("gnn_gat_bwd", g, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t, sg,
                      nullptr, gout, gx, gw, ga_l, ga_r, ws, ws_bytes, stream);
}

// ---- backward call for callers that cannot allocate ---------------------------------
// The scratch of gnn_gat_bwd (dz, the destination-side table, der, del, the partial sums of
// the parameter gradients) lives in a device array of the library's code object instead of a
// caller-provided workspace.  In host code the array's name is only a handle for the runtime:
// its device address is looked up once per device and that pointer is what reaches the kernels.
static __device__ __align__(256) unsigned char scratch[GNN_NOALLOC_SCRATCH_BYTES];

namespace gnn {
constexpr int kMaxScratchDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxScratchDevices];  // per device, null until looked up

static gnn_status_t noalloc_scratch(void** out) {
  int dev = -1;
  GNN_HIP(hipGetDevice(&dev));
  GNN_REQUIRE(dev >= 0 && dev < kMaxScratchDevices, GNN_ERR_UNSUPPORTED,
              "gnn_gat_bwd_noalloc: device index %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    GNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));  // this device's copy of the array
    GNN_REQUIRE(p != nullptr, GNN_ERR_HIP, "gnn_gat_bwd_noalloc: no device address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return GNN_OK;
}
}  // namespace gnn

extern "C" gnn_status_t gnn_gat_bwd_noalloc(const gnn_graph_t* g, int fin, int heads, int f, float slope,
                                            const float* x, const float* w, const float* a_l,
                                            const float* a_r, const float* z, const float* el,
                                            const float* er, const float* m, const float* d, const float* out,
                                            const float* t, const float* sg, const float* gout, float* gx,
                                            float* gw, float* ga_l, float* ga_r, void* stream) {
  clear_error();
  GNN_TRY(check_gat_dims(g, fin, heads, f, "gnn_gat_bwd_noalloc"));
  const size_t need = gat_ws_layout(g, fin, heads, f).total;
  GNN_REQUIRE(need <= (size_t)GNN_NOALLOC_SCRATCH_BYTES, GNN_ERR_WORKSPACE,
              "gnn_gat_bwd_noalloc: this graph and these widths need %zu bytes of scratch, the built-in "
              "array holds %zu; use gnn_gat_bwd with a workspace", need, (size_t)GNN_NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  GNN_TRY(noalloc_scratch(&ws));
  // Every kernel of the backward pass writes its part of the scratch before reading it (the row
  // counters of the column-blocked kernels are reset by a fill kernel), so what an earlier call
  // left behind is never read.
  return gat_bwd_impl("gnn_gat_bwd_noalloc", g, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t, sg,
                      nullptr, gout, gx, gw, ga_l, ga_r, ws, (size_t)GNN_NOALLOC_SCRATCH_BYTES, stream);
}

extern "C" int gnn_gat_stash_layout(const gnn_graph_t* g, int heads, int f) {
  return g != nullptr && heads > 0 && f > 0 && gat_blocked_applies(g, heads, f) ? 1 : 0;
}

extern "C" gnn_status_t gnn_gat_stash_alpha(const gnn_graph_t* g, int heads, int f, float slope, const float* el,
                                            const float* er, const float* m, const float* d, float* alpha_t,
                                            void* stream) {
  clear_error();
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "gnn_gat_stash_alpha: graph is null");
  GNN_REQUIRE(heads > 0 && heads <= 64 && f > 0, GNN_ERR_INVALID_ARG, "gnn_gat_stash_alpha: sizes out of range");
  if (g->nnz == 0) return GNN_OK;
  GNN_REQUIRE(el && er && m && d && alpha_t, GNN_ERR_INVALID_ARG, "gnn_gat_stash_alpha: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (gat_blocked_applies(g, heads, f)) return gat_blocked_stash_alpha(g, heads, slope, el, er, m, d, alpha_t, st);
  ProfScope p("gat_stash_alpha", st);
  const int64_t count = g->nnz * heads;
  k_gat_stash_alpha<<<(unsigned)cdiv(count, 256), 256, 0, st>>>(count, heads, slope, g->indices, g->indices_t,
                                                               g->eid_t, el, er, m, d, alpha_t);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

extern "C" gnn_status_t gnn_gat_bwd_stashed(const gnn_graph_t* g, int fin, int heads, int f, float slope,
                                            const float* x, const float* w, const float* a_l,
                                            const float* a_r, const float* z, const float* el,
                                            const float* er, const float* m, const float* d, const float* out,
                                            const float* t, const float* sg, const float* alpha_t,
                                            const float* gout, float* gx, float* gw, float* ga_l, float* ga_r,
                                            void* ws, size_t ws_bytes, void* stream) {
  if (g != nullptr && g->nnz != 0 && alpha_t == nullptr) {
    clear_error();
    set_error("gnn_gat_bwd_stashed: alpha_t is null");
    return GNN_ERR_INVALID_ARG;
  }
  return gat_bwd_impl("gnn_gat_bwd_stashed", g, fin, heads, f, slope, x, w, a_l, a_r, z, el, er, m, d, out, t, sg,
                      alpha_t, gout, gx, gw, ga_l, ga_r, ws, ws_bytes, stream);
}

namespace gnn {
static gnn_status_t gat_bwd_impl(const char* who, const gnn_graph_t* g, int fin, int heads, int f, float slope,
                                 const float* x, const float* w, const float* a_l, const float* a_r,
                                 const float* z, const float* el, const float* er, const float* m,
                                 const float* d, const float* out, const float* t, const float* sg,
                                 const float* alpha_t, const float* gout, float* gx, float* gw, float* ga_l,
                                 float* ga_r, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(check_gat_dims(g, fin, heads, f, who));
  GNN_REQUIRE((t == nullptr) == (sg == nullptr), GNN_ERR_INVALID_ARG,
              "%s: t and sg must be given together", who);
  GNN_REQUIRE(t == nullptr || aligned16(t), GNN_ERR_INVALID_ARG, "%s: t must be 16-byte aligned", who);
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && a_l && a_r && z && el && er && m && d && out && gout && gw && ga_l && ga_r,
              GNN_ERR_INVALID_ARG, "%s: null pointer", who);
  GNN_REQUIRE(aligned16(z) && aligned16(out) && aligned16(gout) && aligned16(a_l) && aligned16(a_r),
              GNN_ERR_INVALID_ARG, "%s: z, out, gout, a_l, a_r must be 16-byte aligned", who);
  const int64_t n = g->n;
  const int HF = heads * f;
  const GatWs L = gat_ws_layout(g, fin, heads, f);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, L.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", who);
  char* base = static_cast<char*>(ws);
  float* dz = reinterpret_cast<float*>(base + L.dz);
  float4* vstate = reinterpret_cast<float4*>(base + L.vstate);
  float* der = reinterpret_cast<float*>(base + L.der);
  float* del = reinterpret_cast<float*>(base + L.del);
  float* partial = reinterpret_cast<float*>(base + L.partial);
  float* gemm_part = reinterpret_cast<float*>(base + L.gemm);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const GatDims dm = make_dims(heads, f, slope);
  const GroupShape gs = pick_group(HF);

  // the per-edge stash is laid out for whichever source-side kernel this graph and shape take
  const bool blocked = gat_blocked_applies(g, heads, f);
  const int dst_flags = (blocked ? kDstHeadMajor : 0) | (blocked && gat_blocked_half(g, heads, f) ? kDstHalfGout : 0);
  // a4: destination side.  With t and sg stashed by the forward call it is a vertex pass;
  // without them the sums are recomputed over the in-edges.
  if (t) {
    GNN_TRY(gat_dst_finish(g, dm, gout, t, out, sg, er, m, d, dst_flags, der, vstate, st));
  } else if (blocked) {
    float* rows_buf = reinterpret_cast<float*>(base + L.blk_rows);
    float* scal_buf = reinterpret_cast<float*>(base + L.blk_scal);
    float* el_t = reinterpret_cast<float*>(base + L.blk_elt);
    int32_t* queue = reinterpret_cast<int32_t*>(base + L.blk_queue);
    GNN_TRY(gat_blocked_bwd_dst(g, dm, z, el, er, m, d, out, gout, der, vstate, rows_buf, scal_buf, el_t,
                                queue, st));
  } else {
    GNN_TRY(dispatch_group<BwdDstLauncher>(gs, g, z, el, er, m, d, out, gout, dm, der, vstate, st));
  }
  if (blocked) {
    float* scal_buf = reinterpret_cast<float*>(base + L.blk_scal);
    GNN_TRY(gat_blocked_bwd_src(g, dm, z, el, vstate, der, gout, a_l, a_r, dz, del, scal_buf,
                                gat_blocked_half(g, heads, f) ? base + L.blk_half : nullptr, st, alpha_t));
  } else {
    // a5: source side
    GNN_TRY(dispatch_group<BwdSrcLauncher>(gs, g, z, el, (const float4*)vstate, (const float*)der,
                                           gout, a_l, a_r, dm, dz, del, alpha_t, st));
  }
  // a6: parameter gradients
  {
    ProfScope p("gat_param_grad", st);
    const int64_t rpb = cdiv(n, L.nblk);
    k_gat_param_partial<<<L.nblk, kParamThreads, 0, st>>>(n, heads, f, rpb, z, del, der, partial);
    GNN_LAUNCH_CHECK();
    // partial is [nblk][2][HF]: the l and the r halves summed by one launch, block order fixed
    GNN_TRY(sum_partials_pair(HF, L.nblk, partial, ga_l, ga_r, st));
  }
  // gw = x^T dz   (x read k-major: row index of x is the contraction index)
  GNN_TRY(gemm_f32(fin, HF, n, x, fin, true, dz, HF, false, gw, HF, L.split_k, gemm_part, st));
  // gx = dz w^T   (w read with its row index as the output column)
  if (gx) GNN_TRY(gemm_f32(n, fin, HF, dz, HF, false, w, HF, true, gx, fin, 1, nullptr, st));
  return GNN_OK;
}
}  // namespace gnn
