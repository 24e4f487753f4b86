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
template <int L, int NV>
__global__ __launch_bounds__(kGcnBlock) void k_rowsum(
    RowLaunch rl, const int32_t* __restrict__ order, const int32_t* __restrict__ ptr,
    const int32_t* __restrict__ cols, const float* __restrict__ feat, int F,
    const float* __restrict__ scale, float* __restrict__ out) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kGcnBlock / kWave);
  constexpr int NC = 4 * NV;
  constexpr int U = 4;
  __shared__ int lds[GPB * L];
  __shared__ float coop_buf[GPB * L * NC];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  int64_t r;
  int gi, ngrp;
  RowRange rr;
  if (!pick_row<GPB>(rl, grp, rr, r, gi, ngrp)) return;
  int* l_idx = lds + grp * L;
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
    wave_lds_fence();
    float4 part[NV];  // this chunk's share (two-level summation)
#pragma unroll
    for (int j = 0; j < NV; ++j) part[j] = make_float4(0.f, 0.f, 0.f, 0.f);
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
        float4 rowv[U];
#pragma unroll
        for (int t = 0; t < U; ++t) rowv[t] = ld4(feat + (int64_t)uu[t] * F + 4 * (li + j * L));
#pragma unroll
        for (int t = 0; t < U; ++t) fma4(part[j], t0 + t < cnt ? 1.f : 0.f, rowv[t]);  // padding adds 0 * row 0
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
  const float s = scale[v];
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j])
      st4(out + (int64_t)v * F + 4 * (li + j * L), make_float4(s * acc[j].x, s * acc[j].y, s * acc[j].z, s * acc[j].w));
}

// ---- one column block of the same sum (running sums in acc_buf) -----------------------
template <int SL>
__global__ __launch_bounds__(kGcnBlock) void k_rowsum_blk(
    int32_t n_rows, const int32_t* __restrict__ order, const int2* __restrict__ bseg_b,
    const int32_t* __restrict__ bcol, const float* __restrict__ feat, int32_t col_begin, int F,
    int first, float* __restrict__ acc_buf) {
  constexpr int GPB = kGcnBlock / SL;
  constexpr int R = kGcnRows;
  constexpr int U = SL < 8 ? 4 : 8;
  constexpr int GS = SL + 4 * R;  // LDS ints per group: idx | row, beg, end, pad
  static_assert(SL >= R, "one lane per pipelined row loads its metadata");
  __shared__ __align__(16) int lds[GPB * GS];
  const int lane = threadIdx.x & 63;
  const int li = lane & (SL - 1);
  const int grp = threadIdx.x / SL;
  const int slice = blockIdx.x % kGcnSlices;
  const int64_t r0 = ((int64_t)(blockIdx.x / kGcnSlices) * GPB + grp) * R;
  if (r0 >= n_rows) return;
  int* l_idx = lds + grp * GS;
  int* l_row = l_idx + SL;
  int* l_beg = l_row + R;
  int* l_end = l_row + 2 * R;
  const int col = slice * 4 * SL + 4 * li;

  if (li < R) {
    const int64_t r = r0 + li;
    int32_t row = -1;
    int2 seg = make_int2(0, 0);
    if (r < n_rows) {
      row = order[r];
      seg = bseg_b[r];
      if (!first && seg.x == seg.y) row = -1;  // nothing to add to this row in this block
    }
    l_row[li] = row;
    l_beg[li] = seg.x;
    l_end[li] = seg.y;
  }
  wave_lds_fence();

  struct Row {
    int32_t row, beg, end, c_first;
    float4 acc;
  };
  auto fetch = [&](int k, Row& s) {
    s.row = l_row[k];
    s.beg = l_beg[k];
    s.end = l_end[k];
    s.c_first = col_begin;
    s.acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s.row < 0) return;
    if (s.beg + li < s.end) s.c_first = bcol[s.beg + li];
    if (!first) s.acc = ld4_stream(acc_buf + (int64_t)s.row * F + col);
  };

  Row cur, nxt;
  fetch(0, cur);
  for (int k = 0; k < R; ++k) {
    if (k + 1 < R) fetch(k + 1, nxt);
    if (cur.row >= 0) {
      const int32_t end = cur.end;
      float4 acc = cur.acc;
      int32_t c_next = cur.c_first;
      for (int32_t c0 = cur.beg; c0 < end; c0 += SL) {
        // lanes past the end point at the block's first vertex (valid, cache-resident) and
        // their rows are multiplied by 0
        const int32_t c = c0 + li < end ? c_next : col_begin;
        if (c0 + SL + li < end) c_next = bcol[c0 + SL + li];
        l_idx[li] = c;
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
          for (int t = 0; t < U; ++t) rowv[t] = ld4(feat + (int64_t)idv[t] * F + col);
#pragma unroll
          for (int t = 0; t < U; ++t) fma4(part, t0 + t < cnt ? 1.f : 0.f, rowv[t]);
        }
        add4(acc, part);
        wave_lds_fence();
      }
      st4_stream(acc_buf + (int64_t)cur.row * F + col, acc);
    }
    cur = nxt;
  }
}

static bool gcn_blocked_applies(const gnn_graph_t* g, int F) {
  if (g->nblk <= 1 || config_get(kCfgForceSimple)) return false;
  if (F % (4 * kGcnSlices) != 0) return false;
  const int SL = F / (4 * kGcnSlices);
  return SL == 4 || SL == 8 || SL == 16 || SL == 32;
}

template <int SL>
static gnn_status_t launch_rowsum_blocks(const gnn_graph_t* g, int side, const char* name, const float* feat,
                                         int F, float* acc, hipStream_t st) {
  const int rows_per_wg = (kGcnBlock / SL) * kGcnRows;
  const unsigned grid = (unsigned)(cdiv(g->n, rows_per_wg) * kGcnSlices);
  for (int b = 0; b < g->nblk; ++b) {
    const int2* bseg_b = reinterpret_cast<const int2*>(g->bseg[side]) + (int64_t)b * g->n;
    ProfScope p(name, st);  // one timed bracket per launch
    k_rowsum_blk<SL><<<grid, kGcnBlock, 0, st>>>(g->n, g->order[side], bseg_b, g->bcol[side], feat,
                                                b * g->block_cols, F, b == 0, acc);
    GNN_LAUNCH_CHECK();
  }
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

// out[row,:] = scale[row] * sum of feat over the row's neighbours on `side` (0: in-edges, 1: out-edges)
static gnn_status_t gcn_aggregate(const gnn_graph_t* g, int side, const char* name, const float* feat, int F,
                                  const float* scale, float* out, hipStream_t st) {
  if (gcn_blocked_applies(g, F)) {
    switch (F / (4 * kGcnSlices)) {
      case 4: GNN_TRY(launch_rowsum_blocks<4>(g, side, name, feat, F, out, st)); break;
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
  const GroupShape gs = pick_group(F);
  switch (gs.L) {
    case 4: return RowsumLauncher<4, 1>::run(g, side, name, feat, F, scale, out, st);
    case 8: return RowsumLauncher<8, 1>::run(g, side, name, feat, F, scale, out, st);
    case 16: return RowsumLauncher<16, 1>::run(g, side, name, feat, F, scale, out, st);
    case 32: return RowsumLauncher<32, 1>::run(g, side, name, feat, F, scale, out, st);
    case 64:
      switch (gs.NV) {
        case 1: return RowsumLauncher<64, 1>::run(g, side, name, feat, F, scale, out, st);
        case 2: return RowsumLauncher<64, 2>::run(g, side, name, feat, F, scale, out, st);
        case 3: return RowsumLauncher<64, 3>::run(g, side, name, feat, F, scale, out, st);
        case 4: return RowsumLauncher<64, 4>::run(g, side, name, feat, F, scale, out, st);
      }
  }
  set_error("unsupported row-group shape L=%d NV=%d", gs.L, gs.NV);
  return GNN_ERR_UNSUPPORTED;
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
