// EdgeConv layer (App. A.2 "EdgeConv") in its reorganized form (Sec. 4):
//   Theta (h_u - h_v) + Phi h_v = (x Theta)[u] + (x (Phi - Theta))[v] = P[u] + Q[v]
// so the linear layers run once per vertex as ONE product x [Theta | Phi - Theta],
// and the fused kernel is a gather-max over P with the arg-max positions as the
// only saved state (Sec. 7.2 "EdgeConv": O(|V|) indices, nothing per edge).
//
// Backward: the gradient of reduce_max goes to the winning in-edge only.  The
// source-side sum  dP[u,j] = sum over out-edges e = (u -> v) [argmax[v,j] == e] gout[v,j]
// walks the CSC transpose (no atomics); dQ = gout.  Then
//   [gTheta' | gQ'] = x^T [dP | dQ],  gTheta = gTheta' - gQ',  gPhi = gQ',
//   gx = [dP | dQ] [Theta | Phi - Theta]^T.
#include "common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kEcBlock = 256;

// wcat[i, :] = [theta[i, :] | phi[i, :] - theta[i, :]]
__global__ void k_ec_concat_weights(int fin, int fout, const float* __restrict__ theta,
                                    const float* __restrict__ phi, float* __restrict__ wcat) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= fin * fout) return;
  int r = i / fout, c = i % fout;
  float t = theta[i];
  wcat[(int64_t)r * 2 * fout + c] = t;
  wcat[(int64_t)r * 2 * fout + fout + c] = phi[i] - t;
}

// gtheta = gcat[:, :fout] - gcat[:, fout:], gphi = gcat[:, fout:]
__global__ void k_ec_split_weight_grads(int fin, int fout, const float* __restrict__ gcat,
                                        float* __restrict__ gtheta, float* __restrict__ gphi) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= fin * fout) return;
  int r = i / fout, c = i % fout;
  float gp = gcat[(int64_t)r * 2 * fout + c];
  float gq = gcat[(int64_t)r * 2 * fout + fout + c];
  gtheta[i] = gp - gq;
  gphi[i] = gq;
}

// ---- a7: fused gather-max ------------------------------------------------------------
template <int L, int NV>
__global__ __launch_bounds__(kEcBlock) void k_edgeconv_fwd(
    int32_t n_rows, const int32_t* __restrict__ order, const int32_t* __restrict__ indptr,
    const int32_t* __restrict__ indices, const float* __restrict__ pq, int F,
    float* __restrict__ out, int32_t* __restrict__ argmax) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kEcBlock / kWave);
  __shared__ int lds[GPB * L];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  // order == nullptr: vertex order in XCD-contiguous ranges (near-uniform degrees)
  const int64_t r = order ? (int64_t)blockIdx.x * GPB + grp : xcd_contiguous_row(blockIdx.x, gridDim.x, GPB, grp);
  if (r >= n_rows) return;
  int* l_idx = lds + grp * L;
  const int32_t v = order ? order[r] : (int32_t)r;
  const int32_t beg = indptr[v], end = indptr[v + 1];
  const int ld = 2 * F;

  bool slot_ok[NV];
  float4 best[NV];
  int4 arg[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    slot_ok[j] = 4 * (li + j * L) < F;
    best[j] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    arg[j] = make_int4(-1, -1, -1, -1);
  }
  for (int32_t c0 = beg; c0 < end; c0 += L) {
    const int32_t e = c0 + li;
    l_idx[li] = e < end ? indices[e] : 0;
    wave_lds_fence();
    const int cnt = min(L, end - c0);
    int t = 0;
    for (; t + 4 <= cnt; t += 4) {
      float4 row[4][NV];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        int u = l_idx[t + k];
        if (L == 64) u = __builtin_amdgcn_readfirstlane(u);
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) row[k][j] = ld4(pq + (int64_t)u * ld + 4 * (li + j * L));
      }
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (slot_ok[j]) {
            const int32_t ee = c0 + t + k;  // strict '>' keeps the earliest edge on a tie
            if (row[k][j].x > best[j].x) { best[j].x = row[k][j].x; arg[j].x = ee; }
            if (row[k][j].y > best[j].y) { best[j].y = row[k][j].y; arg[j].y = ee; }
            if (row[k][j].z > best[j].z) { best[j].z = row[k][j].z; arg[j].z = ee; }
            if (row[k][j].w > best[j].w) { best[j].w = row[k][j].w; arg[j].w = ee; }
          }
    }
    for (; t < cnt; ++t) {
      int u = l_idx[t];
      if (L == 64) u = __builtin_amdgcn_readfirstlane(u);
      const int32_t ee = c0 + t;
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (slot_ok[j]) {
          const float4 row = ld4(pq + (int64_t)u * ld + 4 * (li + j * L));
          if (row.x > best[j].x) { best[j].x = row.x; arg[j].x = ee; }
          if (row.y > best[j].y) { best[j].y = row.y; arg[j].y = ee; }
          if (row.z > best[j].z) { best[j].z = row.z; arg[j].z = ee; }
          if (row.w > best[j].w) { best[j].w = row.w; arg[j].w = ee; }
        }
    }
    wave_lds_fence();
  }
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j]) {
      const int col = 4 * (li + j * L);
      float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
      if (beg != end) {
        const float4 q = ld4(pq + (int64_t)v * ld + F + col);
        o = make_float4(best[j].x + q.x, best[j].y + q.y, best[j].z + q.z, best[j].w + q.w);
      }
      st4(out + (int64_t)v * F + col, o);
      *reinterpret_cast<int4*>(argmax + (int64_t)v * F + col) = arg[j];
    }
}

// ---- a8: source-side routing of the gradient (CSC walk) ----------------------------
// dpq[u, :F] = sum over out-edges [argmax[v, j] == e] gout[v, j];  dpq[u, F:] = gout[u, :]
// (zero when u has no in-edge: then out[u] = 0 does not depend on Q[u])
template <int L, int NV>
__global__ __launch_bounds__(kEcBlock) void k_edgeconv_bwd_src(
    int32_t n_rows, const int32_t* __restrict__ order_t, const int32_t* __restrict__ indptr_t,
    const int32_t* __restrict__ indices_t, const int32_t* __restrict__ eid_t,
    const int32_t* __restrict__ argmax, const float* __restrict__ gout, int F,
    float* __restrict__ dpq) {
  constexpr int G = kWave / L;
  constexpr int GPB = G * (kEcBlock / kWave);
  __shared__ int lds[GPB * 2 * L];
  const int lane = threadIdx.x & 63;
  const int li = lane & (L - 1);
  const int grp = threadIdx.x / L;
  const int64_t r = order_t ? (int64_t)blockIdx.x * GPB + grp : xcd_contiguous_row(blockIdx.x, gridDim.x, GPB, grp);
  if (r >= n_rows) return;
  int* l_v = lds + grp * 2 * L;
  int* l_e = l_v + L;
  const int32_t u = order_t ? order_t[r] : (int32_t)r;
  const int32_t beg = indptr_t[u], end = indptr_t[u + 1];

  bool slot_ok[NV];
  float4 acc[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    slot_ok[j] = 4 * (li + j * L) < F;
    acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  for (int32_t c0 = beg; c0 < end; c0 += L) {
    const int32_t i = c0 + li;
    l_v[li] = i < end ? indices_t[i] : 0;
    l_e[li] = i < end ? eid_t[i] : -2;
    wave_lds_fence();
    // slots past the end of the row hold vertex 0 and edge id -2, which no arg-max equals:
    // the loop runs in steps of U with all 2U row loads issued before they are used
    constexpr int U = 4;
    const int cnt = min(L, end - c0);
    for (int t0 = 0; t0 < cnt; t0 += U) {
      int vv[U], ee[U];
#pragma unroll
      for (int t = 0; t < U; ++t) {
        vv[t] = l_v[t0 + t];
        ee[t] = l_e[t0 + t];
        if (L == 64) { vv[t] = __builtin_amdgcn_readfirstlane(vv[t]); ee[t] = __builtin_amdgcn_readfirstlane(ee[t]); }
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        if (!slot_ok[j]) continue;
        int4 a[U];
        float4 gg[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
          const int64_t off = (int64_t)vv[t] * F + 4 * (li + j * L);
          a[t] = *reinterpret_cast<const int4*>(argmax + off);
          gg[t] = ld4(gout + off);
        }
#pragma unroll
        for (int t = 0; t < U; ++t) {
          acc[j].x += a[t].x == ee[t] ? gg[t].x : 0.f;
          acc[j].y += a[t].y == ee[t] ? gg[t].y : 0.f;
          acc[j].z += a[t].z == ee[t] ? gg[t].z : 0.f;
          acc[j].w += a[t].w == ee[t] ? gg[t].w : 0.f;
        }
      }
    }
    wave_lds_fence();
  }
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (slot_ok[j]) {
      const int col = 4 * (li + j * L);
      st4(dpq + (int64_t)u * 2 * F + col, acc[j]);
      // dQ[u] = gout[u], except that a vertex without in-edges has a constant output
      const int4 own = *reinterpret_cast<const int4*>(argmax + (int64_t)u * F + col);
      float4 gq = ld4(gout + (int64_t)u * F + col);
      if (own.x < 0) gq = make_float4(0.f, 0.f, 0.f, 0.f);
      st4(dpq + (int64_t)u * 2 * F + F + col, gq);
    }
}

// Degree order (heaviest rows first) balances skewed graphs; when the largest degree is within
// a small factor of the mean it buys nothing and vertex order keeps neighbourhoods together.
static bool near_uniform_degrees(const gnn_graph_t* g, int side) {
  if (config_get(kCfgForceSimple)) return false;
  const int64_t mean = g->n > 0 ? (g->nnz + g->n - 1) / g->n : 0;
  return (int64_t)g->max_degree[side] <= 4 * (mean > 1 ? mean : 1);
}

template <int L, int NV>
struct EcFwdLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const float* pq, int F, float* out, int32_t* argmax,
                          hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kEcBlock / kWave);
    ProfScope p("edgeconv_fwd_fused", st);
    const bool by_id = near_uniform_degrees(g, 0);
    const unsigned grid = by_id ? xcd_contiguous_grid(g->n, GPB) : (unsigned)cdiv(g->n, GPB);
    k_edgeconv_fwd<L, NV><<<grid, kEcBlock, 0, st>>>(g->n, by_id ? nullptr : g->order[0], g->indptr,
                                                     g->indices, pq, F, out, argmax);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};

template <int L, int NV>
struct EcBwdLauncher {
  static gnn_status_t run(const gnn_graph_t* g, const int32_t* argmax, const float* gout, int F,
                          float* dpq, hipStream_t st) {
    constexpr int GPB = (kWave / L) * (kEcBlock / kWave);
    ProfScope p("edgeconv_bwd_src", st);
    const bool by_id = near_uniform_degrees(g, 1);
    const unsigned grid = by_id ? xcd_contiguous_grid(g->n, GPB) : (unsigned)cdiv(g->n, GPB);
    k_edgeconv_bwd_src<L, NV><<<grid, kEcBlock, 0, st>>>(g->n, by_id ? nullptr : g->order[1], g->indptr_t,
                                                         g->indices_t, g->eid_t, argmax, gout, F, dpq);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
  }
};

template <template <int, int> class Launcher, typename... Args>
static gnn_status_t ec_dispatch(GroupShape gs, Args... args) {
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

struct EcWs {
  size_t total, wcat, dpq, gcat, gemm;
  int split_k;
};

static EcWs ec_ws_layout(int64_t n, int fin, int fout) {
  EcWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += ws_granule(bytes); return o; };
  w.wcat = take(sizeof(float) * 2 * (size_t)fin * fout);
  w.dpq = take(sizeof(float) * 2 * (size_t)n * fout);
  w.gcat = take(sizeof(float) * 2 * (size_t)fin * fout);
  w.split_k = gemm_pick_split_k(fin, 2 * fout, n);
  w.gemm = take(w.split_k > 1 ? sizeof(float) * (size_t)w.split_k * fin * 2 * fout : 0);
  w.total = off;
  return w;
}

static gnn_status_t ec_check(const gnn_graph_t* g, int fin, int fout, const char* who) {
  GNN_REQUIRE(g != nullptr, GNN_ERR_INVALID_ARG, "%s: graph is null", who);
  GNN_REQUIRE(fin > 0 && fout > 0, GNN_ERR_INVALID_ARG, "%s: sizes must be positive", who);
  GNN_REQUIRE(fout % 4 == 0 && fout <= 1024, GNN_ERR_UNSUPPORTED,
              "%s: fout = %d must be a multiple of 4, at most 1024", who, fout);
  return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" size_t gnn_edgeconv_workspace_bytes(const gnn_graph_t* g, int fin, int fout) {
  if (!g || fin <= 0 || fout <= 0) return 0;
  return ec_ws_layout(g->n, fin, fout).total;
}

extern "C" gnn_status_t gnn_edgeconv_fwd(const gnn_graph_t* g, int fin, int fout, const float* x,
                                         const float* theta, const float* phi, float* pq, float* out,
                                         int32_t* argmax, void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(ec_check(g, fin, fout, "gnn_edgeconv_fwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && theta && phi && pq && out && argmax, GNN_ERR_INVALID_ARG,
              "gnn_edgeconv_fwd: null pointer");
  GNN_REQUIRE(aligned16(pq) && aligned16(out) && aligned16(argmax), GNN_ERR_INVALID_ARG,
              "gnn_edgeconv_fwd: pq, out, argmax must be 16-byte aligned");
  const EcWs L = ec_ws_layout(g->n, fin, fout);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "gnn_edgeconv_fwd: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* wcat = reinterpret_cast<float*>(static_cast<char*>(ws) + L.wcat);
  {
    ProfScope p("edgeconv_concat_weights", st);
    k_ec_concat_weights<<<(unsigned)cdiv((int64_t)fin * fout, 256), 256, 0, st>>>(fin, fout, theta, phi, wcat);
    GNN_LAUNCH_CHECK();
  }
  // projection before propagation: [P | Q] = x [Theta | Phi - Theta]
  GNN_TRY(gemm_f32(g->n, 2 * fout, fin, x, fin, false, wcat, 2 * fout, false, pq, 2 * fout, 1, nullptr, st));
  return ec_dispatch<EcFwdLauncher>(pick_group(fout), g, (const float*)pq, fout, out, argmax, st);
}

extern "C" gnn_status_t gnn_edgeconv_bwd(const gnn_graph_t* g, int fin, int fout, const float* x,
                                         const float* theta, const float* phi, const int32_t* argmax,
                                         const float* gout, float* gx, float* gtheta, float* gphi,
                                         void* ws, size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(ec_check(g, fin, fout, "gnn_edgeconv_bwd"));
  if (g->n == 0) return GNN_OK;
  GNN_REQUIRE(x && theta && phi && argmax && gout && gtheta && gphi, GNN_ERR_INVALID_ARG,
              "gnn_edgeconv_bwd: null pointer");
  GNN_REQUIRE(aligned16(argmax) && aligned16(gout), GNN_ERR_INVALID_ARG,
              "gnn_edgeconv_bwd: argmax, gout must be 16-byte aligned");
  const EcWs L = ec_ws_layout(g->n, fin, fout);
  GNN_REQUIRE(ws != nullptr && ws_bytes >= L.total, GNN_ERR_WORKSPACE,
              "gnn_edgeconv_bwd: workspace of %zu bytes given, %zu needed", ws_bytes, L.total);
  GNN_REQUIRE(aligned16(ws), GNN_ERR_INVALID_ARG, "gnn_edgeconv_bwd: workspace must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  float* wcat = reinterpret_cast<float*>(base + L.wcat);
  float* dpq = reinterpret_cast<float*>(base + L.dpq);
  float* gcat = reinterpret_cast<float*>(base + L.gcat);
  float* part = reinterpret_cast<float*>(base + L.gemm);
  const int64_t n = g->n;

  GNN_TRY(ec_dispatch<EcBwdLauncher>(pick_group(fout), g, argmax, gout, fout, dpq, st));
  GNN_TRY(gemm_f32(fin, 2 * fout, n, x, fin, true, dpq, 2 * fout, false, gcat, 2 * fout, L.split_k, part, st));
  {
    ProfScope p("edgeconv_split_weight_grads", st);
    k_ec_split_weight_grads<<<(unsigned)cdiv((int64_t)fin * fout, 256), 256, 0, st>>>(fin, fout, gcat, gtheta, gphi);
    GNN_LAUNCH_CHECK();
  }
  if (gx) {
    {
      ProfScope p("edgeconv_concat_weights", st);
      k_ec_concat_weights<<<(unsigned)cdiv((int64_t)fin * fout, 256), 256, 0, st>>>(fin, fout, theta, phi, wcat);
      GNN_LAUNCH_CHECK();
    }
    GNN_TRY(gemm_f32(n, fin, 2 * fout, dpq, 2 * fout, false, wcat, 2 * fout, true, gx, fin, 1, nullptr, st));
  }
  return GNN_OK;
}
