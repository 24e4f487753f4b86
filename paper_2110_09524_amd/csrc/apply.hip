// Lightweight vertex operators around the graph layers (Sec. 3: element-wise Apply- operators
// on vertices are cheap next to the graph operators and the projections): bias + activation
// between two layers, the softmax cross-entropy that closes a node-classification step
// (the end-to-end setting of Sec. 7.2), and the plain SGD update.  All are streaming kernels
// over [n, f] matrices; sums over vertices are taken in two fixed-order stages (reproducible).
#include "common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kApplyThreads = 256;
constexpr int kApplyMaxParts = 1024;

__device__ __forceinline__ float act_fwd(int act, float slope, float x) {
  switch (act) {
    case GNN_ACT_RELU: return x > 0.f ? x : 0.f;
    case GNN_ACT_ELU: return x > 0.f ? x : expm1f(x);
    case GNN_ACT_LEAKY: return x > 0.f ? x : slope * x;
    default: return x;
  }
}
// derivative of the activation, from its OUTPUT y (so the pre-activation need not be kept):
// ReLU y > 0; LeakyReLU (slope >= 0) has the sign of its input, slope at 0; ELU' = exp(x) = y + 1
__device__ __forceinline__ float act_grad(int act, float slope, float y) {
  switch (act) {
    case GNN_ACT_RELU: return y > 0.f ? 1.f : 0.f;
    case GNN_ACT_ELU: return y > 0.f ? 1.f : y + 1.f;
    case GNN_ACT_LEAKY: return y > 0.f ? 1.f : slope;
    default: return 1.f;
  }
}

__global__ __launch_bounds__(kApplyThreads) void k_bias_act_fwd(
    int64_t quads, int q_per_row, int act, float slope, const float* in, const float* __restrict__ bias,
    float* out) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= quads) return;
  float4 v = ld4(in + 4 * i);
  if (bias) {
    const float4 b = ld4(bias + 4 * (i % q_per_row));
    v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
  }
  st4(out + 4 * i, make_float4(act_fwd(act, slope, v.x), act_fwd(act, slope, v.y), act_fwd(act, slope, v.z),
                               act_fwd(act, slope, v.w)));
}

// gin = gout * act'(y); the workgroup's column sums of gin go to partial[blockIdx.x][f].
// Lanes = float4 column slots (QP of them, a power of two >= f/4), the other thread-index bits
// spread over rows; a workgroup owns rows_per_wg consecutive rows.
__global__ __launch_bounds__(kApplyThreads) void k_bias_act_bwd(
    int64_t n, int f, int qp_log2, int64_t rows_per_wg, int act, float slope, const float* __restrict__ y,
    const float* gout, float* gin, float* __restrict__ partial /* nullable */) {
  __shared__ float4 red[kApplyThreads];
  const int QP = 1 << qp_log2;
  const int q = threadIdx.x & (QP - 1);
  const int rl = threadIdx.x >> qp_log2, nrl = kApplyThreads >> qp_log2;
  const bool q_ok = 4 * q < f;
  const int64_t r0 = blockIdx.x * rows_per_wg;
  const int64_t r1 = r0 + rows_per_wg < n ? r0 + rows_per_wg : n;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (q_ok) {
    for (int64_t r = r0 + rl; r < r1; r += nrl) {
      const int64_t o = r * f + 4 * q;
      const float4 g = ld4(gout + o);
      float4 d = make_float4(1.f, 1.f, 1.f, 1.f);
      if (act != GNN_ACT_IDENTITY) {
        const float4 yy = ld4(y + o);
        d = make_float4(act_grad(act, slope, yy.x), act_grad(act, slope, yy.y), act_grad(act, slope, yy.z),
                        act_grad(act, slope, yy.w));
      }
      const float4 gi = make_float4(g.x * d.x, g.y * d.y, g.z * d.z, g.w * d.w);
      if (gin != gout || act != GNN_ACT_IDENTITY) st4(gin + o, gi);
      add4(s, gi);
    }
  }
  if (partial == nullptr) return;  // uniform
  red[threadIdx.x] = s;
  __syncthreads();
  if (rl == 0 && q_ok) {
    for (int k = 1; k < nrl; ++k) add4(s, red[(k << qp_log2) + q]);  // fixed order
    st4(partial + (int64_t)blockIdx.x * f + 4 * q, s);
  }
}

// ---- softmax cross-entropy ---------------------------------------------------------------
// A workgroup takes kXentVerts consecutive vertices, 16 lanes per vertex (lane j owns classes
// j, j + 16, ...: the 16 groups of a pass read 16 consecutive rows, one contiguous run), 4 passes;
// per-workgroup loss sums to partial[], in a fixed order.
constexpr int kXentVerts = 64;
__global__ __launch_bounds__(kApplyThreads) void k_softmax_xent(
    int64_t n, int c, float inv_count, const float* __restrict__ logits, const int32_t* __restrict__ labels,
    float* __restrict__ glogits, float* __restrict__ partial) {
  constexpr int L = 16, G = kApplyThreads / L;
  __shared__ float red[G];
  const int li = threadIdx.x & (L - 1), grp = threadIdx.x / L;
  float loss = 0.f;  // lane 0 of a group: the sum over the group's vertices, in pass order
  for (int pass = 0; pass < kXentVerts / G; ++pass) {
    const int64_t v = blockIdx.x * (int64_t)kXentVerts + pass * G + grp;
    if (v >= n) break;  // uniform over the group
    const float* z = logits + v * c;
    float* g = glogits + v * c;
    const int32_t lab = labels[v];
    if (lab < 0 || lab >= c) {  // unlabelled
      for (int j = li; j < c; j += L) g[j] = 0.f;
      continue;
    }
    float mx = -INFINITY;
    for (int j = li; j < c; j += L) mx = fmaxf(mx, z[j]);
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, L));
    float se = 0.f;
    for (int j = li; j < c; j += L) se += expf(z[j] - mx);
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) se += __shfl_xor(se, o, L);
    const float inv = 1.f / se;
    for (int j = li; j < c; j += L) g[j] = (expf(z[j] - mx) * inv - (j == lab ? 1.f : 0.f)) * inv_count;
    loss += (mx + logf(se)) - z[lab];
  }
  if (li == 0) red[grp] = loss;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < G; ++i) s += red[i];  // fixed order
    partial[blockIdx.x] = s;
  }
}

// loss = inv_count * sum of the partials, in a fixed tree order (one workgroup)
__global__ __launch_bounds__(kApplyThreads) void k_xent_finish(int parts, float inv_count,
                                                               const float* __restrict__ partial,
                                                               float* __restrict__ loss) {
  __shared__ float red[kApplyThreads];
  float s = 0.f;
  for (int i = threadIdx.x; i < parts; i += kApplyThreads) s += partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = kApplyThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = red[0] * inv_count;
}

__global__ void k_sgd_update(int64_t count, float lr, const float* __restrict__ grad, float* __restrict__ param) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < count) param[i] = fmaf(-lr, grad[i], param[i]);
}

static int bias_parts(int64_t n) {
  // about 64 rows per workgroup, at most kApplyMaxParts workgroups
  int64_t parts = cdiv(n, 64);
  if (parts > kApplyMaxParts) parts = kApplyMaxParts;
  return parts < 1 ? 1 : (int)parts;
}

static gnn_status_t check_act(int64_t n, int f, int act, float slope, const char* who) {
  GNN_REQUIRE(n >= 0 && f > 0, GNN_ERR_INVALID_ARG, "%s: sizes must be positive", who);
  GNN_REQUIRE(f % 4 == 0 && f <= 1024, GNN_ERR_UNSUPPORTED, "%s: f = %d must be a multiple of 4, at most 1024",
              who, f);
  GNN_REQUIRE(act >= GNN_ACT_IDENTITY && act <= GNN_ACT_LEAKY, GNN_ERR_INVALID_ARG, "%s: unknown activation %d",
              who, act);
  GNN_REQUIRE(act != GNN_ACT_LEAKY || slope >= 0.f, GNN_ERR_INVALID_ARG, "%s: slope must not be negative", who);
  return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" gnn_status_t gnn_bias_act_fwd(int64_t n, int f, int act, float slope, const float* in,
                                         const float* bias, float* out, void* stream) {
  clear_error();
  GNN_TRY(check_act(n, f, act, slope, "gnn_bias_act_fwd"));
  if (n == 0) return GNN_OK;
  GNN_REQUIRE(in && out, GNN_ERR_INVALID_ARG, "gnn_bias_act_fwd: null pointer");
  GNN_REQUIRE(aligned16(in) && aligned16(out) && aligned16(bias), GNN_ERR_INVALID_ARG,
              "gnn_bias_act_fwd: in, bias, out must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope p("bias_act_fwd", st);
  const int64_t quads = n * (f / 4);
  k_bias_act_fwd<<<(unsigned)cdiv(quads, kApplyThreads), kApplyThreads, 0, st>>>(quads, f / 4, act, slope, in,
                                                                                bias, out);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

extern "C" size_t gnn_bias_act_workspace_bytes(int64_t n, int f) {
  if (n <= 0 || f <= 0) return 0;
  return ws_granule(sizeof(float) * (size_t)bias_parts(n) * f);
}

extern "C" gnn_status_t gnn_bias_act_bwd(int64_t n, int f, int act, float slope, const float* y,
                                         const float* gout, float* gin, float* gbias, void* ws,
                                         size_t ws_bytes, void* stream) {
  clear_error();
  GNN_TRY(check_act(n, f, act, slope, "gnn_bias_act_bwd"));
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (n == 0) return gbias ? sum_partials(f, 0, nullptr, gbias, st) : GNN_OK;  // a sum of no parts: zeros
  GNN_REQUIRE(gout && gin && (y || act == GNN_ACT_IDENTITY), GNN_ERR_INVALID_ARG,
              "gnn_bias_act_bwd: null pointer");
  GNN_REQUIRE(aligned16(y) && aligned16(gout) && aligned16(gin), GNN_ERR_INVALID_ARG,
              "gnn_bias_act_bwd: y, gout, gin must be 16-byte aligned");
  const int parts = bias_parts(n);
  float* partial = nullptr;
  if (gbias) {
    GNN_REQUIRE(ws != nullptr && ws_bytes >= gnn_bias_act_workspace_bytes(n, f) && aligned16(ws),
                GNN_ERR_WORKSPACE, "gnn_bias_act_bwd: workspace of %zu bytes given, %zu needed (16-byte aligned)",
                ws_bytes, gnn_bias_act_workspace_bytes(n, f));
    partial = static_cast<float*>(ws);
  }
  {
    ProfScope p("bias_act_bwd", st);
    const int qp_log2 = ilog2(next_pow2(f / 4));
    k_bias_act_bwd<<<parts, kApplyThreads, 0, st>>>(n, f, qp_log2, cdiv(n, parts), act, slope, y, gout, gin,
                                                    partial);
    GNN_LAUNCH_CHECK();
  }
  if (gbias) {
    ProfScope p("bias_grad_sum", st);
    GNN_TRY(sum_partials(f, parts, partial, gbias, st));
  }
  return GNN_OK;
}

extern "C" size_t gnn_softmax_xent_workspace_bytes(int64_t n) {
  if (n <= 0) return 0;
  return ws_granule(sizeof(float) * (size_t)cdiv(n, kXentVerts));
}

extern "C" gnn_status_t gnn_softmax_xent(int64_t n, int c, int64_t n_labelled, const float* logits,
                                         const int32_t* labels, float* loss, float* glogits, void* ws,
                                         size_t ws_bytes, void* stream) {
  clear_error();
  GNN_REQUIRE(n >= 0 && c > 0 && n_labelled >= 0, GNN_ERR_INVALID_ARG, "gnn_softmax_xent: sizes must be positive");
  GNN_REQUIRE(c <= 4096, GNN_ERR_UNSUPPORTED, "gnn_softmax_xent: %d classes exceed 4096", c);
  GNN_REQUIRE(loss != nullptr, GNN_ERR_INVALID_ARG, "gnn_softmax_xent: loss is null");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int64_t parts = cdiv(n, kXentVerts);
  GNN_REQUIRE(parts < (int64_t)INT32_MAX, GNN_ERR_UNSUPPORTED, "gnn_softmax_xent: too many vertices");
  if (n != 0) {
    GNN_REQUIRE(logits && labels && glogits, GNN_ERR_INVALID_ARG, "gnn_softmax_xent: null pointer");
    GNN_REQUIRE(ws != nullptr && ws_bytes >= gnn_softmax_xent_workspace_bytes(n), GNN_ERR_WORKSPACE,
                "gnn_softmax_xent: workspace of %zu bytes given, %zu needed", ws_bytes,
                gnn_softmax_xent_workspace_bytes(n));
  }
  const float inv_count = n_labelled > 0 ? 1.f / (float)n_labelled : 0.f;
  ProfScope p("softmax_xent", st);
  float* partial = static_cast<float*>(ws);
  if (n != 0) {
    k_softmax_xent<<<(unsigned)parts, kApplyThreads, 0, st>>>(n, c, inv_count, logits, labels, glogits, partial);
    GNN_LAUNCH_CHECK();
  }
  k_xent_finish<<<1, kApplyThreads, 0, st>>>((int)parts, inv_count, partial, loss);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

extern "C" gnn_status_t gnn_sgd_update(int64_t count, float lr, const float* grad, float* param, void* stream) {
  clear_error();
  GNN_REQUIRE(count >= 0, GNN_ERR_INVALID_ARG, "gnn_sgd_update: negative count");
  if (count == 0) return GNN_OK;
  GNN_REQUIRE(grad && param, GNN_ERR_INVALID_ARG, "gnn_sgd_update: null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope p("sgd_update", st);
  k_sgd_update<<<(unsigned)cdiv(count, 256), 256, 0, st>>>(count, lr, grad, param);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}
