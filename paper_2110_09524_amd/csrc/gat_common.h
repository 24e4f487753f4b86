// Pieces shared by the single-launch and the column-blocked GAT kernels.
#pragma once

#include "common.h"
#include "rowgroup.h"

namespace gnn {

struct GatDims {
  int H, F, HF;
  int log2Hp;  // heads padded to a power of two; lanes of a group = (edge, head) pairs
  float slope;
};

inline GatDims make_dims(int H, int F, float slope) {
  GatDims dm;
  dm.H = H;
  dm.F = F;
  dm.HF = H * F;
  dm.log2Hp = ilog2(next_pow2(H));
  dm.slope = slope;
  return dm;
}

__device__ __forceinline__ float leaky(float x, float slope) { return x > 0.f ? x : slope * x; }

// ---- column-blocked path (gat_blocked.hip) -----------------------------------------
// True when the blocked kernels apply: several column blocks in the plan, a row of
// heads*f floats that splits into 8 slices (one per XCD) of 4..64 float4 each, and every
// slice inside one head.
bool gat_blocked_applies(const gnn_graph_t* g, int heads, int f);
size_t gat_blocked_ws_bytes(const gnn_graph_t* g, int heads, int f);  // extra workspace (bwd)
// t, sg: optional stash of the destination-side backward sums (both or neither);
// state: n * 8 float4 of scratch for the running softmax statistics (required)
gnn_status_t gat_blocked_fwd(const gnn_graph_t* g, GatDims dm, const float* z, const float* el,
                             const float* er, float* m, float* d, float* out, float* t, float* sg,
                             float* el_t /* [H][n] scratch or null */,
                             int32_t* queue /* nblk * 8 row counters or null */, float4* state,
                             void* half_buf /* n * HF * 2 bytes or null: room for an fp16 copy of z */,
                             hipStream_t st);
// true when the blocked kernels would gather from an fp16 copy for this shape (configuration)
bool gat_blocked_half(const gnn_graph_t* g, int heads, int f);
// vertex-side closing steps shared by both paths (gat.hip); flags: see k_gat_dst_finish
constexpr int kDstHeadMajor = 1, kDstHalfGout = 2;
gnn_status_t gat_dst_finish(const gnn_graph_t* g, GatDims dm, const float* gout, const float* t,
                            const float* out, const float* sg, const float* er, const float* m,
                            const float* d, int flags, float* der, float4* vstate,
                            hipStream_t st);
gnn_status_t gat_src_finish(const gnn_graph_t* g, GatDims dm, const float* z, const float* a2,
                            const float* sd, const float* der, const float* a_l, const float* a_r,
                            float* dz, float* del, hipStream_t st);
// writes der, vstate (like the single-launch destination kernel); t_buf is an [n, HF] scratch
gnn_status_t gat_blocked_bwd_dst(const gnn_graph_t* g, GatDims dm, const float* z, const float* el,
                                 const float* er, const float* m, const float* d, const float* out,
                                 const float* gout, float* der, float4* vstate, float* t_buf,
                                 float* sg_buf, float* el_t /* [H][n] scratch or null */,
                                 int32_t* queue /* nblk * 8 row counters or null */, hipStream_t st);
// writes dz, del; sd_buf is an [n, 8] scratch (per-slice shares of del)
gnn_status_t gat_blocked_bwd_src(const gnn_graph_t* g, GatDims dm, const float* z, const float* el,
                                 const float4* vstate, const float* der, const float* gout,
                                 const float* a_l, const float* a_r, float* dz, float* del,
                                 float* sd_buf, void* half_buf /* n * HF * 2 bytes or null */,
                                 hipStream_t st,
                                 const float* alpha_b = nullptr /* [H][nnz] stash in blocked order, or null */);
// writes the per-edge stash in the order gat_blocked_bwd_src reads it
gnn_status_t gat_blocked_stash_alpha(const gnn_graph_t* g, int H, float slope, const float* el, const float* er,
                                     const float* m, const float* d, float* alpha_b, hipStream_t st);

}  // namespace gnn
