/*
 * gnn_fused.h — C ABI of the reorganized, fused GNN layers for MI355X (gfx950).
 *
 * One GNN layer = an expensive per-vertex projection done BEFORE propagation
 * (Sec. 4, propagation-postponed reorganization), then ONE fused pass per
 * destination vertex that does Scatter, the lightweight ApplyEdge, the
 * ReduceScatter (edge-softmax) and the Aggregate under a single vertex-balanced
 * thread mapping (Sec. 5), and a backward pass that recomputes every per-edge
 * value from O(|V|) saved state (Sec. 6).  The layer calls of the scope table (GAT,
 * EdgeConv, GMM with degree-pair coordinates, GCN) neither read nor write a tensor
 * with one row per edge.  Two groups of calls do, and say so where they are declared:
 * the general-pseudo-coordinate GMM layer (pseudo and gpseudo are [nnz, r] inputs /
 * outputs of the layer's definition) and the "fusion with stashing" ablation arm
 * (gnn_gat_stash_alpha, gnn_gat_bwd_stashed: [nnz, heads]).
 *
 * Conventions
 *   - A graph is the edge set {(u, e, v)} of App. A.1 stored as CSR by
 *     DESTINATION: indptr[n+1], indices[nnz]; row v lists the sources u of the
 *     in-edges of v; the edge id e is the CSR position.  Duplicate edges are
 *     distinct edges.  0 <= nnz < 2^31.
 *   - Every pointer is a DEVICE pointer to contiguous row-major memory, float
 *     (fp32) or int32_t, unless a comment says "host".  The caller owns every
 *     buffer it passes.  Rows of feature matrices must start 16-byte aligned
 *     where noted (feature widths that are multiples of 4 floats).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; layer calls never synchronise with the host and
 *     never allocate.  Scratch comes from a caller-provided workspace whose size
 *     the matching *_workspace_bytes() call returns (0 is possible; then ws may
 *     be NULL).
 *   - Every function returns a gnn_status_t.  On failure nothing useful has been
 *     written and gnn_last_error() returns a thread-local, library-owned string.
 *   - Outputs are bit-reproducible from run to run: sums are taken in a fixed order and
 *     there are no floating-point atomics.  One exception, never taken silently: the
 *     edge-balanced mapping of the GCN sums, of the GMM forward pass and of the source side
 *     of the GMM backward pass adds the pieces of rows that span several runs with atomics;
 *     it runs only after gnn_gcn_tune / gnn_gmm_tune / gnn_gmm_tune_bwd has measured it
 *     faster on a graph, or when the configuration key
 *     gcn_mapping / gmm_mapping is set to 1, and rows above 64 (32) edges may then
 *     differ in the last bits from run to run.
 */
#ifndef GNN_FUSED_H
#define GNN_FUSED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gnn_status {
  GNN_OK = 0,
  GNN_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned buffer            */
  GNN_ERR_BAD_GRAPH = 2,   /* indptr not monotone / wrong ends, source id outside [0,n) */
  GNN_ERR_WORKSPACE = 3,   /* workspace smaller than *_workspace_bytes()                */
  GNN_ERR_UNSUPPORTED = 4, /* shape outside what the kernels are built for              */
  GNN_ERR_HIP = 5          /* a HIP runtime call failed; text in gnn_last_error()       */
} gnn_status_t;

/* Text of the last error raised on the calling thread ("" if none).  Library-owned. */
const char* gnn_last_error(void);

/* ------------------------------------------------------------------------- *
 * Graph plan (once per graph; its cost is preprocessing, cf. Sec. 8.1 "GNN
 * runtime optimization").  The vertex-balanced mapping of Sec. 5 loops over the
 * in-edge set of a vertex; the source-side gradients loop over the out-edge set,
 * which needs the transpose.  The plan holds integer tables only:
 *
 *   CSC transpose   edges ordered by (source ascending, CSR position ascending):
 *                   indptr_t[n+1], indices_t[nnz] = destination of each out-edge,
 *                   eid_t[nnz] = CSR position of that edge.
 *   degree order    per side (0 = in-degree / CSR rows, 1 = out-degree / CSC rows)
 *                   the vertices sorted by degree descending, ties by ascending id.
 *                   Kernels hand out rows in this order, heaviest first.
 *   degree bucket   clz32(degree): number of leading zero bits of the degree as a
 *                   32-bit integer, 32 for degree 0 (GNN_NUM_BUCKETS = 33 values);
 *                   bucket ids ascend along the degree order;
 *                   bucket_offsets[b] = first position of bucket b in the order,
 *                   bucket_offsets[33] = n.
 *
 * All of it is a pure function of (indptr, indices) and is bit-exact.
 * ------------------------------------------------------------------------- */
#define GNN_NUM_BUCKETS 33

typedef struct gnn_graph gnn_graph_t;

/* Validates the CSR arrays on the device, builds the plan and returns a handle.
 * indptr/indices are BORROWED: they must stay valid and unchanged until
 * gnn_graph_destroy.  This call allocates device memory for the plan tables
 * (about 8*nnz + 32*n bytes kept, plus sort scratch released before returning)
 * and synchronises `stream` once to read the validation result.
 * Errors: INVALID_ARG (n < 0, nnz < 0, null pointers with n > 0), UNSUPPORTED
 * (nnz >= 2^31), BAD_GRAPH, HIP. */
gnn_status_t gnn_graph_create(int32_t n, int64_t nnz, const int32_t* indptr, const int32_t* indices,
                              void* stream, gnn_graph_t** graph);

/* Frees the plan tables (not the borrowed CSR arrays).  NULL is accepted.  Waits for the
 * device first (kernels still reading the tables must have finished, because the memory goes
 * back to a free list that the next gnn_graph_create may draw from at once). */
gnn_status_t gnn_graph_destroy(gnn_graph_t* graph);

/* Introspection for bit-exact tests: copies plan tables into caller buffers
 * (device pointers; any of them may be NULL to skip it). */
gnn_status_t gnn_graph_get_csc(const gnn_graph_t* graph, int32_t* indptr_t /*n+1*/,
                               int32_t* indices_t /*nnz*/, int32_t* eid_t /*nnz*/, void* stream);
gnn_status_t gnn_graph_get_buckets(const gnn_graph_t* graph, int side /*0 = dst rows, 1 = src rows*/,
                                   int32_t* bucket_of_vertex /*n*/, int32_t* order /*n*/,
                                   int32_t* bucket_offsets /*GNN_NUM_BUCKETS+1*/, void* stream);

/* Column-blocked edge lists (built when n > block_cols; else num_blocks = 1 and
 * nothing is copied).  A gathered feature matrix that exceeds the L2 caches is
 * walked one block of `block_cols` gathered vertices at a time, so that the rows a
 * launch gathers stay cache-resident.  For each side (0: rows = destinations,
 * columns = sources; 1: rows = sources, columns = destinations) the edges are
 * stable-sorted by (column / block_cols, row):
 *   bcol[nnz]                 column (gathered vertex) of each edge in that order
 *   bptr[num_blocks * n + 1]  bptr[b*n + r] .. bptr[b*n + r + 1] = edges of row r
 *                             whose column lies in block b
 * num_blocks and block_cols are written to HOST ints; bptr, bcol are device
 * pointers (may be NULL). */
gnn_status_t gnn_graph_get_blocked(const gnn_graph_t* graph, int side, int32_t* num_blocks /*host*/,
                                   int32_t* block_cols /*host*/, int32_t* bptr, int32_t* bcol,
                                   void* stream);

/* Launch groups of the column-blocked kernels.  Such a kernel reads and writes a row's running
 * sums once per launch, which costs as much as gathering some ten to twenty neighbour rows; blocks
 * in which a row has fewer edges than that are therefore walked several per launch (a row's
 * segments of up to 8 adjacent blocks one after the other), at the price of a wider set of
 * gathered rows competing for the L2.  gnn_graph_create picks the partition of the block sequence
 * with the least modelled cost from the edge counts of the blocks, once for kernels that keep one
 * running sum per row (`sums` = 1: the GCN sum, the GAT forward pass without stash) and once for
 * those that keep two (`sums` = 2: the GAT forward pass with stash, the source side of its
 * backward pass).  Group j covers the blocks groups[j] .. groups[j + 1] - 1; *count = number of
 * groups (0 when the graph has no blocked lists), groups (HOST, num_blocks + 1 ints, may be NULL)
 * receives count + 1 boundaries. */
gnn_status_t gnn_graph_get_launch_groups(const gnn_graph_t* graph, int side, int sums,
                                         int32_t* groups /*host*/, int32_t* count /*host*/);

/* Plan tables and the temporaries of gnn_graph_create come from a free list inside the library
 * (blocks of up to 64 MB, at most 512 MB idle in total), so that graphs which are rebuilt all
 * the time (a k-nearest-neighbour graph per training step) do not pay hipMalloc / hipFree each
 * time.  gnn_graph_destroy waits for the device, then returns the graph's blocks to that list;
 * this call hands every idle block back to the driver. */
gnn_status_t gnn_release_cached_memory(void);

/* Tuning knobs, read when a graph is created or a layer is called.  Keys:
 *   "block_cols"            gathered vertices per column block (default 12288:
 *                           12288 rows x one 256-byte slice = 3 MB of an XCD's 4 MB L2);
 *                           0 disables blocking.  Read by gnn_graph_create.
 *   "resident_sums"         1 (default): where rows are cut into 256-byte slices (and for single-head
 *                           or GCN rows of at most 64 floats, one slice) the column-blocked
 *                           GAT and GCN kernels run all blocks of a pass in ONE persistent launch
 *                           (one 1024-thread workgroup per CU) that keeps the rows' running sums
 *                           and softmax statistics in LDS, a few thousand rows per workgroup at a
 *                           time, instead of reading and writing them once per block.  The
 *                           workgroups of an XCD meet at the end of every such batch of rows
 *                           through counters the graph handle owns (a bounded wait that only
 *                           serves cache residency); layer calls on ONE graph that overlap in
 *                           time share those counters: their results stay right, their cache
 *                           hit rates suffer.  0: one launch per block or group of blocks.
 *                           Both give the same bits as one launch per block.
 *   "resident_spin"         polls after which a workgroup of that launch stops waiting for the
 *                           others of its XCD (default 4096; 0 = never wait; meant for tests)
 *   "resident_sync_every"   the workgroups of an XCD meet after every k-th column block instead
 *                           of once per batch of rows (default 0 = once per batch)
 *   "merge_blocks"          1 (default): adjacent column blocks with few edges share one
 *                           launch of a column-blocked kernel (up to 8 blocks; a row's running
 *                           sums are then read and written once for all of them), chosen per
 *                           graph from the edge counts of the blocks.  0: one launch per block.
 *                           Read by gnn_graph_create.
 *   "blocked_min_edges"     mean number of edges per (row, column block) from which the
 *                           column-blocked kernels are used (default 16; sparser graphs take
 *                           the single-launch kernels even when they span several blocks).
 *                           Read by the layer calls and by gnn_graph_create, which builds no
 *                           blocked lists for a graph below it (lowering the key afterwards
 *                           does not bring them back for that graph).
 *   "gather_precision"      0 (default): fp32 throughout.  1: the column-blocked GAT kernels
 *                           gather the neighbour rows (z in forward, gout in the source-side
 *                           backward) from an fp16 copy, sums in fp32: about half the gather
 *                           traffic; errors of about 1e-3 of a tensor's rms (several 1e-3 in
 *                           the worst gradient entries) instead of the 1e-4 contract.  Set it before workspace sizes are
 *                           queried; shapes it does not cover (heads*f % 64 != 0, a 64-column
 *                           slice spanning heads) stay fp32.
 *   "wide_offsets"          1: the column-blocked GAT kernels address the gathered rows with 64-bit
 *                           offsets also where 32 bits reach every row (the code path of gathered
 *                           matrices of 4 GB and more; meant for tests).  Default 0.
 *   "force_simple_kernels"  1: always use the single-launch kernels
 *   "lds_scalar_table"      1 (default): the column-blocked destination-side GAT kernels
 *                           keep a block's per-vertex score table in LDS (one persistent
 *                           1024-thread workgroup per CU drawing rows from a counter);
 *                           0: every edge gathers its scalar from L2
 *   "gcn_mapping"           thread mapping of the GCN aggregation: 0 vertex-balanced,
 *                           1 edge-balanced, 2 (default) what gnn_gcn_tune measured as
 *                           faster on the graph (vertex-balanced if it never ran)
 *   "gmm_mapping"           the same for the forward aggregation of the GMM layer and the two
 *                           halves of its backward pass (gnn_gmm_tune, gnn_gmm_tune_bwd; the
 *                           edge-balanced mapping takes at most 4 kernels)
 * Errors: INVALID_ARG for an unknown key or a value out of range. */
gnn_status_t gnn_config_set(const char* key, int64_t value);

/* ------------------------------------------------------------------------- *
 * Projection: the ExpensiveApply on vertices, y = x w  (Sec. 3, Sec. 4; App. A.2
 * "H~ = H W").  x [n, fin], w [fin, fout], y [n, fout]; any positive sizes.
 * fp32 MFMA (v_mfma_f32_32x32x2_f32), fp32 accumulate.  No workspace.
 * ------------------------------------------------------------------------- */
gnn_status_t gnn_linear_fwd(int64_t n, int fin, int fout, const float* x, const float* w, float* y,
                            void* stream);

/* ------------------------------------------------------------------------- *
 * GAT layer (App. A.2 "GAT"; score of Sec. 4 Eq. 1 in its reorganized form
 * a_l.Wh_u + a_r.Wh_v; fused M0..H^(l+1) operator of App. A.2 / Sec. 5; saved
 * max and denominator of Sec. 6).
 *
 *   z   = x w                         [n, heads*f]   head-major columns
 *   el  = <z[u,h,:], a_l[h,:]>        [n, heads]     source half
 *   er  = <z[v,h,:], a_r[h,:]>        [n, heads]     destination half
 *   s_e = LeakyReLU_slope(el[u,h] + er[v,h])         e = (u -> v)
 *   m   = max over in-edges of s_e    [n, heads]     (0 for an empty row)
 *   d   = sum exp(s_e - m)            [n, heads]     (1 for an empty row)
 *   out = sum (exp(s_e - m) / d) z[u] [n, heads*f]   (0 for an empty row)
 *
 *   t   = sum alpha_e g_e z[u]        [n, heads*f]   optional, g_e = LeakyReLU'(el[u]+er[v])
 *   sg  = sum alpha_e g_e             [n, heads]     optional
 *
 * Requirements: f % 4 == 0, heads*f <= 1024, heads <= 64; x, w any width.
 * Forward writes z, el, er, m, d, out (all of them are the saved state the
 * backward call needs; none has a per-edge dimension).  t and sg (both or neither,
 * may be NULL) are the destination-side sums of the backward pass; they ride on the
 * rows the forward pass gathers anyway and are vertex-sized, so by the criterion of
 * Sec. 6 (recompute only if computation / memory is O(1); here it is |E|/|V|) they
 * are worth stashing: the backward call then skips one whole pass over the edges.
 * Pass NULL for inference, or to have the backward call recompute them.
 * The workspace is optional in the forward call (NULL is accepted; the column-blocked
 * kernels keep a head-major copy of el and their running softmax statistics there, so
 * without it large graphs fall back to the slower single-launch kernels).
 * ------------------------------------------------------------------------- */
size_t gnn_gat_workspace_bytes(const gnn_graph_t* graph, int fin, int heads, int f);

gnn_status_t gnn_gat_fwd(const gnn_graph_t* graph, int fin, int heads, int f, float slope,
                         const float* x /*[n,fin]*/, const float* w /*[fin,heads*f]*/,
                         const float* a_l /*[heads,f]*/, const float* a_r /*[heads,f]*/,
                         float* z /*[n,heads*f]*/, float* el, float* er, float* m, float* d /*[n,heads]*/,
                         float* out /*[n,heads*f]*/, float* t /*[n,heads*f] nullable*/,
                         float* sg /*[n,heads] nullable*/, void* ws, size_t ws_bytes, void* stream);

/* Gradients of L = <gout, out>.  Per-edge scores and softmax values are
 * recomputed from el, er, m, d; LeakyReLU'(0) = slope.  t, sg: what the forward
 * call wrote, or both NULL (then they are recomputed with one more pass over the
 * in-edges).  gx may be NULL (skip the input gradient).
 * Writes gx [n,fin], gw [fin,heads*f], ga_l, ga_r [heads,f]. */
gnn_status_t gnn_gat_bwd(const gnn_graph_t* graph, int fin, int heads, int f, float slope,
                         const float* x, const float* w, const float* a_l, const float* a_r,
                         const float* z, const float* el, const float* er, const float* m,
                         const float* d, const float* out, const float* t /*nullable*/,
                         const float* sg /*nullable*/, const float* gout /*[n,heads*f]*/,
                         float* gx /*nullable*/, float* gw, float* ga_l, float* ga_r,
                         void* ws, size_t ws_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): gnn_gat_bwd with its scratch in a
 * device array built into the library, GNN_NOALLOC_SCRATCH_BYTES long (every GPU the library runs
 * on holds its copy until the process ends).  Same arguments, kernels and results as gnn_gat_bwd
 * minus (ws, ws_bytes); calls no hipMalloc/hipFree.  Fails with GNN_ERR_WORKSPACE and a message
 * naming both sizes when gnn_gat_workspace_bytes(graph, fin, heads, f) exceeds the array.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or threads) race and must be serialised by the caller.  Nothing the array holds is
 * expected to survive from one call to the next. */
#define GNN_NOALLOC_SCRATCH_BYTES (64u << 20)
gnn_status_t gnn_gat_bwd_noalloc(const gnn_graph_t* graph, int fin, int heads, int f, float slope,
                                 const float* x, const float* w, const float* a_l, const float* a_r,
                                 const float* z, const float* el, const float* er, const float* m,
                                 const float* d, const float* out, const float* t /*nullable*/,
                                 const float* sg /*nullable*/, const float* gout /*[n,heads*f]*/,
                                 float* gx /*nullable*/, float* gw, float* ga_l, float* ga_r, void* stream);

/* Introspection for measurement scripts: the instantiation of the column-blocked edge kernel that
 * a pass over this graph launches for `heads` x `f` (mode 0 forward, 1 destination side recomputing,
 * 2 source side, 3 forward with stash) under the current configuration, spelled as a profiler
 * prints it, e.g. "k_gat_res<16, 2, true, false, true>" (the persistent launch) or
 * "k_gat_blk<16, 2, false, false, true>" (one launch per block); the empty string when the
 * single-launch kernels run.  buf is a HOST buffer of len bytes. */
gnn_status_t gnn_gat_blocked_kernel_name(const gnn_graph_t* graph, int heads, int f, int mode,
                                         char* buf /*host*/, size_t len);

/* The "fusion with stashing" arm of the recomputation study (Sec. 7.3): the fused kernels, but
 * the per-edge softmax values are stored after the forward pass and read back in the
 * backward pass instead of being recomputed.  Kept for that comparison; it needs O(|E|)
 * memory, which the default path avoids.
 * gnn_gat_stash_alpha: nnz * heads floats, value = softmax weight of an edge with the sign of
 *   its raw score (negative: LeakyReLU' = slope), laid out for the source-side kernel that the
 *   backward pass of this graph and shape (heads x f) takes; gnn_gat_stash_layout says which:
 *     0  alpha_t[p, h], p = position in the plan's CSC transpose ((source, CSR position) order),
 *        for the single-launch kernel;
 *     1  alpha_t[h, q], q = position in the source side's column-blocked edge list
 *        (gnn_graph_get_blocked, side 1), for the column-blocked kernel.
 *   Call after gnn_gat_fwd (needs el, er, m, d).
 * gnn_gat_bwd_stashed: as gnn_gat_bwd, with the source side reading the stash instead of
 *   recomputing the softmax values (the per-destination scalar D is still gathered). */
int gnn_gat_stash_layout(const gnn_graph_t* graph, int heads, int f);
gnn_status_t gnn_gat_stash_alpha(const gnn_graph_t* graph, int heads, int f, float slope, const float* el,
                                 const float* er, const float* m, const float* d,
                                 float* alpha_t /*nnz*heads floats*/, void* stream);
gnn_status_t gnn_gat_bwd_stashed(const gnn_graph_t* graph, int fin, int heads, int f, float slope,
                                 const float* x, const float* w, const float* a_l, const float* a_r,
                                 const float* z, const float* el, const float* er, const float* m,
                                 const float* d, const float* out, const float* t /*nullable*/,
                                 const float* sg /*nullable*/, const float* alpha_t /*[nnz,heads]*/,
                                 const float* gout, float* gx /*nullable*/, float* gw, float* ga_l,
                                 float* ga_r, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------- *
 * EdgeConv layer (App. A.2 "EdgeConv"), in the reorganized form of Sec. 4:
 * Theta(h_u - h_v) + Phi h_v = (x Theta)[u] + (x (Phi - Theta))[v].
 *
 *   pq  = x [Theta | Phi - Theta]                [n, 2*fout]  (P | Q), saved
 *   out = max over in-edges of P[u] + Q[v]       [n, fout]    (0 for an empty row)
 *   argmax[v, j] = CSR position of the winning in-edge, the earliest one on an
 *                  exact tie, -1 for an empty row             [n, fout] int32
 *
 * Requirements: fout % 4 == 0, fout <= 1024.  theta, phi are [fin, fout].
 * Only argmax (O(|V|)) is needed by the backward pass (Sec. 7.2 "EdgeConv").
 * ------------------------------------------------------------------------- */
size_t gnn_edgeconv_workspace_bytes(const gnn_graph_t* graph, int fin, int fout);

gnn_status_t gnn_edgeconv_fwd(const gnn_graph_t* graph, int fin, int fout, const float* x,
                              const float* theta, const float* phi, float* pq /*[n,2*fout]*/,
                              float* out /*[n,fout]*/, int32_t* argmax /*[n,fout]*/,
                              void* ws, size_t ws_bytes, void* stream);

/* Gradients of L = <gout, out>: gx [n,fin] (nullable), gtheta, gphi [fin,fout]. */
gnn_status_t gnn_edgeconv_bwd(const gnn_graph_t* graph, int fin, int fout, const float* x,
                              const float* theta, const float* phi, const int32_t* argmax,
                              const float* gout /*[n,fout]*/, float* gx /*nullable*/, float* gtheta,
                              float* gphi, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------- *
 * MoNet / GMMConv layer (App. A.2 "GMMConv").
 *
 *   hk  = x w_fc                                   [n, k*fout] viewed [n, k, fout], saved
 *   m_e = (c[u], c[v])                             2-D pseudo-coordinates of e = (u -> v)
 *   w_j(m) = exp(-1/2 sum_d ((m_d - mu[j,d]) * inv_sigma[j,d])^2)        j < k
 *   out[v] = (1/k) sum over in-edges sum_j w_j(m_e) hk[u, j, :]          [n, fout]
 *
 * The covariance is diagonal, Sigma_j^-1 = diag(inv_sigma[j]^2); c is a
 * per-vertex scalar supplied by the caller (no gradient).  The Gaussian
 * weights are never stored: backward recomputes them (Sec. 7.3).
 * Requirements: fout % 4 == 0, fout <= 256, 1 <= k <= 8.
 *
 * Order of projection and aggregation (the reorganization argument of Sec. 4: a linear
 * operator commutes with the weighted sums, so it runs on whichever side is cheaper).
 * When an input row is narrower than the k projected rows (fin < k*fout, fin % 4 == 0,
 * fin <= 256) and the forward call is given the workspace, the layer aggregates first,
 *   out = (1/k) [ sum_e w_j(m_e) x[u] ]_j  W',   W' = w_fc regrouped to [k*fin, fout],
 * so an edge gathers fin floats once instead of k*fout, and hk is NOT written (the backward
 * call then does not read it either: its destination side gathers x against gout W'^T).
 * Otherwise (or without a workspace in the forward call) hk = x w_fc is written and the
 * edges gather the projected rows; hk must then be passed unchanged to the backward call.
 * ------------------------------------------------------------------------- */
size_t gnn_gmm_workspace_bytes(const gnn_graph_t* graph, int fin, int fout, int k);

gnn_status_t gnn_gmm_fwd(const gnn_graph_t* graph, int fin, int fout, int k, const float* x,
                         const float* w_fc /*[fin,k*fout]*/, const float* c /*[n]*/,
                         const float* mu /*[k,2]*/, const float* inv_sigma /*[k,2]*/,
                         float* hk /*[n,k*fout]*/, float* out /*[n,fout]*/,
                         void* ws, size_t ws_bytes, void* stream);

/* Gradients of L = <gout, out>: gx [n,fin] (nullable), gw_fc [fin,k*fout],
 * gmu, ginv_sigma [k,2]. */
gnn_status_t gnn_gmm_bwd(const gnn_graph_t* graph, int fin, int fout, int k, const float* x,
                         const float* w_fc, const float* c, const float* mu, const float* inv_sigma,
                         const float* hk, const float* gout /*[n,fout]*/, float* gx /*nullable*/,
                         float* gw_fc, float* gmu, float* ginv_sigma,
                         void* ws, size_t ws_bytes, void* stream);

/* Profile-driven choice of the thread mapping of the forward aggregation (Sec. 5), as
 * gnn_gcn_tune: runs the fused Gaussian-weight + aggregate pass on the given tensors (the
 * ones of a forward call: hk already projected) in the vertex-balanced and in the
 * edge-balanced mapping (groups own runs of 32 edges, atomic adds between runs, at most 4
 * kernels), and records the faster one in the graph handle; gnn_gmm_fwd uses it while the
 * configuration key "gmm_mapping" is 2 (default; 0 / 1 force one).  out holds the layer's
 * result afterwards.  ms_out (host, nullable): 2 floats, milliseconds per pass
 * {vertex-balanced, edge-balanced} (zeros when k > 4 or the graph has no edges: nothing to
 * choose).  Waits for the stream.  Errors: INVALID_ARG, UNSUPPORTED, HIP. */
gnn_status_t gnn_gmm_tune(gnn_graph_t* graph, int fout, int k, const float* hk /*[n,k*fout]*/,
                          const float* c, const float* mu, const float* inv_sigma, float* out /*[n,fout]*/,
                          void* stream, float* ms_out /*host [2], nullable*/);

/* The same choice for the two halves of gnn_gmm_bwd (Sec. 5): the destination side (gradients of
 * mu and inv_sigma; its edge-balanced form needs no atomics, a row's pieces are complete on their
 * own because the gradients are linear in the per-edge terms) and the source side (dhk; pieces of
 * rows that span several runs of 32 edges are added atomically).  Runs each half in both mappings
 * on the tensors of a backward call and records the faster mapping per half in the graph handle;
 * gnn_gmm_bwd follows it while "gmm_mapping" is 2 (the destination side only where the layer
 * projects first, which is what the timing compares with).  ws as for gnn_gmm_bwd; its contents
 * are scratch afterwards.  ms_out (host, nullable): 4 floats, milliseconds per pass {destination
 * vertex-balanced, edge-balanced, source vertex-balanced, edge-balanced} (zeros when k > 4 or the
 * graph has no edges).  Waits for the stream.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
gnn_status_t gnn_gmm_tune_bwd(gnn_graph_t* graph, int fin, int fout, int k, const float* hk /*[n,k*fout]*/,
                              const float* c, const float* mu, const float* inv_sigma,
                              const float* gout /*[n,fout]*/, void* ws, size_t ws_bytes, void* stream,
                              float* ms_out /*host [4], nullable*/);

/* ------------------------------------------------------------------------- *
 * MoNet / GMMConv layer with general pseudo-coordinates (App. A.2 "GMMConv"; Sec. 7.2 uses
 * pseudo-coordinate dimensions r = 1, 2, 3 and 2 or 3 kernels):
 *   w_j(e) = exp(-1/2 sum_d ((pseudo[e,d] - mu[j,d]) inv_sigma[j,d])^2),   d < r
 *   out[v] = (1/k) sum over in-edges e = (u -> v) sum_j w_j(e) hk[u,j,:],   hk = x w_fc
 * pseudo [nnz, r] is a per-edge INPUT in CSR order (position e of `indices`).  The backward
 * call recomputes the weights and also returns gpseudo [nnz, r] (nullable), the gradient
 * with respect to the pseudo-coordinates, for a caller that learns them.  pseudo_t (nullable)
 * holds the same coordinates in the order of the transposed edge list (position p of
 * gnn_graph_get_csc's indices_t): the source side of backward walks that list, and without
 * pseudo_t it reads pseudo through the plan's position -> edge table, one scattered 4r-byte read
 * per edge (3.2 against 1.4 ms at Reddit scale).  Rows of up to 64 projected floats (k fout <= 64,
 * the paper's 16 hidden features) take kernels that walk an edge set in chunks with 8 gathers
 * in flight per lane.
 * Limits: k <= 4, r <= 4, fout % 4 == 0, fout <= 256.  Errors as for gnn_gmm_*.
 *
 * gnn_pseudo_proj_fwd / _bwd: the projection that makes such coordinates from a per-vertex
 * scalar c (1/sqrt(degree) in the paper's models): pseudo[e,d] = tanh(proj_w[d,0] c[u] +
 * proj_w[d,1] c[v] + proj_b[d]), written in CSR order to pseudo and, if pseudo_t is not null, in the
 * transposed list's order to pseudo_t (computed from c a second time, not permuted); backward returns gproj_w [r,2], gproj_b [r] from gpseudo
 * (workspace of gnn_pseudo_proj_workspace_bytes, sums in a fixed order).
 * ------------------------------------------------------------------------- */
size_t gnn_gmmp_workspace_bytes(const gnn_graph_t* graph, int fin, int fout, int k);
gnn_status_t gnn_gmmp_fwd(const gnn_graph_t* graph, int fin, int fout, int k, int r, const float* x,
                          const float* w_fc /*[fin,k*fout]*/, const float* pseudo /*[nnz,r]*/,
                          const float* mu /*[k,r]*/, const float* inv_sigma /*[k,r]*/,
                          float* hk /*[n,k*fout]*/, float* out /*[n,fout]*/, void* stream);
gnn_status_t gnn_gmmp_bwd(const gnn_graph_t* graph, int fin, int fout, int k, int r, const float* x,
                          const float* w_fc, const float* pseudo, const float* mu, const float* inv_sigma,
                          const float* hk, const float* gout /*[n,fout]*/, float* gx /*nullable*/,
                          float* gw_fc, float* gmu, float* ginv_sigma, float* gpseudo /*[nnz,r] nullable*/,
                          const float* pseudo_t /*[nnz,r] nullable*/, void* ws, size_t ws_bytes, void* stream);
size_t gnn_pseudo_proj_workspace_bytes(const gnn_graph_t* graph);
gnn_status_t gnn_pseudo_proj_fwd(const gnn_graph_t* graph, int r, const float* c /*[n]*/,
                                 const float* proj_w /*[r,2]*/, const float* proj_b /*[r]*/,
                                 float* pseudo /*[nnz,r]*/, float* pseudo_t /*[nnz,r] nullable*/, void* stream);
gnn_status_t gnn_pseudo_proj_bwd(const gnn_graph_t* graph, int r, const float* c, const float* pseudo,
                                 const float* gpseudo, float* gproj_w /*[r,2]*/, float* gproj_b /*[r]*/,
                                 void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------- *
 * MoNet layer with the projection fused in (the paper's MoNet models, Sec. 7.2 / 7.3: pseudo-
 * coordinates are a learnable projection of the degree pair, then App. A.2 "GMMConv"):
 *   m[e,d] = tanh(proj_w[d,0] c[u] + proj_w[d,1] c[v] + proj_b[d]),   w_j(e), out as above.
 * Every edge function of the chain (projection, tanh, Gaussian weight, weighting) is evaluated
 * inside the gather kernels from the per-vertex scalar c at the two ends of the edge, forward and
 * again in both halves of backward; no per-edge tensor is read, written or kept (Sec. 4, Sec. 6).
 * Same results as gnn_pseudo_proj_fwd + gnn_gmmp_fwd and gnn_gmmp_bwd + gnn_pseudo_proj_bwd.
 * c [n], proj_w [r,2], proj_b [r]; backward returns gproj_w [r,2], gproj_b [r] besides the
 * gradients of gnn_gmmp_bwd (gx nullable).  Limits: those of gnn_gmmp_* and k * fout <= 64 (the
 * paper's 16 hidden features; wider layers take the two-call form), else GNN_ERR_UNSUPPORTED.
 * Workspace: gnn_monet_workspace_bytes; parameter gradients are summed in a fixed order.
 * ------------------------------------------------------------------------- */
size_t gnn_monet_workspace_bytes(const gnn_graph_t* graph, int fin, int fout, int k);
gnn_status_t gnn_monet_fwd(const gnn_graph_t* graph, int fin, int fout, int k, int r, const float* x,
                           const float* w_fc /*[fin,k*fout]*/, const float* c /*[n]*/,
                           const float* proj_w /*[r,2]*/, const float* proj_b /*[r]*/, const float* mu /*[k,r]*/,
                           const float* inv_sigma /*[k,r]*/, float* hk /*[n,k*fout]*/, float* out /*[n,fout]*/,
                           void* stream);
gnn_status_t gnn_monet_bwd(const gnn_graph_t* graph, int fin, int fout, int k, int r, const float* x,
                           const float* w_fc, const float* c, const float* proj_w, const float* proj_b,
                           const float* mu, const float* inv_sigma, const float* hk,
                           const float* gout /*[n,fout]*/, float* gx /*nullable*/, float* gw_fc, float* gmu,
                           float* ginv_sigma, float* gproj_w, float* gproj_b, void* ws, size_t ws_bytes,
                           void* stream);

/* ------------------------------------------------------------------------- *
 * GCN layer with separable static edge weights (App. A.2 "GCN", no bias, identity
 * activation):
 *   out[v] = sum over in-edges (u -> v) of  c_src[u] c_dst[v] (x w)[u]
 * c_src, c_dst [n] are per-vertex factors of the gradient-free edge weight (both
 * 1/sqrt(degree) for the symmetric normalisation; (1, 1/degree) for the mean).
 * Both factors are applied on vertices (Sec. 4), so the fused pass is an unweighted
 * gather-sum.  zs [n,fout] receives c_src * (x w) (an output; the backward call does
 * not need it).  fout % 4 == 0, fout <= 1024; zs, out, gout 16-byte aligned.
 * gnn_gcn_bwd: gradients of L = <gout, out> w.r.t. x (gx [n,fin], nullable) and
 * w (gw [fin,fout]); workspace of gnn_gcn_workspace_bytes (vertex-sized).
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP as for the other layers.
 * ------------------------------------------------------------------------- */
size_t gnn_gcn_workspace_bytes(const gnn_graph_t* graph, int fin, int fout);

gnn_status_t gnn_gcn_fwd(const gnn_graph_t* graph, int fin, int fout, const float* x /*[n,fin]*/,
                         const float* w /*[fin,fout]*/, const float* c_src /*[n]*/,
                         const float* c_dst /*[n]*/, float* zs /*[n,fout]*/, float* out /*[n,fout]*/,
                         void* stream);

gnn_status_t gnn_gcn_bwd(const gnn_graph_t* graph, int fin, int fout, const float* x, const float* w,
                         const float* c_src, const float* c_dst, const float* gout /*[n,fout]*/,
                         float* gx /*nullable*/, float* gw, void* ws, size_t ws_bytes, void* stream);

/* The same layer with a GENERAL static weight per edge (App. A.2 "GCN": e_uv is any gradient-free
 * scalar of the edge):  out[v] = sum over in-edges e = (u -> v) of edge_w[e] (x w)[u].
 * The weights are static, so they are copied ONCE into every order the kernels walk (CSR, the CSC
 * transpose and, on graphs that span several column blocks, both blocked edge lists: 4 * nnz bytes
 * each); gnn_edge_weights_create does that (it allocates from the plan's free list and waits for
 * the stream, like gnn_graph_create) and the layer calls then read one more coalesced stream
 * next to the index list: no per-edge gather, no allocation.  edge_w is [nnz] in CSR order (the
 * order of `indices`), duplicate edges carry their own weights; it is an input of the layer's
 * definition, not a stash.  The handle belongs to the graph it was made for and must be
 * destroyed before it.  z [n,fout] receives x w.  Vertex-balanced mapping only.
 * Workspace of the backward call: gnn_gcn_workspace_bytes.  Errors as for gnn_gcn_fwd / bwd, plus
 * INVALID_ARG for a handle made for another graph. */
typedef struct gnn_edge_weights gnn_edge_weights_t;
gnn_status_t gnn_edge_weights_create(const gnn_graph_t* graph, const float* edge_w /*[nnz]*/, void* stream,
                                     gnn_edge_weights_t** weights);
gnn_status_t gnn_edge_weights_destroy(gnn_edge_weights_t* weights);
gnn_status_t gnn_gcn_edge_fwd(const gnn_graph_t* graph, const gnn_edge_weights_t* weights, int fin, int fout,
                              const float* x /*[n,fin]*/, const float* w /*[fin,fout]*/,
                              float* z /*[n,fout]*/, float* out /*[n,fout]*/, void* stream);
gnn_status_t gnn_gcn_edge_bwd(const gnn_graph_t* graph, const gnn_edge_weights_t* weights, int fin, int fout,
                              const float* x, const float* w, const float* gout /*[n,fout]*/,
                              float* gx /*nullable*/, float* gw, void* ws, size_t ws_bytes, void* stream);

/* Profile-driven choice of the thread mapping (Sec. 5: the fused Gather runs either
 * vertex-balanced, one thread group per row, or edge-balanced, one group per fixed run of
 * edges with atomic adds where a row spans several runs; the faster one is picked by
 * profiling).  Times both mappings of the aggregation at width fout on this graph, for the
 * in-edge side (forward) and the out-edge side (backward), and records the faster one per
 * side in the graph handle; gnn_gcn_fwd / gnn_gcn_bwd use it while the configuration key
 * "gcn_mapping" is 2 (the default; 0 forces vertex-balanced, 1 edge-balanced).  The
 * edge-balanced mapping sums the pieces of a row longer than 64 edges in arrival order:
 * results agree to rounding but are not bit-reproducible from run to run.
 * ws: device scratch of gnn_gcn_workspace_bytes(graph, 1, fout) bytes (contents destroyed).
 * ms_out (host, nullable) receives 4 floats: milliseconds per aggregation for
 * {in-edge side vertex-balanced, edge-balanced, out-edge side vertex-balanced, edge-balanced}.
 * Unlike the layer calls this one waits for the stream (a set-up call, like
 * gnn_graph_create).  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
gnn_status_t gnn_gcn_tune(gnn_graph_t* graph, int fout, void* ws, size_t ws_bytes, void* stream,
                          float* ms_out /*host [4], nullable*/);

/* The same for the GCN sums over rows of `fout` floats (weighted = 1: the layer with a general weight
 * per edge), e.g. "k_rowsum_res<16, false>" or "k_rowsum_blk<16, true, false>"; the empty string
 * when the single-launch or edge-balanced kernels run. */
gnn_status_t gnn_gcn_blocked_kernel_name(const gnn_graph_t* graph, int fout, int weighted,
                                         char* buf /*host*/, size_t len);

/* ------------------------------------------------------------------------- *
 * Lightweight vertex operators and the loss of a node-classification step (Sec. 3:
 * element-wise Apply- operators on vertices; Sec. 7.2: the end-to-end runs train
 * two-layer node classifiers).  All matrices are [n, f] fp32, rows 16-byte aligned
 * (f % 4 == 0, f <= 1024).
 *
 * gnn_bias_act_fwd:  out = act(in + bias); bias [f] may be NULL; in == out allowed.
 *   act: GNN_ACT_IDENTITY, GNN_ACT_RELU, GNN_ACT_ELU (alpha 1), GNN_ACT_LEAKY (slope >= 0).
 * gnn_bias_act_bwd:  gin = gout * act'(.) taken from the forward OUTPUT y (ReLU'(0) = 0,
 *   LeakyReLU'(0) = slope, ELU' = y + 1 for y <= 0), gbias [f] = column sums of gin
 *   (NULL to skip; needs the workspace of gnn_bias_act_workspace_bytes, summed in a fixed
 *   order).  gin == gout allowed; y may be NULL for the identity.
 * gnn_softmax_xent:  loss (device scalar) = mean over the labelled vertices of
 *   log sum_c exp(z[v,c]) - z[v, label[v]];  glogits [n,c] = (softmax(z[v]) - onehot) /
 *   n_labelled, zero rows for unlabelled vertices.  A label outside [0, c) marks a vertex
 *   as unlabelled; n_labelled is the caller's count of the others (0: loss 0).
 *   Any c <= 4096, no alignment needed.
 * gnn_sgd_update:    param -= lr * grad over `count` floats.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP as for the layers.
 * ------------------------------------------------------------------------- */
enum { GNN_ACT_IDENTITY = 0, GNN_ACT_RELU = 1, GNN_ACT_ELU = 2, GNN_ACT_LEAKY = 3 };

gnn_status_t gnn_bias_act_fwd(int64_t n, int f, int act, float slope, const float* in /*[n,f]*/,
                              const float* bias /*[f] nullable*/, float* out /*[n,f]*/, void* stream);
size_t gnn_bias_act_workspace_bytes(int64_t n, int f);
gnn_status_t gnn_bias_act_bwd(int64_t n, int f, int act, float slope, const float* y /*[n,f]*/,
                              const float* gout /*[n,f]*/, float* gin /*[n,f]*/,
                              float* gbias /*[f] nullable*/, void* ws, size_t ws_bytes, void* stream);
size_t gnn_softmax_xent_workspace_bytes(int64_t n);
gnn_status_t gnn_softmax_xent(int64_t n, int c, int64_t n_labelled, const float* logits /*[n,c]*/,
                              const int32_t* labels /*[n]*/, float* loss /*device, 1 float*/,
                              float* glogits /*[n,c]*/, void* ws, size_t ws_bytes, void* stream);
gnn_status_t gnn_sgd_update(int64_t count, float lr, const float* grad, float* param, void* stream);

/* ------------------------------------------------------------------------- *
 * k-nearest-neighbour graph of a batch of point clouds (the EdgeConv model builds its
 * graph from the points, Sec. 7.2: k = 20 / 40 inside each cloud).  coords is
 * [clouds*points, dim] fp32; vertex id = cloud * points + i.  For every point: the k
 * points of its own cloud with the smallest squared Euclidean distance, itself included,
 * ties towards the lower index.  The squared distance is accumulated in float32,
 * coordinate by coordinate in index order, each operation rounded on its own, so the
 * choice is reproducible bit for bit.  Output: CSR by destination, indptr [n+1]
 * (= i*k), indices [n*k] (sources ascending in a row), ready for gnn_graph_create.
 * Limits: k <= points <= 2048, n*k < 2^31.  Coordinates must not be NaN.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 * ------------------------------------------------------------------------- */
gnn_status_t gnn_knn_graph(int clouds, int points, int dim, int k, const float* coords,
                           int32_t* indptr /*[n+1]*/, int32_t* indices /*[n*k]*/, void* stream);

/* ------------------------------------------------------------------------- *
 * Per-kernel timing (measurement aid, Sec. 7 metrics).  While enabled, every
 * kernel the library launches is bracketed by HIP events recorded on the
 * caller's stream.  gnn_prof_collect synchronises those events (host sync) and
 * folds them into per-kernel totals; gnn_prof_get reads entry i (name is a
 * library-owned string).  The bookkeeping is process-wide (one mutex); meant for benchmarks.
 * ------------------------------------------------------------------------- */
gnn_status_t gnn_prof_enable(int on);
gnn_status_t gnn_prof_collect(void);
gnn_status_t gnn_prof_reset(void);
int gnn_prof_count(void);
gnn_status_t gnn_prof_get(int i, const char** name, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* GNN_FUSED_H */
