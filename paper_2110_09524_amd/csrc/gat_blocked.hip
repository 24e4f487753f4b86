// Column-blocked, XCD-sliced variants of the three GAT edge kernels, for graphs whose
// projected feature matrix does not fit the L2 caches.
//
// The single-launch kernels gather one full row (heads*f floats) per edge from
// anywhere in a matrix of hundreds of MB; on MI355X each of the 8 XCDs has its own
// 4 MB L2, so nearly every gather misses and the kernels run at the speed of the
// fabric behind the L2s.  Here the same sums are re-associated so that what a
// launch gathers is cache-resident:
//   * columns are cut into 8 slices, workgroup id mod 8 picks the slice; workgroups
//     are handed to the XCDs round-robin, so XCD k only ever touches slice k of a row;
//   * the gathered vertices are cut into blocks of `block_cols`; launch b walks only
//     the edges whose gathered vertex lies in block b (plan tables bptr/bcol), so one
//     launch touches block_cols * slice_bytes per XCD (2 MB by default);
//   * per-row partial sums live in an [n, heads*f] buffer that every launch after the
//     first reads, adds to and writes back (launches on one stream run in order, so
//     there is no race and the summation order is fixed).
// The edge-softmax of the forward pass runs online across the launches: every (row, slice)
// carries its running maximum and sums from block to block and the last block normalises,
// which also yields m and d (Sec. 6: exactly the O(|V|) state that is saved).
// All per-edge values are still recomputed on the fly; nothing per-edge is stored.
#include <atomic>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>

#include <hip/hip_fp16.h>

#include "common.h"
#include "gat_common.h"
#include "rowgroup.h"

namespace gnn {

constexpr int kBlkThreads = 256;
constexpr int kSlices = 8;  // column slices of a wide row: one per XCD

// How a row of HF floats is cut: `ns` slices of SL float4 each.  Wide rows (>= 1 KB) give every
// XCD its own slice.  512-byte rows keep slices of a full 128-byte line (SL = 8) and have four of
// them: workgroup id mod 4 picks the slice, so XCD k and XCD k + 4 work on the same columns (for
// different rows) and each L2 still holds one slice of the column block.  A gather of a half line
// would cost the L1 the same fill as a full one.  Rows of 256 bytes and less are not blocked: at
// Reddit scale the single-launch kernels were faster there (the whole matrix then fits the
// Infinity Cache, and a launch per block costs more than it saves).
struct Slicing {
  int SL, ns;
};
static bool pick_slicing(int heads, int HF, Slicing& sl) {
  // One head of at most 64 columns: the row is a single slice of up to 256 bytes, every XCD holds the
  // whole column block (12288 x 256 bytes = 3 MB).  Only the persistent kernels take it: a launch per
  // block measured slower than the single-launch kernels here (4.04 against 3.69 ms for the source
  // side of a 1 x 64 layer at Reddit scale), its read-add-write of the sums being as large as the
  // gathered block.
  if (heads == 1 && HF <= 64 && HF % 4 == 0 && config_get(kCfgResidentSums)) {
    sl = Slicing{16, 1};
    return true;
  }
  if (HF % 32 != 0) return false;
  const int q = HF / 32;  // 128-byte lines per row
  // Slices of 256 bytes (two lines, 16 lanes) where the row has 2, 4 or 8 of them and a slice
  // stays inside one head: an edge then costs one scalar gather per two row lines instead of
  // one per line, and a launch reads its index list and row metadata half as often.  With
  // fewer than 8 slices, workgroup id mod `ns` picks the slice, so XCD k and XCD k + ns work on
  // the same columns for different rows.  Measured at 1 KB rows (Reddit-scale GAT layer):
  // 23.6 -> 21.9 ms per step against 8 slices of 128 bytes; slices of 512 bytes lose
  // (the GCN sum: 17.8 -> 17.2 ms with 256-byte slices, 22.9 ms with 512-byte ones).
  if (q % 2 == 0 && (q / 2 == 2 || q / 2 == 4 || q / 2 == 8) && (q / 2) % heads == 0) {
    sl = Slicing{16, q / 2};
    return true;
  }
  if (q >= kSlices) {
    sl = Slicing{q, kSlices};
    return (q == 8 || q == 16 || q == 32) && kSlices % heads == 0;
  }
  if (q == 4 && q % heads == 0) {
    sl = Slicing{8, q};
    return true;
  }
  sl = Slicing{q, kSlices};  // 64-byte slices, every slice inside one head
  return q == 4 && kSlices % heads == 0;
}

// ---- one column block of a weighted row aggregation ---------------------------------
// MODE 0: forward        acc[v]  += sum_e alpha_e           z[u]      (acc = out)
// MODE 1: bwd, dst side  acc[v]  += sum_e alpha_e g_e       z[u]      (acc = T), sg += sum alpha g
// MODE 2: bwd, src side  acc[u]  += sum_e alpha_e           gout[v]   (acc = dz)
//                        scal[u, slice] += sum_e alpha_e g_e (<z[u], gout[v]>_slice - [leader] D[v])
//                        The dot product is taken lane by lane: a lane multiplies its four columns
//                        of the gathered row with its four columns of z[u] (kept in registers for
//                        the whole row) and adds alpha g times that to a per-lane sum; the lanes are
//                        added once per row.  The slices of a head add up to del[u, h].
// MODE 3: forward that also stashes the destination-side sums of the backward pass:
//                        acc = out as MODE 0, acc2[v] += sum_e alpha_e g_e z[u] (= t), sg += sum alpha g
// A group of SL lanes owns (row, slice); lane li owns the float4 at column slice*4*SL + 4*li.
//
// Each group walks kRowsPerGroup consecutive rows of the degree order, software-pipelined:
// while the edges of one row are processed, the segment bounds, the first index chunk,
// the per-row scalars and the running sums of the next row are already in flight, so the
// chain of dependent loads at the start of a row is paid once per group, not once per row.
constexpr int kRowsPerGroup = 4;
// LDS floats of one group: SL gathered indices, 2 * SL edge weights, the rows of its run and
// their (begin, end) in each of the launch's blocks; a multiple of 4 keeps the 16-byte reads aligned
template <int SL>
constexpr int kBlkGroupFloats = 3 * SL + kRowsPerGroup + 2 * kRowsPerGroup * kMaxMerge;
static_assert(kBlkGroupFloats<4> % 4 == 0 && kBlkGroupFloats<8> % 4 == 0 && kBlkGroupFloats<16> % 4 == 0 &&
              kBlkGroupFloats<32> % 4 == 0, "group scratch must stay 16-byte aligned");

template <int NA>
struct BlkRow {
  int32_t row, beg, end, c_first;
  float r_a, r_m, r_d, scal;
  float4 acc[NA], acc2[NA];
};

// HALF: the gathered matrix is an fp16 copy (the sums stay fp32).  A lane then owns 8 columns
// (16 bytes of the copy) instead of 4, and a 128-byte slice covers 64 columns.
__device__ __forceinline__ void fma8_half(float4 (&acc)[2], float w, const uint4& r) {
  const __half2* h = reinterpret_cast<const __half2*>(&r);
  const float2 a = __half22float2(h[0]), b = __half22float2(h[1]), c = __half22float2(h[2]),
               d = __half22float2(h[3]);
  acc[0].x = fmaf(w, a.x, acc[0].x); acc[0].y = fmaf(w, a.y, acc[0].y);
  acc[0].z = fmaf(w, b.x, acc[0].z); acc[0].w = fmaf(w, b.y, acc[0].w);
  acc[1].x = fmaf(w, c.x, acc[1].x); acc[1].y = fmaf(w, c.y, acc[1].y);
  acc[1].z = fmaf(w, d.x, acc[1].z); acc[1].w = fmaf(w, d.y, acc[1].w);
}

__device__ __forceinline__ float dot8_half(const float4 (&zr)[2], const uint4& r) {
  const __half2* h = reinterpret_cast<const __half2*>(&r);
  const float2 a = __half22float2(h[0]), b = __half22float2(h[1]), c = __half22float2(h[2]),
               d = __half22float2(h[3]);
  return dot4(zr[0], make_float4(a.x, a.y, b.x, b.y)) + dot4(zr[1], make_float4(c.x, c.y, d.x, d.y));
}

// STAGE: the per-edge scalar el[u] of the slice's head is read from an LDS copy of the block's
// part of the head-major table instead of being gathered from L2.  Such a scalar gather
// costs a CU one 128-byte line fill per edge, as much as the 128-byte row slice itself; with
// the table in LDS the row gathers have the L1 to themselves (15 -> 24 TB/s on the bare access
// pattern).  The table takes 4 * block_cols bytes (96 KB), so one 1024-thread workgroup per CU
// runs persistently and the groups draw their rows, four at a time in degree order, from a
// per-slice counter in device memory (zeroed before the launch).
constexpr int kStageThreads = 1024;

template <int SL, int MODE, bool STAGE, bool HALF, bool SKIP>
__global__ __launch_bounds__(STAGE ? kStageThreads : kBlkThreads) void k_gat_blk(
    int32_t n_rows, const int32_t* __restrict__ order, const int2* __restrict__ bseg_b,
    const int32_t* __restrict__ bcol, const float* __restrict__ feat /* gathered rows: z or gout */,
    const float* __restrict__ rowfeat /* MODE 2: z, whose row u meets every gathered gout[v] */,
    const float* __restrict__ el, const float* __restrict__ er, const float* __restrict__ m_in,
    const float* __restrict__ d_in, const float4* __restrict__ vstate, int32_t col_begin,
    GatDims dm, int sph, int first, int narrow, int el_hm /* el is head-major [H][n] */,
    float* __restrict__ acc_buf, float* __restrict__ acc2_buf, float* __restrict__ scal_buf,
    int32_t* __restrict__ queue /* STAGE: one row counter per slice */, int32_t cols_here,
    int32_t quads_per_grab, int ns /* column slices: 8, 4, 2 or 1 */,
    int last /* forward modes: this is the last block */,
    float4* __restrict__ state /* forward modes: running (max, sum, sum2) per (row, slice) */,
    float* __restrict__ m_out, float* __restrict__ d_out,
    int nseg /* adjacent column blocks of this launch (1 .. kMaxMerge): segment j of the row at
                position r of the degree order is bseg_b[j * n_rows + r] */,
    const float* __restrict__ alpha_b /* MODE 2, nullable: stashed signed softmax values, [H][nnz] in the
                                         order of bcol (the "fusion with stashing" arm) */,
    int64_t nnz) {
  constexpr int THREADS = STAGE ? kStageThreads : kBlkThreads;
  constexpr int G = kWave / SL;
  constexpr int GPB = THREADS / SL;
  constexpr int R = kRowsPerGroup;
  constexpr int U = SL < 8 ? 4 : 8;   // gathered rows in flight per lane
  constexpr bool DUAL = MODE == 3;  // two vector accumulators per lane
  constexpr bool SRC = MODE == 2;   // one vector accumulator, the row's own z in registers, a per-lane dot sum
  constexpr int CPL = HALF ? 8 : 4;              // columns per lane
  constexpr int NA = CPL / 4;                    // float4 accumulators per lane and sum
  // The forward modes run the edge-softmax online across the block launches: every (row, slice)
  // carries its running maximum and sums from launch to launch, the running sums are rescaled
  // when the maximum grows, and the last block divides by the denominator.  No separate pass
  // over the edges is needed for the softmax statistics.
  constexpr bool ONLINE = MODE == 0 || MODE == 3;
  constexpr int GS = kBlkGroupFloats<SL>;  // LDS floats per group: idx | p | p2 | rows | (beg, end) per row and block
  static_assert(SL >= R, "one lane per pipelined row loads its metadata");
  static_assert(!STAGE || MODE != 2, "the source side needs 16 bytes per gathered vertex");
  extern __shared__ __align__(16) float lds[];  // GPB * GS floats, then (STAGE) the el table
  (void)G;

  const int lane = threadIdx.x & 63;
  const int li = lane & (SL - 1);
  const int grp = threadIdx.x / SL;
  const int slice = blockIdx.x % ns;
  const int H = dm.H, HF = dm.HF;
  const int h = slice / sph;
  const float* l_el = lds + GPB * GS;
  // [quad, quad_end): the group's current run of row quadruples (R consecutive rows of the
  // degree order each); a staged group draws the next run from the slice's counter
  int64_t quad = 0, quad_end = 0;
  if (STAGE) {
    float* dst = lds + GPB * GS;
    const float* src = el + (int64_t)h * n_rows + col_begin;
    for (int i = threadIdx.x; i < cols_here; i += THREADS) dst[i] = src[i];
    __syncthreads();
  } else {
    quad = (int64_t)(blockIdx.x / ns) * GPB + grp;
    quad_end = quad + 1;
  }

  int* l_idx = reinterpret_cast<int*>(lds + grp * GS);
  float* l_p = lds + grp * GS + SL;
  float* l_p2 = lds + grp * GS + 2 * SL;
  int* l_row = reinterpret_cast<int*>(lds + grp * GS + 3 * SL);
  int2* l_seg = reinterpret_cast<int2*>(l_row + R);  // [R][kMaxMerge]

  const int col = slice * CPL * SL + CPL * li;
  const bool leader = (slice % sph) == 0;  // one slice per head keeps the per-head scalars

  for (;;) {
    if (STAGE && quad == quad_end) {
      // One quadruple per draw: the rows come in degree order, so consecutive quadruples of the hub
      // rows are all heavy, and a group that took several at once would be the last to finish
      // (measured on the hub block of a Reddit-scale graph: 2.7 ms with one per draw, 6.9 ms with
      // four, 4.8 ms with a static round-robin assignment).
      int q = 0;
      if (li == 0) q = atomicAdd(queue + slice, quads_per_grab);
      quad = __shfl(q, lane & ~(SL - 1), 64);
      quad_end = quad + quads_per_grab;
    }
    const int64_t r0 = quad * R;
    if (r0 >= n_rows) break;  // the counter only grows: every group ends here
    wave_lds_fence();         // the previous rows' metadata reads are done
    // segment bounds of the group's R rows inside this column block, one lane each
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
      if (!first && !any && !(ONLINE && last)) row = -1;  // nothing to add to this row in these blocks
      l_row[li] = row;
    }
    wave_lds_fence();

    // issue every load a row needs before its edge loop
    auto fetch = [&](int k, BlkRow<NA>& s) {
      s.row = l_row[k];
      const int2 seg0 = l_seg[k * kMaxMerge];
      s.beg = seg0.x;
      s.end = seg0.y;
      s.c_first = col_begin;
      s.r_a = 0.f; s.r_m = 0.f; s.r_d = 1.f; s.scal = 0.f;
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        s.acc[a] = make_float4(0.f, 0.f, 0.f, 0.f);
        s.acc2[a] = s.acc[a];
      }
      if (s.row < 0) return;
      if (s.beg + li < s.end) s.c_first = bcol[s.beg + li];
      const int64_t rh = (int64_t)s.row * H + h;
      if (MODE == 2) {
        s.r_a = el[rh];  // row is a source: its el
      } else if (ONLINE) {
        s.r_a = er[rh];  // row is a destination; running max, denominator, second sum so far
        s.r_m = -INFINITY;
        s.r_d = 0.f;
        if (!first) {
          const float4 stt = state[(int64_t)s.row * kSlices + slice];
          s.r_m = stt.x; s.r_d = stt.y; s.scal = stt.z;
        }
      } else {
        s.r_a = er[rh];  // row is a destination: its er, max, denominator
        s.r_m = m_in[rh];
        s.r_d = d_in[rh];
      }
      if (!first) {
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          s.acc[a] = ld4_stream(acc_buf + (int64_t)s.row * HF + col + 4 * a);
          if (DUAL) s.acc2[a] = ld4_stream(acc2_buf + (int64_t)s.row * HF + col + 4 * a);
        }
        if (MODE == 1 && leader && li == 0) s.scal = scal_buf[rh];
        if (SRC && li == 0) s.scal = scal_buf[(int64_t)s.row * kSlices + slice];
      }
      if (SRC) {
#pragma unroll
        for (int a = 0; a < NA; ++a) s.acc2[a] = ld4_stream(rowfeat + (int64_t)s.row * HF + col + 4 * a);
      }
    };

    // Gathered rows are addressed with 32-bit byte offsets when the matrix is below 4 GB
    // (one 24-bit multiply-add per row instead of 64-bit arithmetic).
    const char* feat_bytes = reinterpret_cast<const char*>(feat);
    constexpr uint32_t kElem = HALF ? 2u : 4u;  // bytes per stored element of the gathered matrix
    const uint32_t row_bytes = (uint32_t)HF * kElem, col_bytes = (uint32_t)col * kElem;

    BlkRow<NA> cur, nxt;
    fetch(0, cur);
    for (int k = 0; k < R; ++k) {
      if (k + 1 < R) fetch(k + 1, nxt);
      if (cur.row >= 0) {
        const float r_a = cur.r_a, r_m = cur.r_m, r_invd = ONLINE ? 0.f : 1.f / cur.r_d;
        float4 acc[NA], acc2[NA];
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          acc[a] = cur.acc[a];
          acc2[a] = cur.acc2[a];
        }
        float s_run = 0.f;  // chunk-phase lanes: sum of alpha g (MODE 1), of alpha g D[v] (MODE 2)
        float s_dot = 0.f;  // MODE 2, row-phase lanes: sum of alpha g <z[u], gout[v]> over the lane's columns
        // online state: the running maximum is uniform in the group, the sums are per lane
        // (lane 0 carries what earlier blocks left) and are added across lanes at the end
        float m_run = cur.r_m;
        float d_lane = li == 0 ? cur.r_d : 0.f, s2_lane = li == 0 ? cur.scal : 0.f;
        int32_t beg = cur.beg, end = cur.end, c_next = cur.c_first;
        for (int sgi = 0; sgi < nseg; ++sgi) {
        // the bounds and the first indices of the row's segment in the next block are in
        // flight while this one is processed
        int32_t beg_n = 0, end_n = 0, c_first_n = col_begin;
        if (sgi + 1 < nseg) {
          const int2 sn = l_seg[k * kMaxMerge + sgi + 1];
          beg_n = sn.x;
          end_n = sn.y;
          if (beg_n + li < end_n) c_first_n = bcol[beg_n + li];
        }
        for (int32_t c0 = beg; c0 < end; c0 += SL) {
          const bool e_ok = c0 + li < end;
          const int cnt = min(SL, end - c0);  // valid edges of this chunk (uniform in the group)
          // gathered vertex of edge c0 + li; lanes past the end point at the block's first
          // vertex (a valid, cache-resident row) and get weight 0, so the row phase below
          // needs no per-edge conditionals
          const int32_t c = e_ok ? c_next : col_begin;
          if (c0 + SL + li < end) c_next = bcol[c0 + SL + li];
          l_idx[li] = c;
          // per-edge scalars: issue the loads now, use them after the row loads are in flight
          float e_a = 0.f, a_st = 0.f;
          float4 vs = make_float4(0.f, 0.f, 1.f, 0.f);
          if (MODE == 2 && alpha_b != nullptr && e_ok) a_st = alpha_b[(int64_t)h * nnz + c0 + li];
          if (e_ok) {
            if (MODE == 2) vs = vstate[(int64_t)h * n_rows + c];  // head-major (er, m, 1/d, D) of the destination
            else e_a = STAGE ? l_el[c - col_begin] : (el_hm ? el[(int64_t)h * n_rows + c] : el[(int64_t)c * H + h]);
          }
          wave_lds_fence();
          float4 part[NA], part2[NA];
#pragma unroll
          for (int a = 0; a < NA; ++a) {
            part[a] = make_float4(0.f, 0.f, 0.f, 0.f);
            part2[a] = part[a];
          }
          float dpart = 0.f;
          float sc = 1.f;  // ONLINE: factor that brings the running sums to this chunk's maximum
#pragma unroll
          for (int t0 = 0; t0 < SL; t0 += U) {
            // the group's U gathered vertices in one go (broadcast LDS reads), then U row loads
            int idv[U];
#pragma unroll
            for (int q = 0; q < U / 4; ++q) {
              const int4 i4 = *reinterpret_cast<const int4*>(l_idx + t0 + 4 * q);
              idv[4 * q] = i4.x; idv[4 * q + 1] = i4.y; idv[4 * q + 2] = i4.z; idv[4 * q + 3] = i4.w;
            }
            // SKIP: quadruples of gathered rows that lie entirely past the end of the segment are
            // skipped (a padded load costs the texture path as much as a real one, and the sparse
            // blocks' segments are mostly shorter than a chunk).  The branches keep the compiler
            // from issuing the second half of a chunk's loads before the first half's arithmetic;
            // rows cut into four or more slices gain 1-2 % overall, rows cut into two lose 10 %
            // (measured), so the host instantiates SKIP only for the former.
            uint4 rowv[U];  // 16 bytes of the gathered row: 4 floats, or 8 halves
#pragma unroll
            for (int t4 = 0; t4 < U; t4 += 4) {
              if (!SKIP || t0 + t4 < cnt) {
                if (narrow) {
#pragma unroll
                  for (int t = t4; t < t4 + 4; ++t)
                    rowv[t] = *reinterpret_cast<const uint4*>(
                        feat_bytes + (__umul24((uint32_t)idv[t], row_bytes) + col_bytes));
                } else {
#pragma unroll
                  for (int t = t4; t < t4 + 4; ++t)
                    rowv[t] = *reinterpret_cast<const uint4*>(feat_bytes +
                                                              ((int64_t)idv[t] * row_bytes + col_bytes));
                }
              }
            }
            if (t0 == 0) {
              float p = 0.f, p2 = 0.f;
              if (e_ok) {
                if (MODE == 2) {
                  if (alpha_b != nullptr) {  // read back instead of recomputed; D[v] is still gathered
                    p = fabsf(a_st);
                    p2 = a_st > 0.f ? p : dm.slope * p;
                  } else {
                    const float raw = r_a + vs.x;
                    p = __expf(leaky(raw, dm.slope) - vs.y) * vs.z;
                    p2 = raw > 0.f ? p : dm.slope * p;
                  }
                  s_run = fmaf(p2, vs.w, s_run);
                } else if (!ONLINE) {
                  const float raw = e_a + r_a;
                  p = __expf(leaky(raw, dm.slope) - r_m) * r_invd;
                  p = raw > 0.f ? p : dm.slope * p;  // MODE 1
                  s_run += p;
                }
              }
              if (ONLINE) {
                const float raw = e_a + r_a;
                const float sc_e = e_ok ? leaky(raw, dm.slope) : -INFINITY;
                const float m_new = fmaxf(m_run, group_max_from<SL>(sc_e, 1));  // finite: lane 0 of a chunk is valid
                sc = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
                p = e_ok ? __expf(sc_e - m_new) : 0.f;
                p2 = raw > 0.f ? p : dm.slope * p;
                d_lane = fmaf(d_lane, sc, p);
                s2_lane = fmaf(s2_lane, sc, p2);
                m_run = m_new;
              }
              l_p[li] = p;
              if (DUAL || SRC) l_p2[li] = p2;
              wave_lds_fence();
            }
            float pv[U], pv2[U];
#pragma unroll
            for (int q = 0; q < U / 4; ++q) {
              const float4 p4 = *reinterpret_cast<const float4*>(l_p + t0 + 4 * q);
              pv[4 * q] = p4.x; pv[4 * q + 1] = p4.y; pv[4 * q + 2] = p4.z; pv[4 * q + 3] = p4.w;
              if (DUAL || SRC) {
                const float4 q4 = *reinterpret_cast<const float4*>(l_p2 + t0 + 4 * q);
                pv2[4 * q] = q4.x; pv2[4 * q + 1] = q4.y; pv2[4 * q + 2] = q4.z; pv2[4 * q + 3] = q4.w;
              }
            }
#pragma unroll
            for (int t4 = 0; t4 < U; t4 += 4) {
              if (!SKIP || t0 + t4 < cnt) {
#pragma unroll
                for (int t = t4; t < t4 + 4; ++t) {
                  if constexpr (HALF) {
                    fma8_half(part, pv[t], rowv[t]);
                    if (DUAL) fma8_half(part2, pv2[t], rowv[t]);
                    if constexpr (SRC && NA == 2) dpart = fmaf(pv2[t], dot8_half(acc2, rowv[t]), dpart);
                  } else {
                    const float4 rv = make_float4(__uint_as_float(rowv[t].x), __uint_as_float(rowv[t].y),
                                                  __uint_as_float(rowv[t].z), __uint_as_float(rowv[t].w));
                    fma4(part[0], pv[t], rv);
                    if (DUAL) fma4(part2[0], pv2[t], rv);
                    if (SRC) dpart = fmaf(pv2[t], dot4(acc2[0], rv), dpart);
                  }
                }
              }
            }
          }
#pragma unroll
          for (int a = 0; a < NA; ++a) {
            if (ONLINE) {
              fold4(acc[a], sc, part[a]);
              if (DUAL) fold4(acc2[a], sc, part2[a]);
            } else {
              add4(acc[a], part[a]);
              if (DUAL) add4(acc2[a], part2[a]);
            }
          }
          if (SRC) s_dot += dpart;
          wave_lds_fence();
        }
        beg = beg_n;
        end = end_n;
        c_next = c_first_n;
        }
        if (ONLINE) {
          const float d_tot = group_sum_from<SL>(d_lane, 1);
          const float s2_tot = MODE == 3 ? group_sum_from<SL>(s2_lane, 1) : 0.f;
          if (last) {
            // the row is complete: normalise (a row without in-edges keeps out = 0, m = 0, d = 1)
            const float inv = d_tot > 0.f ? 1.f / d_tot : 0.f;
#pragma unroll
            for (int a = 0; a < NA; ++a) {
              scale4(acc[a], inv);
              if (DUAL) scale4(acc2[a], inv);
            }
            if (leader && li == 0) {
              const int64_t rh = (int64_t)cur.row * H + h;
              m_out[rh] = d_tot > 0.f ? m_run : 0.f;
              d_out[rh] = d_tot > 0.f ? d_tot : 1.f;
              if (MODE == 3) scal_buf[rh] = s2_tot * inv;
            }
          } else if (li == 0) {
            state[(int64_t)cur.row * kSlices + slice] = make_float4(m_run, d_tot, s2_tot, 0.f);
          }
        }
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          st4_stream(acc_buf + (int64_t)cur.row * HF + col + 4 * a, acc[a]);
          if (DUAL) st4_stream(acc2_buf + (int64_t)cur.row * HF + col + 4 * a, acc2[a]);
        }
        if (MODE == 1 && leader) {
          const float tot = group_sum_from<SL>(s_run, 1);
          if (li == 0) scal_buf[(int64_t)cur.row * H + h] = cur.scal + tot;
        }
        if (SRC) {
          // this slice's share of del[u, h]; the D term is counted by one slice per head
          const float tot = group_sum_from<SL>(s_dot - (leader ? s_run : 0.f), 1);
          if (li == 0) scal_buf[(int64_t)cur.row * kSlices + slice] = cur.scal + tot;
        }
      }
      cur = nxt;
    }
    if (!STAGE) break;
    ++quad;
  }
}

// ---- all column blocks in one persistent launch: the running sums stay in LDS -------------------
// The launches of k_gat_blk pay for cache residency with a read-add-write of the rows' running
// sums (and softmax statistics) per block.  Here one 1024-thread workgroup per CU runs for the
// whole pass and keeps the state of kGatResSlots (row, slice) pairs in LDS: the running sums, the
// softmax statistics, the row's own scalars.  It takes all of them through column block 0, then
// all of them through block 1, ... ("phases"), writes each row out in the last phase and then
// takes its next rows ("generation").  Every workgroup of the chip owns the same number of rows
// per generation, dealt from the degree order one position at a time in alternating direction,
// so the workgroups carry nearly equal loads in every phase and walk the blocks in step by
// themselves; the workgroups of an XCD meet once per generation (phase_step_done: a bounded wait
// that only serves cache residency), so an L2 serves one block at a time.  Inside a workgroup the
// groups draw (row, slice) slots from an LDS counter, longest rows first.  A row's chunks are summed in the order of the launch-per-block kernels
// (blocks ascending, edges in list order), so the results do not depend on who draws what.
// MODE as k_gat_blk; one segment per phase, fp32 rows, per-edge scalars gathered from L2.
constexpr int kGatResThreads = 1024;
template <int SL, int MODE>
constexpr int kGatResSlots = (kGatResThreads / SL) * (MODE == 3 ? 4 : 8);
// LDS ints of a workgroup: sums (two for MODE 3) | state float4 | (beg, end) of two phases | rows |
// per group idx, p, p2 | two counters
template <int SL, int MODE>
constexpr int kGatResLdsInts = (MODE == 3 ? 2 : 1) * 4 * SL * kGatResSlots<SL, MODE> + 4 * kGatResSlots<SL, MODE> +
                               4 * kGatResSlots<SL, MODE> + kGatResSlots<SL, MODE> +
                               (kGatResThreads / SL) * 3 * SL + 4;

template <int SL, int MODE, bool SKIP, bool HALF, bool NARROW>
__global__ __launch_bounds__(kGatResThreads) void k_gat_res(
    int32_t n_rows, const int32_t* __restrict__ order, const int2* __restrict__ bseg /* [nblk][n_rows] */,
    const int32_t* __restrict__ bcol, const float* __restrict__ feat /* gathered rows: z or gout */,
    const float* __restrict__ rowfeat /* MODE 2: z */, const float* __restrict__ el,
    const float* __restrict__ er, const float* __restrict__ m_in, const float* __restrict__ d_in,
    const float4* __restrict__ vstate, GatDims dm, int sph, int el_hm, int32_t block_cols,
    int nblk, int ns, float* __restrict__ acc_buf, float* __restrict__ acc2_buf, float* __restrict__ scal_buf,
    float* __restrict__ m_out, float* __restrict__ d_out, int32_t* __restrict__ clock, int spin_limit, int sync_every,
    const float* __restrict__ alpha_b /* MODE 2, nullable: stashed signed softmax values, [H][nnz] in the order of
                                         bcol (the "fusion with stashing" arm) */,
    int64_t nnz) {
  constexpr int GPB = kGatResThreads / SL;
  constexpr int NSLOT = kGatResSlots<SL, MODE>;
  constexpr int R = NSLOT / GPB;
  constexpr int U = SL < 8 ? 4 : 8;
  constexpr bool DUAL = MODE == 3;
  constexpr bool SRC = MODE == 2;
  constexpr bool ONLINE = MODE == 0 || MODE == 3;
  static_assert(NSLOT <= kGatResThreads, "one thread per slot loads its metadata");
  extern __shared__ __align__(16) int lds_gr[];
  const int lane = threadIdx.x & 63;
  const int li = threadIdx.x & (SL - 1);
  const int grp = threadIdx.x / SL;
  const int slice = blockIdx.x % ns;
  const int64_t nwg = gridDim.x / ns, wg = blockIdx.x / ns;  // workgroups that serve this slice
  const int64_t ngroups = nwg * GPB;
  const int H = dm.H, HF = dm.HF;
  const int h = slice / sph;
  const bool leader = (slice % sph) == 0;  // one slice per head keeps the per-head scalars
  // a row narrower than its slice (a single slice of fewer than 64 columns): the lanes past its end
  // gather the row's first columns again (same cache line) and keep zeros where it matters
  const bool col_ok = slice * 4 * SL + 4 * li < HF;
  const int col = col_ok ? slice * 4 * SL + 4 * li : 0;

  float4* l_acc = reinterpret_cast<float4*>(lds_gr);                                   // [NSLOT][SL]
  float4* l_acc2 = l_acc + (DUAL ? SL * NSLOT : 0);                                    // [NSLOT][SL] (MODE 3)
  float4* l_state = l_acc2 + SL * NSLOT;                                               // [NSLOT]
  int2* l_seg = reinterpret_cast<int2*>(l_state + NSLOT);                              // [2][NSLOT]
  int* l_row = reinterpret_cast<int*>(l_seg + 2 * NSLOT);                              // [NSLOT]
  int* l_idx = l_row + NSLOT + grp * 3 * SL;
  float* l_p = reinterpret_cast<float*>(l_idx + SL);
  float* l_p2 = l_p + SL;
  int* l_cnt = l_row + NSLOT + GPB * 3 * SL;                                           // [2]

  const int64_t rows_per_group = (n_rows + ngroups - 1) / ngroups;
  const int ngen = (int)((rows_per_group + R - 1) / R);
  // workgroups go to the XCDs round-robin: those with the same id mod 8 share an L2
  PhaseClock pc{clock ? clock + (blockIdx.x % kXcds) * kClockStride : nullptr, (int)(gridDim.x / kXcds), spin_limit,
                false, sync_every > 0 ? sync_every : nblk};

  const bool gathers_first = ns >= 4;
  const char* feat_bytes = reinterpret_cast<const char*>(feat);
  constexpr uint32_t kElem = HALF ? 2u : 4u;  // bytes per stored element of the gathered matrix
  const uint32_t row_bytes = (uint32_t)HF * kElem, col_bytes = (uint32_t)col * kElem;
  using RowRaw = std::conditional_t<HALF, uint2, float4>;  // a lane's four columns of a gathered row
  auto widen = [](const RowRaw& r) {
    if constexpr (HALF) {
      const __half2* hh = reinterpret_cast<const __half2*>(&r);
      const float2 lo = __half22float2(hh[0]), hi = __half22float2(hh[1]);
      return make_float4(lo.x, lo.y, hi.x, hi.y);
    } else {
      return r;
    }
  };

  struct Item {
    int32_t beg, end, c_first;
    float4 zr;  // MODE 2: the row's own z slice
  };

  for (int gen = 0; gen < ngen; ++gen) {
    const int64_t j0 = gen * rows_per_group / ngen, j1 = (gen + 1) * rows_per_group / ngen;
    const int nslots = (int)(j1 - j0) * GPB;  // slot q: row at position (j0 * GPB + q) * nwg + wg (or + nwg - 1 - wg)
    // (the previous generation ended with a workgroup barrier: its tables are free)
    int64_t pos = -1;                         // thread q < nslots: position of slot q's row in the degree order
    if ((int)threadIdx.x < nslots) {
      // consecutive positions of the degree order go to consecutive workgroups, in alternating
      // direction from one round to the next, so every workgroup gets the same mix of degrees
      const int64_t r = (j0 * GPB + threadIdx.x) * nwg + ((threadIdx.x & 1) ? nwg - 1 - wg : wg);
      if (r < n_rows) pos = r;
      const int32_t row = pos >= 0 ? order[pos] : -1;
      l_row[threadIdx.x] = row;
      l_seg[threadIdx.x] = pos >= 0 ? bseg[pos] : make_int2(0, 0);
      // state: forward (m_run, d, s2, er[row]); MODE 1 (sum alpha g, er, m, 1/d); MODE 2 (del share, el[row])
      float4 stt = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row >= 0) {
        const int64_t rh = (int64_t)row * H + h;
        if (ONLINE) stt = make_float4(-INFINITY, 0.f, 0.f, er[rh]);
        else if (MODE == 1) stt = make_float4(0.f, er[rh], m_in[rh], 1.f / d_in[rh]);
        else stt = make_float4(0.f, el[rh], 0.f, 0.f);
      }
      l_state[threadIdx.x] = stt;
    }
    for (int i = threadIdx.x; i < nslots * SL; i += kGatResThreads) {
      l_acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (DUAL) l_acc2[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (threadIdx.x == 0) l_cnt[0] = 0;
    __syncthreads();  // the tables are in place

    // a group's next slot of phase p, from that phase's counter
    auto grab = [&](int p) {
      int q = 0;
      if (li == 0) q = atomicAdd(l_cnt + (p & 1), 1);
      return __shfl(q, lane & ~(SL - 1), 64);
    };
    // what a slot needs before its edge loop in phase p: bounds, first indices, (MODE 2) the row's own z
    auto fetch = [&](int p, int q) {
      Item it{0, 0, p * block_cols, make_float4(0.f, 0.f, 0.f, 0.f)};
      if (q >= nslots) return it;
      const int2 sg = l_seg[(p & 1) * NSLOT + q];
      it.beg = sg.x;
      it.end = sg.y;
      if (it.beg + li < it.end) it.c_first = bcol[it.beg + li];
      if (SRC) {
        const int32_t row = l_row[q];
        if (row >= 0 && it.beg < it.end && col_ok) it.zr = ld4_stream(rowfeat + (int64_t)row * HF + col);
      }
      return it;
    };
    int q = grab(0);
    Item cur = fetch(0, q);

    for (int p = 0; p < nblk; ++p) {
      const int32_t col_begin = p * block_cols;
      const bool last = p + 1 == nblk;
      // the next phase's bounds travel while this one is worked on
      int2 seg_next = make_int2(0, 0);
      if (!last && pos >= 0) seg_next = bseg[(int64_t)(p + 1) * n_rows + pos];
      if (threadIdx.x == 0) l_cnt[(p + 1) & 1] = 0;

      while (q < nslots) {
        const int qn = grab(p);
        const Item nxt = fetch(p, qn);
        const int32_t row = l_row[q];
        const int32_t beg = cur.beg, end = cur.end;
        if (row >= 0 && (beg < end || last)) {
          const float4 stt = l_state[q];
          float4 acc = l_acc[q * SL + li], acc2 = make_float4(0.f, 0.f, 0.f, 0.f);
          if (DUAL) acc2 = l_acc2[q * SL + li];
          if (SRC) acc2 = cur.zr;
          const float r_a = ONLINE ? stt.w : stt.y;
          const float r_m = stt.z, r_invd = stt.w;  // MODE 1
          float s_run = 0.f;  // chunk-phase lanes: sum of alpha g (MODE 1), of alpha g D[v] (MODE 2)
          float s_dot = 0.f;  // MODE 2, row-phase lanes: sum of alpha g <z[u], gout[v]> over the lane's columns
          float m_run = stt.x;  // ONLINE
          float d_lane = li == 0 ? stt.y : 0.f, s2_lane = li == 0 ? stt.z : 0.f;
          int32_t c_next = cur.c_first;
          for (int32_t c0 = beg; c0 < end; c0 += SL) {
            const bool e_ok = c0 + li < end;
            const int cnt = min(SL, end - c0);
            const int32_t c = e_ok ? c_next : col_begin;
            if (c0 + SL + li < end) c_next = bcol[c0 + SL + li];
            l_idx[li] = c;
            float e_a = 0.f, a_st = 0.f;
            float4 vs = make_float4(0.f, 0.f, 1.f, 0.f);
            if (SRC && alpha_b != nullptr && e_ok) a_st = alpha_b[(int64_t)h * nnz + c0 + li];
            if (e_ok) {
              if (SRC) vs = vstate[(int64_t)h * n_rows + c];  // head-major (er, m, 1/d, D) of the destination
              else e_a = el_hm ? el[(int64_t)h * n_rows + c] : el[(int64_t)c * H + h];
            }
            wave_lds_fence();
            float4 part = make_float4(0.f, 0.f, 0.f, 0.f), part2 = part;
            float dpart = 0.f;
            float sc = 1.f;  // ONLINE: factor that brings the running sums to this chunk's maximum
#pragma unroll
            for (int t0 = 0; t0 < SL; t0 += U) {
              if (SKIP && t0 >= cnt) break;  // nothing of this chunk is left: no index or weight reads either
              int idv[U];
#pragma unroll
              for (int qq = 0; qq < U / 4; ++qq) {
                const int4 i4 = *reinterpret_cast<const int4*>(l_idx + t0 + 4 * qq);
                idv[4 * qq] = i4.x; idv[4 * qq + 1] = i4.y; idv[4 * qq + 2] = i4.z; idv[4 * qq + 3] = i4.w;
              }
              RowRaw rowv[U];
              // a wavefront that is about to issue its gathers goes first on its SIMD (measured on rows of
              // four slices: 7.29 -> 7.16 ms forward, 7.84 -> 7.77 ms source side; rows of one or two slices
              // lose 1-2 % with it)
              if (gathers_first) __builtin_amdgcn_s_setprio(3);
#pragma unroll
              for (int t4 = 0; t4 < U; t4 += 4) {
                if (!SKIP || t0 + t4 < cnt) {
                  if constexpr (NARROW) {  // 32-bit byte offsets from a scalar base reach every row
#pragma unroll
                    for (int t = t4; t < t4 + 4; ++t)
                      rowv[t] = *reinterpret_cast<const RowRaw*>(
                          feat_bytes + (__umul24((uint32_t)idv[t], row_bytes) + col_bytes));
                  } else {
#pragma unroll
                    for (int t = t4; t < t4 + 4; ++t)
                      rowv[t] = *reinterpret_cast<const RowRaw*>(feat_bytes + ((int64_t)idv[t] * row_bytes + col_bytes));
                  }
                }
              }
              if (gathers_first) __builtin_amdgcn_s_setprio(0);
              if (t0 == 0) {
                float pe = 0.f, pe2 = 0.f;
                if (e_ok) {
                  if (SRC) {
                    if (alpha_b != nullptr) {  // read back instead of recomputed; D[v] is still gathered
                      pe = fabsf(a_st);
                      pe2 = a_st > 0.f ? pe : dm.slope * pe;
                    } else {
                      const float raw = r_a + vs.x;
                      pe = __expf(leaky(raw, dm.slope) - vs.y) * vs.z;
                      pe2 = raw > 0.f ? pe : dm.slope * pe;
                    }
                    s_run = fmaf(pe2, vs.w, s_run);
                  } else if (!ONLINE) {
                    const float raw = e_a + r_a;
                    pe = __expf(leaky(raw, dm.slope) - r_m) * r_invd;
                    pe = raw > 0.f ? pe : dm.slope * pe;  // MODE 1
                    s_run += pe;
                  }
                }
                if (ONLINE) {
                  const float raw = e_a + r_a;
                  const float sc_e = e_ok ? leaky(raw, dm.slope) : -INFINITY;
                  const float m_new = fmaxf(m_run, group_max_from<SL>(sc_e, 1));  // finite: lane 0 of a chunk is valid
                  sc = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
                  pe = e_ok ? __expf(sc_e - m_new) : 0.f;
                  pe2 = raw > 0.f ? pe : dm.slope * pe;
                  d_lane = fmaf(d_lane, sc, pe);
                  s2_lane = fmaf(s2_lane, sc, pe2);
                  m_run = m_new;
                }
                l_p[li] = pe;
                if (DUAL || SRC) l_p2[li] = pe2;
                wave_lds_fence();
              }
              float pv[U], pv2[U];
#pragma unroll
              for (int qq = 0; qq < U / 4; ++qq) {
                const float4 p4 = *reinterpret_cast<const float4*>(l_p + t0 + 4 * qq);
                pv[4 * qq] = p4.x; pv[4 * qq + 1] = p4.y; pv[4 * qq + 2] = p4.z; pv[4 * qq + 3] = p4.w;
                if (DUAL || SRC) {
                  const float4 q4 = *reinterpret_cast<const float4*>(l_p2 + t0 + 4 * qq);
                  pv2[4 * qq] = q4.x; pv2[4 * qq + 1] = q4.y; pv2[4 * qq + 2] = q4.z; pv2[4 * qq + 3] = q4.w;
                }
              }
#pragma unroll
              for (int t4 = 0; t4 < U; t4 += 4) {
                if (!SKIP || t0 + t4 < cnt) {
#pragma unroll
                  for (int t = t4; t < t4 + 4; ++t) {
                    const float4 rv = widen(rowv[t]);
                    fma4(part, pv[t], rv);
                    if (DUAL) fma4(part2, pv2[t], rv);
                    if (SRC) dpart = fmaf(pv2[t], dot4(acc2, rv), dpart);
                  }
                }
              }
            }
            if (ONLINE) {
              fold4(acc, sc, part);
              if (DUAL) fold4(acc2, sc, part2);
            } else {
              add4(acc, part);
            }
            if (SRC) s_dot += dpart;
            wave_lds_fence();
          }
          // close the item: statistics back to the slot, or (last phase) the finished row to memory
          float4 st_new = stt;
          if (ONLINE) {
            const float d_tot = group_sum_from<SL>(d_lane, 1);
            const float s2_tot = MODE == 3 ? group_sum_from<SL>(s2_lane, 1) : 0.f;
            st_new = make_float4(m_run, d_tot, s2_tot, stt.w);
            if (last) {
              // the row is complete: normalise (a row without in-edges keeps out = 0, m = 0, d = 1)
              const float inv = d_tot > 0.f ? 1.f / d_tot : 0.f;
              scale4(acc, inv);
              if (DUAL) scale4(acc2, inv);
              if (leader && li == 0) {
                const int64_t rh = (int64_t)row * H + h;
                m_out[rh] = d_tot > 0.f ? m_run : 0.f;
                d_out[rh] = d_tot > 0.f ? d_tot : 1.f;
                if (MODE == 3) scal_buf[rh] = s2_tot * inv;
              }
            }
          } else if (MODE == 1) {
            if (leader) st_new.x = stt.x + group_sum_from<SL>(s_run, 1);
            if (last && leader && li == 0) scal_buf[(int64_t)row * H + h] = st_new.x;
          } else {
            // this slice's share of del[u, h]; the D term is counted by one slice per head
            st_new.x = stt.x + group_sum_from<SL>(s_dot - (leader ? s_run : 0.f), 1);
            if (last && li == 0) scal_buf[(int64_t)row * kSlices + slice] = st_new.x;
          }
          if (last) {
            if (col_ok) {
              st4_stream(acc_buf + (int64_t)row * HF + col, acc);
              if (DUAL) st4_stream(acc2_buf + (int64_t)row * HF + col, acc2);
            }
          } else {
            l_acc[q * SL + li] = acc;
            if (DUAL) l_acc2[q * SL + li] = acc2;
            if (li == 0) l_state[q] = st_new;
          }
        }
        q = qn;
        cur = nxt;
      }
      if ((int)threadIdx.x < nslots) l_seg[((p + 1) & 1) * NSLOT + threadIdx.x] = seg_next;
      __syncthreads();  // the workgroup is done with this block; the next phase's bounds are in LDS
      if (!last) {      // first slot of the next phase: its loads travel during the wait below
        q = grab(p + 1);
        cur = fetch(p + 1, q);
      }
      phase_step_done(pc, gen * nblk + p);
      __syncthreads();  // every workgroup of the XCD is done with this block (or the wait ran out)

    }
  }
}

__global__ void k_gat_zero_clock(int32_t* __restrict__ clock) { clock[threadIdx.x] = 0; }

// elT[h][v] = el[v][h]: a column block of gathered vertices then spans 4 B per vertex in
// the head a slice needs instead of 4*H (fewer L2 lines for the per-edge scalar gathers)
__global__ void k_gat_head_major(int64_t n, int H, const float* __restrict__ a, float* __restrict__ aT) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;  // index into aT
  if (i >= n * H) return;
  const int64_t h = i / n, v = i - h * n;
  aT[i] = a[v * H + h];
}

static gnn_status_t head_major(const gnn_graph_t* g, int H, const float* a, float* aT, hipStream_t st) {
  ProfScope p("gat_head_major", st);
  const int64_t cnt = (int64_t)g->n * H;
  k_gat_head_major<<<(unsigned)cdiv(cnt, 256), 256, 0, st>>>(g->n, H, a, aT);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

// ---- host side -------------------------------------------------------------------------
// fp16 copy of the gathered matrix (configuration key "gather_precision" = 1): rows of 2*HF bytes
// are cut into slices of 64 columns (one 128-byte line), each inside one head
bool gat_blocked_half(const gnn_graph_t* g, int heads, int f) {
  if (config_get(kCfgGatherPrecision) != 1 || !gat_blocked_applies(g, heads, f)) return false;
  const int HF = heads * f;
  if (HF % 64 != 0 || HF < 128) return false;
  const int q = HF / 64;
  return (q == 1 || q == 2 || q == 4 || q == 8) && q % heads == 0;
}

__global__ void k_to_half(int64_t quads, const float* __restrict__ src, __half* __restrict__ dst) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= quads) return;
  const float4 v = ld4(src + 4 * i);
  __half2* o = reinterpret_cast<__half2*>(dst + 4 * i);
  o[0] = __floats2half2_rn(v.x, v.y);
  o[1] = __floats2half2_rn(v.z, v.w);
}

static gnn_status_t to_half(const gnn_graph_t* g, int HF, const float* src, void* dst, hipStream_t st) {
  ProfScope p("gat_to_half", st);
  const int64_t quads = (int64_t)g->n * (HF / 4);
  k_to_half<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(quads, src, static_cast<__half*>(dst));
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

bool gat_blocked_applies(const gnn_graph_t* g, int heads, int f) {
  if (!g->blocked_pays() || config_get(kCfgForceSimple)) return false;
  const int HF = heads * f;
  Slicing sl;
  return pick_slicing(heads, HF, sl);
}

size_t gat_blocked_ws_bytes(const gnn_graph_t* g, int heads, int f) {
  if (!gat_blocked_applies(g, heads, f)) return 0;
  return ws_granule(sizeof(float) * (size_t)g->n * heads * f) +   // T, then A2
         ws_granule(sizeof(float) * (size_t)g->n * kSlices) +     // sg, then the slices' shares of del
         ws_granule(sizeof(float) * (size_t)g->n * heads);        // head-major el
}

__global__ void k_zero_i32(int n, int32_t* __restrict__ p) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// LDS bytes of the staged kernel: per-group scratch plus the block's table
template <int SL>
static size_t staged_lds_bytes(int64_t block_cols) {
  constexpr int GS = kBlkGroupFloats<SL>;
  return sizeof(float) * ((size_t)(kStageThreads / SL) * GS + (size_t)block_cols);
}
constexpr size_t kStageLdsLimit = 152 * 1024;  // of the 160 KB a CU has
constexpr int kStageMinEdgesPerRow = 48;        // mean edges per row of a block worth staging

// Name of a launch's timed bracket: the kernel's name, or "name#i" for the i-th launch of a pass
// when the environment variable GNN_PROF_PER_LAUNCH is set (for tuning the launch groups).
static const char* bracket_name(const char* name, size_t launch) {
  static const bool per_launch = std::getenv("GNN_PROF_PER_LAUNCH") != nullptr;
  if (!per_launch) return name;
  static std::mutex mu;
  static std::map<std::string, std::string> names;  // node addresses are stable
  std::lock_guard<std::mutex> lock(mu);
  std::string key = std::string(name) + "#" + std::to_string(launch);
  return names.emplace(key, key).first->second.c_str();
}

template <int SL, int MODE, bool HALF, bool SKIP>
static gnn_status_t launch_blocks_impl(const gnn_graph_t* g, int side, const char* name, GatDims dm,
                                  int el_hm, const float* feat, const float* rowfeat,
                                  const float* el, const float* er, const float* m, const float* d,
                                  const float4* vstate, float* acc, float* acc2, float* scal,
                                  int32_t* queue, float4* state, float* m_out, float* d_out, hipStream_t st,
                                  const float* alpha_b = nullptr) {
  const int ns = dm.HF / ((HALF ? 8 : 4) * SL);
  const int sph = ns / dm.H;
  // 32-bit byte offsets (and 24-bit multiplies) reach every gathered row
  const int narrow = (int64_t)g->n * dm.HF * 4 < ((int64_t)1 << 32) && g->n < (1 << 24) &&
                     !config_get(kCfgWideOffsets);
  constexpr int GS = kBlkGroupFloats<SL>;
  const int rows_per_wg = (kBlkThreads / SL) * kRowsPerGroup;
  const unsigned grid = (unsigned)(cdiv(g->n, rows_per_wg) * ns);
  const size_t lds = sizeof(float) * (size_t)(kBlkThreads / SL) * GS;
  bool stage_ok = false;
  if constexpr (MODE != 2) {
    stage_ok = queue != nullptr && el_hm && (int)g->h_block_begin[side].size() == g->nblk + 1;
    if (stage_ok) {
      // more than 64 KB of dynamic LDS needs the attribute; once per instantiation (the call is
      // idempotent, so a race between two first callers is harmless)
      static std::atomic<bool> attr_set{false};
      if (!attr_set.load(std::memory_order_acquire)) {
        GNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gat_blk<SL, MODE, true, HALF, SKIP>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStageLdsLimit));
        attr_set.store(true, std::memory_order_release);
      }
      ProfScope p("gat_blk_queue_reset", st);
      k_zero_i32<<<cdiv(g->nblk * kSlices, 64), 64, 0, st>>>(g->nblk * kSlices, queue);
      GNN_LAUNCH_CHECK();
    }
  }
  const std::vector<int32_t>& groups = g->h_group[side][(MODE == 2 || MODE == 3) ? 1 : 0];
  GNN_REQUIRE(groups.size() >= 2 && groups.front() == 0 && groups.back() == g->nblk, GNN_ERR_UNSUPPORTED,
              "gat blocked: the plan has no launch groups");
  for (size_t gi = 0; gi + 1 < groups.size(); ++gi) {
    const int b = groups[gi], b_end = groups[gi + 1], nseg = b_end - b;
    GNN_REQUIRE(nseg >= 1 && nseg <= kMaxMerge, GNN_ERR_UNSUPPORTED, "gat blocked: bad launch group");
    const int2* bseg_b = reinterpret_cast<const int2*>(g->bseg[side]) + (int64_t)b * g->n;
    const int32_t col_begin = b * g->block_cols;
    bool staged = false;
    if constexpr (MODE != 2) {
      // The LDS table pays on blocks whose rows are long (measured with 20480 columns: 2.7 ms
      // instead of 3.5 ms at 220 edges per row, 1.28 instead of 1.43 ms at 67, no difference at
      // 42); the persistent launch has a higher fixed cost, which sparser blocks do not repay.
      const int64_t edges = (int64_t)g->h_block_begin[side][b_end] - g->h_block_begin[side][b];
      const int64_t cols_wide = (int64_t)nseg * g->block_cols;
      const size_t stage_bytes = staged_lds_bytes<SL>(cols_wide);
      staged = stage_ok && stage_bytes <= kStageLdsLimit && edges >= (int64_t)kStageMinEdgesPerRow * g->n;
      if (staged) {
        const int32_t cols_here = (int32_t)(g->n - col_begin < cols_wide ? g->n - col_begin : cols_wide);
        // one persistent workgroup per CU, a multiple of 8 so that every XCD serves one slice
        const unsigned pgrid = (unsigned)(device_cu_count() / kSlices * kSlices);
        ProfScope p(bracket_name(name, gi), st);  // one timed bracket per launch
        k_gat_blk<SL, MODE, true, HALF, SKIP><<<pgrid, kStageThreads, stage_bytes, st>>>(
            g->n, g->order[side], bseg_b, g->bcol[side], feat, rowfeat, el, er, m, d, vstate, col_begin, dm, sph,
            b == 0, narrow, el_hm, acc, acc2, scal, queue + b * kSlices, cols_here, 1, ns, b_end == g->nblk, state,
            m_out, d_out, nseg, alpha_b, g->nnz);
        GNN_LAUNCH_CHECK();
      }
    }
    if (!staged) {
      ProfScope p(bracket_name(name, gi), st);  // one timed bracket per launch
      k_gat_blk<SL, MODE, false, HALF, SKIP><<<grid, kBlkThreads, lds, st>>>(
          g->n, g->order[side], bseg_b, g->bcol[side], feat, rowfeat, el, er, m, d, vstate, col_begin, dm, sph,
          b == 0, narrow, el_hm, acc, acc2, scal, nullptr, 0, 1, ns, b_end == g->nblk, state, m_out, d_out, nseg,
          alpha_b, g->nnz);
      GNN_LAUNCH_CHECK();
    }
  }
  return GNN_OK;
}

template <int SL, int MODE, bool HALF = false>
static gnn_status_t launch_blocks(const gnn_graph_t* g, int side, const char* name, GatDims dm,
                                  int el_hm, const float* feat, const float* rowfeat,
                                  const float* el, const float* er, const float* m, const float* d,
                                  const float4* vstate, float* acc, float* acc2, float* scal,
                                  int32_t* queue, float4* state, float* m_out, float* d_out, hipStream_t st,
                                  const float* alpha_b = nullptr) {
  const int ns = dm.HF / ((HALF ? 8 : 4) * SL);
  // the fp16 variant (one sub-iteration per chunk) measured 3 % slower with the skip
  if (ns >= 4 && !HALF)
    return launch_blocks_impl<SL, MODE, HALF, true>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2,
                                                    scal, queue, state, m_out, d_out, st, alpha_b);
  return launch_blocks_impl<SL, MODE, HALF, false>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2,
                                                   scal, queue, state, m_out, d_out, st, alpha_b);
}

// The persistent kernel applies to rows cut into slices of 64 columns (256 bytes of fp32, or one
// 128-byte line of an fp16 copy)
static bool gat_resident_applies(const gnn_graph_t* g, GatDims dm) {
  if (!config_get(kCfgResidentSums) || g->phase_clock == nullptr) return false;
  Slicing sl;
  return pick_slicing(dm.H, dm.HF, sl) && sl.SL == 16;
}

template <int MODE, bool SKIP, bool HALF, bool NARROW>
static gnn_status_t launch_resident_addr(const gnn_graph_t* g, int side, const char* name, GatDims dm, int el_hm,
                                         const float* feat, const float* rowfeat, const float* el, const float* er,
                                         const float* m, const float* d, const float4* vstate, float* acc,
                                         float* acc2, float* scal, float* m_out, float* d_out, hipStream_t st,
                                         const float* alpha_b) {
  constexpr int SL = 16;
  const int ns = dm.HF <= 4 * SL ? 1 : dm.HF / (4 * SL);
  const int sph = ns / dm.H;
  const size_t lds = sizeof(int) * (size_t)kGatResLdsInts<SL, MODE>;
  static_assert(sizeof(int) * (size_t)kGatResLdsInts<SL, MODE> <= 160 * 1024, "the slots must fit the LDS of a CU");
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_acquire)) {
    GNN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(k_gat_res<SL, MODE, SKIP, HALF, NARROW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set.store(true, std::memory_order_release);
  }
  // one workgroup per CU, a multiple of 8 so that every XCD serves one slice
  const unsigned grid = (unsigned)(device_cu_count() / kXcds * kXcds);
  ProfScope p(name, st);
  k_gat_zero_clock<<<1, kXcds * kClockStride, 0, st>>>(g->phase_clock);
  GNN_LAUNCH_CHECK();
  k_gat_res<SL, MODE, SKIP, HALF, NARROW><<<grid, kGatResThreads, lds, st>>>(
      g->n, g->order[side], reinterpret_cast<const int2*>(g->bseg[side]), g->bcol[side], feat, rowfeat, el, er, m, d,
      vstate, dm, sph, el_hm, g->block_cols, g->nblk, ns, acc, acc2, scal, m_out, d_out, g->phase_clock,
      (int)config_get(kCfgResidentSpin), (int)config_get(kCfgResidentSyncEvery), alpha_b, g->nnz);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

// 32-bit byte offsets (and 24-bit multiplies) reach every gathered row
static bool gat_resident_narrow(const gnn_graph_t* g, GatDims dm) {
  return (int64_t)g->n * dm.HF * 4 < ((int64_t)1 << 32) && g->n < (1 << 24) && !config_get(kCfgWideOffsets);
}

template <int MODE, bool SKIP, bool HALF>
static gnn_status_t launch_resident_impl(const gnn_graph_t* g, int side, const char* name, GatDims dm, int el_hm,
                                         const float* feat, const float* rowfeat, const float* el, const float* er,
                                         const float* m, const float* d, const float4* vstate, float* acc,
                                         float* acc2, float* scal, float* m_out, float* d_out, hipStream_t st,
                                         const float* alpha_b) {
  if (gat_resident_narrow(g, dm))
    return launch_resident_addr<MODE, SKIP, HALF, true>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate,
                                                        acc, acc2, scal, m_out, d_out, st, alpha_b);
  return launch_resident_addr<MODE, SKIP, HALF, false>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate,
                                                       acc, acc2, scal, m_out, d_out, st, alpha_b);
}

template <int MODE>
static gnn_status_t launch_resident(const gnn_graph_t* g, int side, const char* name, GatDims dm, int el_hm,
                                    const float* feat, const float* rowfeat, const float* el, const float* er,
                                    const float* m, const float* d, const float4* vstate, float* acc, float* acc2,
                                    float* scal, float* m_out, float* d_out, hipStream_t st, const float* alpha_b,
                                    bool half_feat) {
  if (half_feat) {
    if constexpr (MODE != 1)
      return launch_resident_impl<MODE, true, true>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc,
                                                    acc2, scal, m_out, d_out, st, alpha_b);
  }
  // gathers past a segment's end are skipped on rows of four and more slices; on narrower rows the
  // source side gains from it as well (6.48 -> 6.14 ms for the two layers of a 128 / 44-wide model at
  // Reddit scale), the forward modes lose a little (5.87 -> 5.96 ms)
  if (dm.HF / 64 >= 4 || MODE == 2)
    return launch_resident_impl<MODE, true, false>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2,
                                            scal, m_out, d_out, st, alpha_b);
  return launch_resident_impl<MODE, false, false>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2,
                                           scal, m_out, d_out, st, alpha_b);
}

template <int MODE>
static gnn_status_t run_blocks(const gnn_graph_t* g, int side, const char* name, GatDims dm,
                               int el_hm, const float* feat, const float* rowfeat, const float* el, const float* er, const float* m,
                               const float* d, const float4* vstate, float* acc, float* acc2,
                               float* scal, int32_t* queue, float4* state, float* m_out, float* d_out,
                               hipStream_t st, bool half_feat = false, const float* alpha_b = nullptr) {
  if (gat_resident_applies(g, dm))
    return launch_resident<MODE>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2, scal,
                                 m_out, d_out, st, alpha_b, half_feat);
  if (half_feat) {
    if constexpr (MODE != 1)
      return launch_blocks<8, MODE, true>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2, scal,
                                          queue, state, m_out, d_out, st, alpha_b);
  }
  Slicing sl;
  if (!pick_slicing(dm.H, dm.HF, sl)) sl.SL = 0;
  GNN_REQUIRE(sl.SL == 0 || dm.HF >= 128, GNN_ERR_UNSUPPORTED,
              "gat blocked: rows of one slice are served by the persistent kernels only");
  switch (sl.SL) {
    case 4: return launch_blocks<4, MODE>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2, scal, queue, state, m_out, d_out, st, alpha_b);
    case 8: return launch_blocks<8, MODE>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2, scal, queue, state, m_out, d_out, st, alpha_b);
    case 16: return launch_blocks<16, MODE>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2, scal, queue, state, m_out, d_out, st, alpha_b);
    case 32: return launch_blocks<32, MODE>(g, side, name, dm, el_hm, feat, rowfeat, el, er, m, d, vstate, acc, acc2, scal, queue, state, m_out, d_out, st, alpha_b);
  }
  set_error("gat blocked: unsupported slice width");
  return GNN_ERR_UNSUPPORTED;
}

gnn_status_t gat_blocked_fwd(const gnn_graph_t* g, GatDims dm, const float* z, const float* el,
                             const float* er, float* m, float* d, float* out, float* t, float* sg,
                             float* el_t, int32_t* queue, float4* state, void* half_buf, hipStream_t st) {
  if (el_t) GNN_TRY(head_major(g, dm.H, el, el_t, st));
  if (!config_get(kCfgLdsScalarTable)) queue = nullptr;
  const float* el_use = el_t ? el_t : el;
  const int hm = el_t != nullptr;
  const bool half = half_buf != nullptr && gat_blocked_half(g, dm.H, dm.F);
  const float* feat = z;
  if (half) {  // the rows the edges gather come from an fp16 copy; el, er were made from the fp32 rows
    GNN_TRY(to_half(g, dm.HF, z, half_buf, st));
    feat = static_cast<const float*>(half_buf);
  }
  if (t)
    return run_blocks<3>(g, 0, "gat_fwd_fused", dm, hm, feat, nullptr, el_use, er, nullptr, nullptr, nullptr, out, t, sg,
                         queue, state, m, d, st, half);
  return run_blocks<0>(g, 0, "gat_fwd_fused", dm, hm, feat, nullptr, el_use, er, nullptr, nullptr, nullptr, out, nullptr,
                       nullptr, queue, state, m, d, st, half);
}

gnn_status_t gat_blocked_bwd_dst(const gnn_graph_t* g, GatDims dm, const float* z, const float* el,
                                 const float* er, const float* m, const float* d, const float* out,
                                 const float* gout, float* der, float4* vstate, float* t_buf,
                                 float* sg_buf, float* el_t, int32_t* queue, hipStream_t st) {
  if (el_t) GNN_TRY(head_major(g, dm.H, el, el_t, st));
  if (!config_get(kCfgLdsScalarTable)) queue = nullptr;
  GNN_TRY(run_blocks<1>(g, 0, "gat_bwd_dst", dm, el_t != nullptr, z, nullptr, el_t ? el_t : el, er, m, d, nullptr,
                        t_buf, nullptr, sg_buf, queue, nullptr, nullptr, nullptr, st));
  return gat_dst_finish(g, dm, gout, t_buf, out, sg_buf, er, m, d,
                        kDstHeadMajor | (gat_blocked_half(g, dm.H, dm.F) ? kDstHalfGout : 0), der, vstate, st);
}

// dz[u,h,:] += a_l[h,:] del[u,h] + a_r[h,:] der[u,h], with del[u,h] = the sum of the shares its
// slices left in sd ([n][8], slice-major inside a vertex); one thread per float4 of dz
__global__ void k_gat_src_finish_blk(int64_t n, GatDims dm, int ns, const float* __restrict__ sd,
                                     const float* __restrict__ der, const float* __restrict__ a_l,
                                     const float* __restrict__ a_r, float* __restrict__ dz,
                                     float* __restrict__ del) {
  const int qpr = dm.HF / 4;  // float4 per row
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n * qpr) return;
  const int64_t u = i / qpr;
  const int col = 4 * (int)(i - u * qpr);
  const int h = col / dm.F, sph = ns / dm.H;
  float dl = 0.f;
  for (int s = 0; s < sph; ++s) dl += sd[u * kSlices + h * sph + s];  // fixed order
  if (col == h * dm.F) del[u * dm.H + h] = dl;
  float4 o = ld4(dz + u * dm.HF + col);
  fma4(o, dl, ld4(a_l + col));
  fma4(o, der[u * dm.H + h], ld4(a_r + col));
  st4(dz + u * dm.HF + col, o);
}

// The per-edge stash of the "fusion with stashing" arm in the order the source-side kernel walks:
// alpha_b[h][q] for position q of the source side's blocked edge list = softmax value of that edge
// with the sign of its raw score.  One 16-lane group per source row, its segments block by block.
__global__ __launch_bounds__(256) void k_gat_stash_alpha_blk(
    int32_t n, int32_t nblk, int64_t nnz, int H, float slope, const int32_t* __restrict__ bptr,
    const int32_t* __restrict__ bcol, const float* __restrict__ el, const float* __restrict__ er,
    const float* __restrict__ m, const float* __restrict__ d, float* __restrict__ alpha_b) {
  const int li = threadIdx.x & 15;
  const int64_t u = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 4;
  if (u >= n) return;
  for (int b = 0; b < nblk; ++b) {
    const int32_t beg = bptr[(int64_t)b * n + u], end = bptr[(int64_t)b * n + u + 1];
    for (int32_t q = beg + li; q < end; q += 16) {
      const int64_t v = bcol[q];
      for (int h = 0; h < H; ++h) {
        const float raw = el[u * H + h] + er[v * H + h];
        const float a = __expf(leaky(raw, slope) - m[v * H + h]) / d[v * H + h];
        alpha_b[(int64_t)h * nnz + q] = raw > 0.f ? a : -a;
      }
    }
  }
}

gnn_status_t gat_blocked_stash_alpha(const gnn_graph_t* g, int H, float slope, const float* el, const float* er,
                                     const float* m, const float* d, float* alpha_b, hipStream_t st) {
  ProfScope p("gat_stash_alpha", st);
  k_gat_stash_alpha_blk<<<(unsigned)cdiv((int64_t)g->n * 16, 256), 256, 0, st>>>(
      g->n, g->nblk, g->nnz, H, slope, g->bptr[1], g->bcol[1], el, er, m, d, alpha_b);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

gnn_status_t gat_blocked_bwd_src(const gnn_graph_t* g, GatDims dm, const float* z, const float* el,
                                 const float4* vstate, const float* der, const float* gout,
                                 const float* a_l, const float* a_r, float* dz, float* del,
                                 float* sd_buf /* [n][8] scratch */, void* half_buf, hipStream_t st,
                                 const float* alpha_b) {
  const bool half = half_buf != nullptr && gat_blocked_half(g, dm.H, dm.F);
  const float* feat = gout;
  if (half) {
    GNN_TRY(to_half(g, dm.HF, gout, half_buf, st));
    feat = static_cast<const float*>(half_buf);
  }
  GNN_TRY(run_blocks<2>(g, 1, "gat_bwd_src", dm, 0, feat, z, el, nullptr, nullptr, nullptr, vstate, dz,
                        nullptr, sd_buf, nullptr, nullptr, nullptr, nullptr, st, half, alpha_b));
  Slicing sl;
  int ns = 0;
  if (half) ns = dm.HF / 64;
  else if (pick_slicing(dm.H, dm.HF, sl)) ns = sl.ns;
  GNN_REQUIRE(ns >= dm.H && ns % dm.H == 0 && ns <= kSlices, GNN_ERR_UNSUPPORTED, "gat blocked: bad slicing");
  ProfScope p("gat_bwd_src_finish", st);
  const int64_t quads = (int64_t)g->n * (dm.HF / 4);
  k_gat_src_finish_blk<<<(unsigned)cdiv(quads, 256), 256, 0, st>>>(g->n, dm, ns, sd_buf, der, a_l, a_r, dz, del);
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

}  // namespace gnn

// Which instantiation of the column-blocked kernel a pass launches for this graph and shape
// (the persistent kernel, or the plain, not LDS-staged variant of the launch-per-block kernel),
// spelled as a profiler prints it; "" when the single-launch kernels run instead.  Lets a measurement script check that stored counter readings belong to
// the kernel it times.
extern "C" gnn_status_t gnn_gat_blocked_kernel_name(const gnn_graph_t* g, int heads, int f, int mode,
                                                    char* buf, size_t len) {
  using namespace gnn;
  clear_error();
  GNN_REQUIRE(g != nullptr && buf != nullptr && len > 0, GNN_ERR_INVALID_ARG,
              "gnn_gat_blocked_kernel_name: null argument");
  GNN_REQUIRE(mode >= 0 && mode <= 3, GNN_ERR_INVALID_ARG, "gnn_gat_blocked_kernel_name: mode must be 0..3");
  buf[0] = 0;
  if (heads <= 0 || f <= 0 || !gat_blocked_applies(g, heads, f)) return GNN_OK;
  const bool half = mode != 1 && gat_blocked_half(g, heads, f);
  Slicing sl;
  if (!pick_slicing(heads, heads * f, sl)) return GNN_OK;
  if (gat_resident_applies(g, make_dims(heads, f, 0.2f))) {
    std::snprintf(buf, len, "k_gat_res<16, %d, %s, %s, %s>", mode,
                  (half || heads * f / 64 >= 4 || mode == 2) ? "true" : "false", half ? "true" : "false",
                  gat_resident_narrow(g, make_dims(heads, f, 0.2f)) ? "true" : "false");
    return GNN_OK;
  }
  const int SL = half ? 8 : sl.SL;
  const int ns = heads * f / ((half ? 8 : 4) * SL);
  std::snprintf(buf, len, "k_gat_blk<%d, %d, false, %s, %s>", SL, mode, half ? "true" : "false",
                (ns >= 4 && !half) ? "true" : "false");
  return GNN_OK;
}
