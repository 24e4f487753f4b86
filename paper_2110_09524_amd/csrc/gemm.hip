// fp32 dense products on the MFMA matrix cores (v_mfma_f32_32x32x2_f32): the
// ExpensiveApply projections that the reorganization moves onto vertices
// (Sec. 4) and their two backward products (App. B, "Apply").
//
// Tiling: a 256-thread workgroup (4 wavefronts, 2 x 2) owns a 128 x BN tile of
// C; each wavefront owns 64 x BN/2 of it as 2 x (BN/64) MFMA 32x32 tiles held in
// accumulators.  K advances 16 at a time through LDS; both operands sit in LDS
// k-major ([k][m] and [k][n]) so every MFMA operand read is one conflict-free
// ds_read_b32 with consecutive lanes on consecutive addresses, whatever the
// operands' layout in HBM.  Global loads of the next K-slab are issued before the
// MFMAs of the current one (register prefetch).
#include "common.h"

namespace gnn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int BK = 16;
constexpr int GEMM_THREADS = 256;
constexpr int LDS_PAD = 4;  // row stride = 4 (mod 32) banks: transposing stores spread over banks

// Attention halves in the epilogue of the projection (Sec. 4, text after Eq. 1: the score splits
// into a source half <a_l, z[u]> and a destination half <a_r, z[v]>, both per-vertex): el[m, h] =
// sum_f a_l[h, f] C[m, h*F + f], er likewise, taken from the accumulators before they are stored,
// so z is not read again.  A lane holds one column of a 32-column MFMA tile, so the sum over a
// head is a butterfly over the lanes of the tile that belong to that head (F = 4, 8, 16, 32), or,
// for F = 64 with two tiles per wavefront, over both tiles and all 32 lanes.
// v + (v of the lane the DPP control pairs this lane with), one VALU operation
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true);
  return v + __int_as_float(t);
}
// Sum over aligned segments of `seg` lanes (a power of two, 1 .. 32); every lane of a segment ends
// with the segment's total.  Pairings: lane ^ 1 and lane ^ 2 inside quads, then mirrored halves
// of 8 and of 16 lanes (valid because all lanes of the smaller segment already agree), then the
// other row of 16 through the crossbar.
__device__ __forceinline__ float segment_sum(float v, int seg) {
  if (seg > 1) v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
  if (seg > 2) v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
  if (seg > 4) v = dpp_add<0x141>(v);   // row_half_mirror
  if (seg > 8) v = dpp_add<0x140>(v);   // row_mirror
  if (seg > 16) v += __shfl_xor(v, 16, 64);
  return v;
}

struct AttnEpilogue {
  const float* a_l;
  const float* a_r;
  float* el;
  float* er;
  int H, F;
};

// VEC: operands are fetched and parked in vectors, 2 floats of A and 4 floats of B per load along
// whichever dimension is contiguous in memory (needs even lda, ldb % 4 == 0, matching alignment
// and extents; the host checks).  A slab then costs a thread 6 global loads and 6 to 10 LDS
// stores instead of 16 and 16 (measured on the Reddit-scale projection: +9 % throughput).
template <int BN, bool A_KMAJOR, bool B_KCONTIG, bool EPI = false, bool VEC = false>
__global__ __launch_bounds__(GEMM_THREADS, 3) void k_gemm_f32(
    int64_t M, int N, int64_t K, const float* __restrict__ A, int64_t lda,
    const float* __restrict__ B, int64_t ldb, float* __restrict__ C, int64_t ldc,
    int64_t k_per_split, int64_t split_stride, AttnEpilogue epi) {
  constexpr int TN = BN / 64;          // MFMA tiles per wavefront along n
  constexpr int VA = VEC ? 2 : 1, VB = VEC ? 4 : 1;  // floats per load
  constexpr int A_PER_T = BM * BK / GEMM_THREADS / VA;  // loads per thread and slab
  constexpr int B_PER_T = BN * BK / GEMM_THREADS / VB;
  __shared__ __align__(16) float As[BK][BM + LDS_PAD];
  __shared__ __align__(16) float Bs[BK][BN + LDS_PAD];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm0 = (wave >> 1) * 64;
  const int wn0 = (wave & 1) * (BN / 2);
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;
  const int64_t k_begin = (int64_t)blockIdx.z * k_per_split;
  int64_t k_end = k_begin + k_per_split;
  if (k_end > K) k_end = K;

  floatx16 acc[2][TN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float ra[A_PER_T][VA], rb[B_PER_T][VB];

  // Load i of this thread covers V consecutive elements along the operand's contiguous dimension,
  // at a fixed (row, k) of the slab.  Its address is a uniform base pointer, advanced once per
  // slab, plus a 32-bit offset computed once; rows past M and columns past N are clamped to the
  // last valid one (their products land in rows / columns of C that are never stored), so only
  // the last, partial K-slab needs predicated loads.
  // position of load i inside the slab: (k, x) of its first element; k-contiguous operands are
  // vectorised along k, the others along x
  auto pos_a = [&](int i, int& kk, int& mm) {
    const int idx = tid + GEMM_THREADS * i;
    if (A_KMAJOR) { mm = VA * (idx % (BM / VA)); kk = idx / (BM / VA); }
    else { kk = VA * (idx % (BK / VA)); mm = idx / (BK / VA); }
  };
  auto pos_b = [&](int i, int& kk, int& nn) {
    const int idx = tid + GEMM_THREADS * i;
    if (B_KCONTIG) { kk = VB * (idx % (BK / VB)); nn = idx / (BK / VB); }
    else { nn = VB * (idx % (BN / VB)); kk = idx / (BN / VB); }
  };
  uint32_t offa[A_PER_T], offb[B_PER_T];
  int ka[A_PER_T], kb[B_PER_T];
#pragma unroll
  for (int i = 0; i < A_PER_T; ++i) {
    int kk, mm;
    pos_a(i, kk, mm);
    // a vector along m starts at a multiple of VA and M is one too (host check): it is either
    // whole inside the matrix or whole outside (then clamped as a whole)
    const int64_t last = A_KMAJOR ? M - VA : M - 1;
    const int64_t mrow = (m0 + mm <= last ? m0 + mm : last) - m0;
    offa[i] = (uint32_t)(A_KMAJOR ? kk * lda + mrow : mrow * lda + kk);
    ka[i] = kk;
  }
#pragma unroll
  for (int i = 0; i < B_PER_T; ++i) {
    int kk, nn;
    pos_b(i, kk, nn);
    const int last = B_KCONTIG ? N - 1 : N - VB;
    const int64_t ncol = (n0 + nn <= last ? n0 + nn : last) - n0;
    offb[i] = (uint32_t)(B_KCONTIG ? ncol * ldb + kk : kk * ldb + ncol);
    kb[i] = kk;
  }
  const float* abase = A + (A_KMAJOR ? k_begin * lda + m0 : m0 * lda + k_begin);
  const float* bbase = B + (B_KCONTIG ? (int64_t)n0 * ldb + k_begin : k_begin * ldb + n0);
  const int64_t astep = A_KMAJOR ? BK * lda : BK, bstep = B_KCONTIG ? BK : BK * ldb;

  typedef float vec_a __attribute__((ext_vector_type(VA)));
  typedef float vec_b __attribute__((ext_vector_type(VB)));
  auto load_slab = [&](int64_t k0) {
    const int64_t rem = k_end - k0;
    if (rem >= BK) {
#pragma unroll
      for (int i = 0; i < A_PER_T; ++i) {
        if constexpr (VA == 1) ra[i][0] = abase[offa[i]];
        else {
          const vec_a v = *reinterpret_cast<const vec_a*>(abase + offa[i]);
#pragma unroll
          for (int c = 0; c < VA; ++c) ra[i][c] = v[c];
        }
      }
#pragma unroll
      for (int i = 0; i < B_PER_T; ++i) {
        if constexpr (VB == 1) rb[i][0] = bbase[offb[i]];
        else {
          const vec_b v = *reinterpret_cast<const vec_b*>(bbase + offb[i]);
#pragma unroll
          for (int c = 0; c < VB; ++c) rb[i][c] = v[c];
        }
      }
    } else {  // the last, partial slab: element by element
#pragma unroll
      for (int i = 0; i < A_PER_T; ++i)
#pragma unroll
        for (int c = 0; c < VA; ++c) {
          const int kc = A_KMAJOR ? ka[i] : ka[i] + c;  // k of component c
          ra[i][c] = kc < rem ? abase[offa[i] + c] : 0.f;
        }
#pragma unroll
      for (int i = 0; i < B_PER_T; ++i)
#pragma unroll
        for (int c = 0; c < VB; ++c) {
          const int kc = B_KCONTIG ? kb[i] + c : kb[i];
          rb[i][c] = kc < rem ? bbase[offb[i] + c] : 0.f;
        }
    }
    abase += astep;
    bbase += bstep;
  };
  auto store_slab = [&]() {
#pragma unroll
    for (int i = 0; i < A_PER_T; ++i) {
      int kk, mm;
      pos_a(i, kk, mm);
      if constexpr (A_KMAJOR && VA > 1) {
        vec_a v;
#pragma unroll
        for (int c = 0; c < VA; ++c) v[c] = ra[i][c];
        *reinterpret_cast<vec_a*>(&As[kk][mm]) = v;
      } else {
#pragma unroll
        for (int c = 0; c < VA; ++c) As[A_KMAJOR ? kk : kk + c][A_KMAJOR ? mm + c : mm] = ra[i][c];
      }
    }
#pragma unroll
    for (int i = 0; i < B_PER_T; ++i) {
      int kk, nn;
      pos_b(i, kk, nn);
      if constexpr (!B_KCONTIG && VB > 1) {
        vec_b v;
#pragma unroll
        for (int c = 0; c < VB; ++c) v[c] = rb[i][c];
        *reinterpret_cast<vec_b*>(&Bs[kk][nn]) = v;
      } else {
#pragma unroll
        for (int c = 0; c < VB; ++c) Bs[B_KCONTIG ? kk + c : kk][B_KCONTIG ? nn : nn + c] = rb[i][c];
      }
    }
  };

  const int lrow = lane & 31;   // row (A) / column (B) inside an MFMA tile
  const int lk = lane >> 5;     // which of the 2 k values of one MFMA step

  if (k_begin < k_end) load_slab(k_begin);
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
    store_slab();
    __syncthreads();
    if (k0 + BK < k_end) load_slab(k0 + BK);
#pragma unroll
    for (int ks = 0; ks < BK / 2; ++ks) {
      const int kk = ks * 2 + lk;
      float a[2], b[TN];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = As[kk][wm0 + i * 32 + lrow];
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = Bs[kk][wn0 + j * 32 + lrow];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // accumulator layout of the 32x32 tile: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32
  float* Cout = C + (int64_t)blockIdx.z * split_stride;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn0 + j * 32 + lrow;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm0 + i * 32 + (r >> 2) * 8 + lk * 4 + (r & 3);
        if (m < M && n < N) Cout[m * ldc + n] = acc[i][j][r];
      }
    }

  if constexpr (EPI) {
    const int F = epi.F, H = epi.H;
    float wl[TN], wr[TN];
    int hd[TN];           // head of the lane's column in tile j; -1: this lane stores nothing
    const bool whole = F > 32;            // F == 32 * TN: the wavefront's columns are one head
    const int seg = whole ? 32 : F;       // lanes of a tile that share a head
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn0 + j * 32 + lrow;
      wl[j] = n < N ? epi.a_l[n] : 0.f;  // a_l, a_r are [H, F] = one value per column of C
      wr[j] = n < N ? epi.a_r[n] : 0.f;
      hd[j] = ((lrow & (seg - 1)) == 0 && n < N) ? n / F : -1;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm0 + i * 32 + (r >> 2) * 8 + lk * 4 + (r & 3);
        float vl[TN], vr[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          vl[j] = wl[j] * acc[i][j][r];
          vr[j] = wr[j] * acc[i][j][r];
        }
        if (whole) {
#pragma unroll
          for (int j = 1; j < TN; ++j) {
            vl[0] += vl[j];
            vr[0] += vr[j];
          }
        }
#pragma unroll
        for (int j = 0; j < (whole ? 1 : TN); ++j) {
          const float sl = segment_sum(vl[j], seg), sr = segment_sum(vr[j], seg);
          if (hd[j] >= 0 && m < M) {
            epi.el[m * H + hd[j]] = sl;
            epi.er[m * H + hd[j]] = sr;
          }
        }
      }
  }
}

// c[i] = sum over z of partials[z][i], z ascending (fixed order => reproducible)
// c2 != null: elements from index `cut` on go to c2[i - cut] (two results from one launch)
__device__ __forceinline__ void store_split(float* c, float* c2, int64_t cut, int64_t i, float v) {
  if (c2 != nullptr && i >= cut) c2[i - cut] = v;
  else c[i] = v;
}

__global__ void k_sum_partials(int64_t count, int splits, int64_t stride,
                               const float* __restrict__ partials, float* __restrict__ c,
                               float* __restrict__ c2, int64_t cut) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= count) return;
  // four interleaved running sums keep four loads in flight; their order is fixed
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int z = 0;
  for (; z + 4 <= splits; z += 4) {
    const float* p = partials + (int64_t)z * stride + i;
    const float v0 = p[0], v1 = p[stride], v2 = p[2 * stride], v3 = p[3 * stride];
    s0 += v0; s1 += v1; s2 += v2; s3 += v3;
  }
  for (; z < splits; ++z) s0 += partials[(int64_t)z * stride + i];
  store_split(c, c2, cut, i, (s0 + s1) + (s2 + s3));
}

// Same sum for short outputs and many parts: 8 threads share one output element, each
// adds every 8th part of its range (in four interleaved running sums), then the 8 subtotals are
// added in order through LDS.  blockIdx.y selects a range of `chunk` consecutive parts and writes
// its subtotal to row blockIdx.y of the output (a second call then adds the rows).
// The grouping is fixed, so the result is reproducible.
__global__ __launch_bounds__(256) void k_sum_partials_wide(int64_t count, int parts, int64_t stride,
                                                           const float* __restrict__ partials,
                                                           int chunk, float* __restrict__ c,
                                                           float* __restrict__ c2, int64_t cut) {
  __shared__ float sub[8][32];
  const int col = threadIdx.x & 31, lane8 = threadIdx.x >> 5;
  const int64_t i = (int64_t)blockIdx.x * 32 + col;
  const int z0 = blockIdx.y * chunk;
  const int z1 = z0 + chunk < parts ? z0 + chunk : parts;
  float s = 0.f;
  if (i < count) {
    // four interleaved running sums keep four loads in flight; their order is fixed
    float s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int z = z0 + lane8;
    for (; z + 24 < z1; z += 32) {
      const float* p = partials + (int64_t)z * stride + i;
      const float v0 = p[0], v1 = p[8 * stride], v2 = p[16 * stride], v3 = p[24 * stride];
      s += v0; s1 += v1; s2 += v2; s3 += v3;
    }
    for (; z < z1; z += 8) s += partials[(int64_t)z * stride + i];
    s = (s + s1) + (s2 + s3);
  }
  sub[lane8][col] = s;
  __syncthreads();
  if (lane8 == 0 && i < count) {
    float tot = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) tot += sub[q][col];
    store_split(c, c2, cut, (int64_t)blockIdx.y * count + i, tot);
  }
}

static gnn_status_t sum_partials_launch(int64_t count, int parts, const float* partials, int64_t stride,
                                        float* out, float* out2, int64_t cut, hipStream_t s) {
  if (count <= 0) return GNN_OK;
  if (count >= 32768 || parts < 16) {
    k_sum_partials<<<(unsigned)cdiv(count, 256), 256, 0, s>>>(count, parts, stride, partials, out, out2, cut);
  } else {
    k_sum_partials_wide<<<dim3((unsigned)cdiv(count, 32), 1), 256, 0, s>>>(count, parts, stride, partials,
                                                                           parts, out, out2, cut);
  }
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

gnn_status_t sum_partials_strided(int64_t count, int parts, const float* partials, int64_t stride,
                                  float* out, hipStream_t s) {
  return sum_partials_launch(count, parts, partials, stride, out, nullptr, 0, s);
}

// partials is [parts][2][count]: the first halves are summed into out0, the second into out1
gnn_status_t sum_partials_pair(int64_t count, int parts, const float* partials, float* out0, float* out1,
                               hipStream_t s) {
  return sum_partials_launch(2 * count, parts, partials, 2 * count, out0, out1, count, s);
}

gnn_status_t sum_partials(int64_t count, int parts, const float* partials, float* out, hipStream_t s) {
  return sum_partials_strided(count, parts, partials, count, out, s);
}

// Two levels for very many parts: ranges of kSumChunk parts into `scratch`
// (sum_partials_scratch_rows(parts) rows of `count` floats), then those rows into `out`.
int sum_partials_scratch_rows(int parts) { return (int)cdiv(parts, kSumChunk); }

gnn_status_t sum_partials_two_level(int64_t count, int parts, const float* partials, float* scratch,
                                    float* out, hipStream_t s) {
  if (count <= 0) return GNN_OK;
  const int rows = sum_partials_scratch_rows(parts);
  if (rows <= 1) return sum_partials(count, parts, partials, out, s);
  k_sum_partials_wide<<<dim3((unsigned)cdiv(count, 32), (unsigned)rows), 256, 0, s>>>(
      count, parts, count, partials, kSumChunk, scratch, nullptr, 0);
  GNN_LAUNCH_CHECK();
  return sum_partials(count, rows, scratch, out, s);
}

// 128 output columns per tile unless the last such tile would be at least half empty
static int gemm_tile_cols(int N) {
  if (N <= 64) return 64;
  const int waste = (N + 127) / 128 * 128 - N;
  return waste >= 64 ? 64 : 128;
}

int gemm_pick_split_k(int64_t M, int N, int64_t K) {
  const int bn = gemm_tile_cols(N);
  int64_t tiles = cdiv(M, BM) * cdiv(N, bn);
  if (tiles >= 512 || K < 256) return 1;
  int64_t want = cdiv(1536, tiles);
  int64_t max_by_k = K / 128;  // keep at least 128 of K (8 slabs) per split
  if (want > max_by_k) want = max_by_k;
  if (want > 512) want = 512;
  return want < 1 ? 1 : (int)want;
}

// true when both operands can be fetched in vectors (see VEC of k_gemm_f32)
static bool gemm_vec_ok(int64_t M, int N, const float* a, int64_t lda, bool a_kmajor, const float* b,
                        int64_t ldb, bool b_kcontig) {
  return lda % 2 == 0 && ldb % 4 == 0 && (reinterpret_cast<uintptr_t>(a) & 7u) == 0 &&
         (reinterpret_cast<uintptr_t>(b) & 15u) == 0 && (!a_kmajor || M % 2 == 0) &&
         (b_kcontig || N % 4 == 0);
}

template <int BN, bool AK, bool BKC, bool VEC>
static gnn_status_t launch(int64_t M, int N, int64_t K, const float* a, int64_t lda, const float* b,
                           int64_t ldb, float* c, int64_t ldc, int split_k, float* partials,
                           hipStream_t s) {
  dim3 grid((unsigned)cdiv(M, BM), (unsigned)cdiv(N, BN), (unsigned)split_k);
  const AttnEpilogue none{nullptr, nullptr, nullptr, nullptr, 0, 0};
  if (split_k == 1) {
    ProfScope p("gemm_f32_mfma", s);
    k_gemm_f32<BN, AK, BKC, false, VEC><<<grid, GEMM_THREADS, 0, s>>>(M, N, K, a, lda, b, ldb, c, ldc, K, 0, none);
    GNN_LAUNCH_CHECK();
  } else {
    int64_t kps = cdiv(cdiv(K, split_k), BK) * BK;
    {
      ProfScope p("gemm_f32_mfma_splitk", s);
      k_gemm_f32<BN, AK, BKC, false, VEC><<<grid, GEMM_THREADS, 0, s>>>(M, N, K, a, lda, b, ldb, partials, N, kps,
                                                            M * (int64_t)N, none);
      GNN_LAUNCH_CHECK();
    }
    ProfScope p("gemm_sum_partials", s);
    int64_t count = M * (int64_t)N;
    if (ldc == N) {
      GNN_TRY(sum_partials(count, split_k, partials, c, s));
    } else {
      set_error("gemm_f32: split-K needs a dense output (ldc == N)");
      return GNN_ERR_INVALID_ARG;
    }
  }
  return GNN_OK;
}

gnn_status_t gemm_f32(int64_t M, int N, int64_t K, const float* a, int64_t lda, bool a_kmajor,
                      const float* b, int64_t ldb, bool b_kcontig, float* c, int64_t ldc,
                      int split_k, float* partials, hipStream_t s) {
  if (M <= 0 || N <= 0) return GNN_OK;
  GNN_REQUIRE(K > 0, GNN_ERR_INVALID_ARG, "gemm_f32: K must be positive");
  GNN_REQUIRE(lda > 0 && ldb > 0 && lda < (1 << 24) && ldb < (1 << 24), GNN_ERR_UNSUPPORTED,
              "gemm_f32: leading dimensions must be below 2^24 (32-bit tile offsets)");
  GNN_REQUIRE(cdiv(M, BM) < (int64_t)INT32_MAX && split_k >= 1 && split_k <= 65535,
              GNN_ERR_UNSUPPORTED, "gemm_f32: grid too large");
  GNN_REQUIRE(split_k == 1 || partials != nullptr, GNN_ERR_INVALID_ARG,
              "gemm_f32: split-K without a partials buffer");
  const bool vec = gemm_vec_ok(M, N, a, lda, a_kmajor, b, ldb, b_kcontig);
#define GNN_GEMM_CASE(BN_, AK_, BK_)                                                                      \
  return vec ? launch<BN_, AK_, BK_, true>(M, N, K, a, lda, b, ldb, c, ldc, split_k, partials, s)         \
             : launch<BN_, AK_, BK_, false>(M, N, K, a, lda, b, ldb, c, ldc, split_k, partials, s)
  if (gemm_tile_cols(N) == 128) {
    if (a_kmajor) { if (b_kcontig) GNN_GEMM_CASE(128, true, true); else GNN_GEMM_CASE(128, true, false); }
    else          { if (b_kcontig) GNN_GEMM_CASE(128, false, true); else GNN_GEMM_CASE(128, false, false); }
  } else {
    if (a_kmajor) { if (b_kcontig) GNN_GEMM_CASE(64, true, true); else GNN_GEMM_CASE(64, true, false); }
    else          { if (b_kcontig) GNN_GEMM_CASE(64, false, true); else GNN_GEMM_CASE(64, false, false); }
  }
#undef GNN_GEMM_CASE
}

// z = x w with el, er from the epilogue; only for shapes gemm_attn_epilogue_ok() accepts
bool gemm_attn_epilogue_ok(int heads, int f) {
  const int N = heads * f;
  if (f == 4 || f == 8 || f == 16 || f == 32) return true;
  return f == 64 && gemm_tile_cols(N) == 128;
}

gnn_status_t gemm_f32_attn(int64_t M, int heads, int f, int64_t K, const float* x, const float* w,
                           const float* a_l, const float* a_r, float* z, float* el, float* er,
                           hipStream_t s) {
  const int N = heads * f;
  if (M <= 0) return GNN_OK;
  GNN_REQUIRE(gemm_attn_epilogue_ok(heads, f), GNN_ERR_UNSUPPORTED, "gemm_f32_attn: unsupported head width");
  GNN_REQUIRE(K > 0 && K < (1 << 24) && N < (1 << 24) && cdiv(M, BM) < (int64_t)INT32_MAX, GNN_ERR_UNSUPPORTED,
              "gemm_f32_attn: sizes out of range");
  const AttnEpilogue epi{a_l, a_r, el, er, heads, f};
  ProfScope p("gemm_f32_mfma_attn", s);
  const bool vec = gemm_vec_ok(M, N, x, K, false, w, N, false);
  if (gemm_tile_cols(N) == 128) {
    dim3 grid((unsigned)cdiv(M, BM), (unsigned)cdiv(N, 128), 1);
    if (vec) k_gemm_f32<128, false, false, true, true><<<grid, GEMM_THREADS, 0, s>>>(M, N, K, x, K, w, N, z, N, K, 0, epi);
    else k_gemm_f32<128, false, false, true, false><<<grid, GEMM_THREADS, 0, s>>>(M, N, K, x, K, w, N, z, N, K, 0, epi);
  } else {
    dim3 grid((unsigned)cdiv(M, BM), (unsigned)cdiv(N, 64), 1);
    if (vec) k_gemm_f32<64, false, false, true, true><<<grid, GEMM_THREADS, 0, s>>>(M, N, K, x, K, w, N, z, N, K, 0, epi);
    else k_gemm_f32<64, false, false, true, false><<<grid, GEMM_THREADS, 0, s>>>(M, N, K, x, K, w, N, z, N, K, 0, epi);
  }
  GNN_LAUNCH_CHECK();
  return GNN_OK;
}

}  // namespace gnn

using namespace gnn;

extern "C" gnn_status_t gnn_linear_fwd(int64_t n, int fin, int fout, const float* x, const float* w,
                                       float* y, void* stream) {
  clear_error();
  GNN_REQUIRE(n >= 0 && fin > 0 && fout > 0, GNN_ERR_INVALID_ARG, "gnn_linear_fwd: bad sizes");
  if (n == 0) return GNN_OK;
  GNN_REQUIRE(x && w && y, GNN_ERR_INVALID_ARG, "gnn_linear_fwd: null pointer");
  return gemm_f32(n, fout, fin, x, fin, false, w, fout, false, y, fout, 1, nullptr,
                  static_cast<hipStream_t>(stream));
}
