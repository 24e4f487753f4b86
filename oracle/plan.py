"""Integer plan tables, computed the slow obvious way.  Test infrastructure only.

The vertex-balanced thread mapping (Sec. 5) walks the in-edge set of a vertex;
source-side gradients walk the out-edge set instead, which needs the transpose
of the CSR-by-destination graph.  The specification these tables follow:

  CSC transpose  edges ordered by (source ascending, CSR position ascending):
                 indptr_t[N+1], indices_t[E] = destination of each out-edge,
                 eid_t[E] = CSR position of that edge.
  degree order   vertices sorted by degree descending, ties by ascending id
                 (in-degree for side 0, out-degree for side 1).
  bucket         clz32(degree): the number of leading zero bits of the degree
                 as a 32-bit integer (32 for degree 0), so bucket ids ascend
                 along the degree order; bucket_offsets[b] = first position of
                 bucket b in the order, bucket_offsets[33] = N.
"""
import numpy as np

NUM_BUCKETS = 33


def csc_transpose(indptr, indices):
    n = indptr.shape[0] - 1
    nnz = indices.shape[0]
    dst = np.repeat(np.arange(n, dtype=np.int64), np.diff(indptr))
    triples = sorted(zip(indices.tolist(), range(nnz)))   # (src, csr position)
    eid_t = np.array([p for _, p in triples], dtype=np.int32).reshape(-1)
    indices_t = dst[eid_t].astype(np.int32) if nnz else np.zeros(0, np.int32)
    counts = np.zeros(n, dtype=np.int64)
    for s in indices.tolist():
        counts[s] += 1
    indptr_t = np.zeros(n + 1, dtype=np.int32)
    indptr_t[1:] = np.cumsum(counts)
    return indptr_t, indices_t, eid_t


def clz32(d):
    d = int(d)
    return 32 if d == 0 else 32 - d.bit_length()


def degree_buckets(indptr_side):
    """(bucket_of_vertex[N], order[N], bucket_offsets[34]) for the rows of `indptr_side`."""
    n = indptr_side.shape[0] - 1
    deg = [int(indptr_side[v + 1]) - int(indptr_side[v]) for v in range(n)]
    bucket = np.array([clz32(d) for d in deg], dtype=np.int32).reshape(-1)
    order = np.array(sorted(range(n), key=lambda v: (-deg[v], v)), dtype=np.int32).reshape(-1)
    offsets = np.zeros(NUM_BUCKETS + 1, dtype=np.int32)
    for b in range(NUM_BUCKETS):
        offsets[b + 1] = offsets[b] + int((bucket == b).sum())
    return bucket, order, offsets


def blocked_edges(ptr, cols, block_cols):
    """Column-blocked edge list of one side: edges stable-sorted by
    (column // block_cols, row); returns (num_blocks, bptr[num_blocks*n + 1], bcol[nnz])."""
    n = ptr.shape[0] - 1
    nblk = -(-n // block_cols)
    triples = []
    for r in range(n):
        for pos in range(int(ptr[r]), int(ptr[r + 1])):
            triples.append((int(cols[pos]) // block_cols, r, pos))
    triples.sort()
    bcol = np.array([int(cols[p]) for _, _, p in triples], dtype=np.int32).reshape(-1)
    bptr = np.zeros(nblk * n + 1, dtype=np.int64)
    for b, r, _ in triples:
        bptr[b * n + r + 1] += 1
    return nblk, np.cumsum(bptr).astype(np.int32), bcol
