"""Seeded synthetic graph generators (inputs only).

This module produces the graphs that both the CPU oracle and the HIP library
are fed with.  It holds none of the layers' arithmetic: only random structure.
Every graph is returned as CSR *by destination*:

    indptr  int32 [N+1]   indptr[v]..indptr[v+1] is the in-edge range of v
    indices int32 [E]     source vertex of each in-edge, ascending inside a row

An edge (u, e, v) of the operator definition (App. A.1) is stored at CSR
position e with u = indices[e] and v the row that contains e.

The real datasets of the evaluation (Sec. 7.1: Cora, Citeseer, Pubmed, Reddit,
ModelNet40) are not available here; these generators stand in for them by
vertex count, edge count and degree distribution only.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "rng_for",
    "csr_from_pairs",
    "erdos_renyi",
    "chung_lu",
    "knn_point_clouds",
    "dst_of_edges",
]


def rng_for(seed: int) -> np.random.Generator:
    """Counter-based generator (Philox) so a seed fixes the stream on any host."""
    return np.random.Generator(np.random.Philox(int(seed) & 0xFFFFFFFFFFFFFFFF))


def dst_of_edges(indptr: np.ndarray) -> np.ndarray:
    """Destination vertex of every CSR position."""
    n = indptr.shape[0] - 1
    return np.repeat(np.arange(n, dtype=np.int32), np.diff(indptr))


def csr_from_pairs(n: int, src: np.ndarray, dst: np.ndarray, *, self_loops: bool,
                   dedupe: bool = True, drop_loops: bool = True):
    """Sort (dst, src) pairs into CSR by destination with ascending sources.

    drop_loops removes u == v pairs from the input; self_loops then adds exactly
    one (v, v) per vertex.  dedupe keeps one copy of a repeated pair.
    """
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if drop_loops:
        keep = src != dst
        src, dst = src[keep], dst[keep]
    key = dst * n + src
    if self_loops:
        v = np.arange(n, dtype=np.int64)
        key = np.concatenate([key, v * n + v])
    key.sort()
    if dedupe and key.size:
        keep = np.empty(key.shape, dtype=bool)
        keep[0] = True
        np.not_equal(key[1:], key[:-1], out=keep[1:])
        key = key[keep]
    d = key // n
    indices = (key - d * n).astype(np.int32)
    counts = np.bincount(d, minlength=n)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=indptr[1:])
    if indptr[-1] >= 2**31:
        raise ValueError("edge count does not fit int32 offsets")
    return indptr.astype(np.int32), indices


def erdos_renyi(n: int, m: int, seed: int, *, self_loops: bool = True):
    """G(n, m): m distinct directed non-loop pairs drawn uniformly, plus loops."""
    rng = rng_for(seed)
    total = n * (n - 1)
    if m > total:
        raise ValueError("m exceeds the number of ordered pairs")
    # draw distinct codes in [0, n(n-1)) and decode to (dst, src != dst)
    codes = np.unique(rng.integers(0, total, size=int(m * 1.2) + 16, dtype=np.int64))
    while codes.size < m:
        extra = rng.integers(0, total, size=m, dtype=np.int64)
        codes = np.unique(np.concatenate([codes, extra]))
    codes = rng.permutation(codes)[:m]
    dst = codes // (n - 1)
    off = codes - dst * (n - 1)
    src = off + (off >= dst)
    return csr_from_pairs(n, src, dst, self_loops=self_loops)


def chung_lu_weights(n: int, total_weight: float, gamma: float) -> np.ndarray:
    """Power-law expected degrees w_i ~ (i + i0)^(-1/(gamma-1)), sum = total_weight.

    i0 is chosen so that max(w) = sqrt(sum(w)), the largest value for which every
    pair probability w_i w_j / sum(w) stays <= 1.
    """
    expo = -1.0 / (gamma - 1.0)
    i = np.arange(n, dtype=np.float64)

    def ratio(i0):
        w = (i + i0) ** expo
        s = w.sum()
        # w_max * scale  vs sqrt(total): scale = total/s
        return (w[0] * total_weight / s) / np.sqrt(total_weight)

    lo, hi = 1e-9, float(n) * 1e3
    if ratio(lo) <= 1.0:
        i0 = lo
    else:
        for _ in range(200):
            mid = np.sqrt(lo * hi)
            if ratio(mid) > 1.0:
                lo = mid
            else:
                hi = mid
        i0 = hi
    w = (i + i0) ** expo
    return w * (total_weight / w.sum())


def chung_lu(n: int, m: int, gamma: float, seed: int, *, self_loops: bool = True):
    """Chung-Lu directed graph: m (src, dst) pairs drawn independently with
    probability proportional to w_src * w_dst; loops and duplicates dropped
    (so the edge count is about m), then one self-loop per vertex if asked.

    Both the in- and the out-degree sequence follow the power law.
    """
    rng = rng_for(seed)
    w = chung_lu_weights(n, float(m), gamma)
    p = w / w.sum()
    # The multiset of destinations of m independent draws is multinomial; the
    # sources are drawn the same way and then matched to them in random order,
    # which is the same distribution as m independent pairs.
    cnt_dst = rng.multinomial(m, p)
    cnt_src = rng.multinomial(m, p)
    ids = np.arange(n, dtype=np.int32)
    dst = np.repeat(ids, cnt_dst)
    src = np.repeat(ids, cnt_src)
    rng.shuffle(src)
    return csr_from_pairs(n, src, dst, self_loops=self_loops)


def knn_point_clouds(batch: int, points: int, k: int, seed: int):
    """`batch` clouds of `points` 3-D points uniform in the unit cube; every
    point receives an edge from each of its k nearest points of the same cloud
    (squared Euclidean distance, the point itself included, ties to the lower
    index).  Vertex id = cloud * points + i.  Every in-degree equals k.

    Returns (indptr, indices, coords[float32, batch*points, 3]).
    """
    rng = rng_for(seed)
    coords = rng.random((batch, points, 3), dtype=np.float32)
    n = batch * points
    indices = np.empty((n, k), dtype=np.int32)
    for b in range(batch):
        c = coords[b].astype(np.float64)
        d2 = ((c[:, None, :] - c[None, :, :]) ** 2).sum(axis=2)
        nearest = np.argsort(d2, axis=1, kind="stable")[:, :k]
        nearest.sort(axis=1)
        indices[b * points:(b + 1) * points] = nearest + b * points
    indptr = (np.arange(n + 1, dtype=np.int64) * k).astype(np.int32)
    return indptr, indices.reshape(-1), coords.reshape(n, 3)
