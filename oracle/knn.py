"""k-nearest-neighbour graph of batched point clouds.  Test infrastructure only.

The EdgeConv model builds its graph from the points themselves (Sec. 7.2: "k nearest
neighbours", k = 20 / 40, per point cloud of a batch).  Definition used here: for every
point, the k points of the same cloud with the smallest squared Euclidean distance, the
point itself included, ties broken towards the lower index; an edge runs from each chosen
neighbour to the point.  The result is the CSR by destination with sources ascending.

Floating point decides integers here, so the precision is part of the definition: the
squared distance is accumulated in float32, coordinate by coordinate in index order,
each step rounded ( ((d0*d0 + d1*d1) + d2*d2) + ... with d_i = a_i - b_i rounded first ).
"""
import numpy as np


def squared_distances_f32(cloud):
    """[P, P] float32 squared distances of one cloud [P, D], accumulated as the header says."""
    c = np.asarray(cloud, dtype=np.float32)
    P, D = c.shape
    acc = np.zeros((P, P), dtype=np.float32)
    for i in range(D):
        diff = (c[:, None, i] - c[None, :, i]).astype(np.float32)
        sq = (diff * diff).astype(np.float32)
        acc = sq if i == 0 else (acc + sq).astype(np.float32)
    return acc


def knn_graph(coords, clouds, points, k):
    """coords [clouds*points, D] -> (indptr int32 [n+1], indices int32 [n*k])."""
    coords = np.asarray(coords, dtype=np.float32)
    n = clouds * points
    assert coords.shape[0] == n and 0 < k <= points
    indices = np.empty((n, k), dtype=np.int32)
    for b in range(clouds):
        d2 = squared_distances_f32(coords[b * points:(b + 1) * points])
        nearest = np.argsort(d2, axis=1, kind="stable")[:, :k]   # stable: ties to the lower index
        nearest.sort(axis=1)
        indices[b * points:(b + 1) * points] = nearest + b * points
    indptr = (np.arange(n + 1, dtype=np.int64) * k).astype(np.int32)
    return indptr, indices.reshape(-1)
