"""GCN layer with separable static edge weights, fp64, every per-edge tensor materialised.
Test infrastructure only.

Definition (App. A.2 "GCN", without bias and with the identity activation):

    H'[v] = sum over in-edges e = (u -> v) of  e_uv * (H W)[u]

with the static, gradient-free edge weight e_uv = c_src[u] * c_dst[v] (the symmetric
normalisation 1/sqrt(deg_u deg_v), mean aggregation and plain sums are all of this
form).  Dataflow of Fig. 11(a): ApplyVertex (H W), Scatter (copy the source row to the
edge), ApplyEdge (multiply by the edge weight), Gather (sum).
"""
import numpy as np

from .segments import edge_dst, segment_sum


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def gcn_forward(indptr, indices, H, W, c_src, c_dst):
    H, W, c_src, c_dst = map(_f64, (H, W, c_src, c_dst))
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)
    Z = H @ W                                   # ApplyVertex
    ew = c_src[src] * c_dst[dst]                # static edge weights [E]
    copied = Z[src]                             # Scatter: copy_u            [E, Fout]
    msg = ew[:, None] * copied                  # ApplyEdge: multiply        [E, Fout]
    out = segment_sum(indptr, msg)              # Gather: sum
    return dict(src=src, dst=dst, Z=Z, ew=ew, msg=msg, out=out)


def gcn_backward(indptr, indices, H, W, c_src, c_dst, gout, fwd=None):
    """Gradients of L = <gout, H'> w.r.t. H and W (the edge weights carry none)."""
    if fwd is None:
        fwd = gcn_forward(indptr, indices, H, W, c_src, c_dst)
    H, W, g = map(_f64, (H, W, gout))
    src, dst, ew = fwd["src"], fwd["dst"], fwd["ew"]
    dmsg = g[dst]                               # Gather^T: copy to the edges
    dcopied = ew[:, None] * dmsg                # ApplyEdge^T
    dZ = np.zeros_like(fwd["Z"])
    np.add.at(dZ, src, dcopied)                 # Scatter^T: sum over out-edges
    return dict(gx=dZ @ W.T, gw=H.T @ dZ, dZ=dZ)
