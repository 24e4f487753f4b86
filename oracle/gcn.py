"""GCN layer with static edge weights, fp64, every per-edge tensor materialised.
Test infrastructure only.  The separable form e_uv = c_src[u] c_dst[v] comes first; the general
form with an arbitrary static scalar per edge (gcn_edge_forward / gcn_edge_backward) is at the end.

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


# ---- general static edge weights --------------------------------------------------------------
# App. A.2 "GCN": H'[v] = sum over in-edges e = (u -> v) of e_uv * (H W)[u] with e_uv ANY static,
# gradient-free scalar per edge, given here as ew [E] in CSR-by-destination order (duplicate
# edges carry their own weights).  Same dataflow: ApplyVertex, Scatter, ApplyEdge, Gather.
def gcn_edge_forward(indptr, indices, H, W, ew):
    H, W, ew = map(_f64, (H, W, ew))
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)
    Z = H @ W                                   # ApplyVertex
    copied = Z[src]                             # Scatter: copy_u            [E, Fout]
    msg = ew[:, None] * copied                  # ApplyEdge: multiply        [E, Fout]
    out = segment_sum(indptr, msg)              # Gather: sum
    return dict(src=src, dst=dst, Z=Z, ew=ew, msg=msg, out=out)


def gcn_edge_backward(indptr, indices, H, W, ew, gout, fwd=None):
    """Gradients of L = <gout, H'> w.r.t. H and W (the edge weights are static)."""
    if fwd is None:
        fwd = gcn_edge_forward(indptr, indices, H, W, ew)
    H, W, g = map(_f64, (H, W, gout))
    src, dst, w_e = fwd["src"], fwd["dst"], fwd["ew"]
    dmsg = g[dst]                               # Gather^T
    dcopied = w_e[:, None] * dmsg               # ApplyEdge^T
    dZ = np.zeros_like(fwd["Z"])
    np.add.at(dZ, src, dcopied)                 # Scatter^T
    return dict(gx=dZ @ W.T, gw=H.T @ dZ, dZ=dZ)
