"""EdgeConv layer, original dataflow, fp64.  Test infrastructure only.

Definition (App. A.2 "EdgeConv"):

    H'[v] = max over in-edges (u -> v) of  Theta (H[u] - H[v]) + Phi H[v]

computed in the un-reorganized operator order the appendix lists:

    E      = u_sub_v(H)            [E, Fin]    Scatter
    E_T    = E Theta               [E, Fout]   linear ApplyEdge (the redundant per-edge product)
    N_P    = H Phi                 [N, Fout]   linear ApplyVertex
    E_TP   = e_add_v(E_T, N_P)     [E, Fout]
    H'     = reduce_max(E_TP)      [N, Fout]   Gather

Theta and Phi are stored [Fin, Fout] and applied as row-vector times matrix.
Only the arg-max positions (O(|V|)) are needed by the backward pass (Sec. 7.2).
Ties: the first in-edge in CSR order that attains the maximum wins.  An empty
row gives H'[v] = 0 and arg-max -1.
"""
import numpy as np

from .segments import edge_dst, segment_max, segment_sum


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def edgeconv_forward(indptr, indices, H, Theta, Phi):
    H, Theta, Phi = _f64(H), _f64(Theta), _f64(Phi)
    n = indptr.shape[0] - 1
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)
    nnz = src.shape[0]

    E = H[src] - H[dst]                       # u_sub_v
    E_T = E @ Theta                           # per-edge linear projection
    N_P = H @ Phi
    E_TP = E_T + N_P[dst]                     # e_add_v

    nonempty = np.diff(indptr) > 0
    mx = segment_max(indptr, E_TP, empty=-np.inf)
    out = np.where(nonempty[:, None], mx, 0.0)
    # first CSR position attaining the maximum
    pos = np.arange(nnz, dtype=np.int64)[:, None]
    cand = np.where(E_TP == mx[dst], pos, np.int64(nnz))
    first = -segment_max(indptr, -cand, empty=1.0)      # segment min
    argmax = np.where(nonempty[:, None], first, -1).astype(np.int64)
    return dict(src=src, dst=dst, E=E, E_T=E_T, N_P=N_P, E_TP=E_TP, out=out, argmax=argmax)


def near_tie_mask(indptr, fwd, tol):
    """[N, Fout] bool: more than one in-edge lies within `tol` of the maximum,
    so a lower-precision evaluation may legitimately pick another winner."""
    E_TP, dst, out = fwd["E_TP"], fwd["dst"], fwd["out"]
    close = (E_TP >= out[dst] - tol).astype(np.float64)
    return segment_sum(indptr, close) > 1.5


def edgeconv_backward(indptr, indices, H, Theta, Phi, gout, fwd=None):
    """Gradients of L = <gout, H'> w.r.t. H, Theta, Phi."""
    if fwd is None:
        fwd = edgeconv_forward(indptr, indices, H, Theta, Phi)
    H, Theta, Phi, g = _f64(H), _f64(Theta), _f64(Phi), _f64(gout)
    src, dst, E, argmax = fwd["src"], fwd["dst"], fwd["E"], fwd["argmax"]
    nnz = src.shape[0]
    pos = np.arange(nnz, dtype=np.int64)[:, None]

    # backward of reduce_max: the vertex gradient goes to the winning edge only
    dE_TP = np.where(argmax[dst] == pos, g[dst], 0.0)           # [E, Fout]
    # e_add_v
    dE_T = dE_TP
    dN_P = segment_sum(indptr, dE_TP)
    # the two linear layers
    gTheta = E.T @ dE_T
    dE = dE_T @ Theta.T
    gPhi = H.T @ dN_P
    gH = dN_P @ Phi.T
    # u_sub_v
    np.add.at(gH, src, dE)
    np.add.at(gH, dst, -dE)
    return dict(gx=gH, gtheta=gTheta, gphi=gPhi, dE_TP=dE_TP)
