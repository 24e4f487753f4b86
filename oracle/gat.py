"""GAT layer, original (un-reorganized) dataflow, fp64.  Test infrastructure only.

Definition (App. A.2 "GAT"; attention score of Sec. 4 Eq. 1):

    Ht        = H W                                        (ExpensiveApply on vertices)
    M0[e]     = a^T [ Ht[u] || Ht[v] ]    e = (u -> v)     (Scatter u_concat_v, then LP)
    M1[e]     = LeakyReLU(M0[e])                           (ApplyEdge)
    M2[e]     = edge_softmax over the in-edges of v        (ReduceScatter, App. A.1)
    H'[v]     = sum_e M2[e] * Ht[u]                        (Aggregate, reduce_sum)

u is the source and v the destination of an edge; a = [a_l || a_r] with a_l
meeting the source half.  With several heads every head has its own column
block of W and its own a; heads are concatenated.  All per-edge tensors are
materialised ("stash everything", Sec. 2.2 / Fig. 2), and the backward pass is
the explicit chain rule through them (operator rules of App. B).

Shapes: H [N, Fin], W [Fin, heads*F], a_l/a_r [heads, F], edge tensors [E, heads(, F)].
"""
import numpy as np

from .segments import edge_dst, segment_max, segment_sum


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def gat_forward(indptr, indices, H, W, a_l, a_r, slope, Ht=None):
    """Forward pass; returns every intermediate tensor in a dict.

    Ht may be passed to reuse a projection this oracle computed before.
    An empty row yields H'[v] = 0 with saved max 0 and denominator 1.
    """
    a_l, a_r = _f64(a_l), _f64(a_r)
    heads, F = a_l.shape
    n = indptr.shape[0] - 1
    if Ht is None:
        Ht = _f64(H) @ _f64(W)
    Ht = Ht.reshape(n, heads, F)
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)

    a = np.concatenate([a_l, a_r], axis=1)                      # [heads, 2F]
    cat = np.concatenate([Ht[src], Ht[dst]], axis=2)            # u_concat_v: [E, heads, 2F]
    M0 = np.einsum("ehk,hk->eh", cat, a)                        # LP
    M1 = np.where(M0 > 0, M0, slope * M0)                       # LeakyReLU

    # edge-softmax = two ReduceScatter steps (RS1: max/copy/subtract, RS2: sum/copy/divide)
    mx = segment_max(indptr, M1, empty=0.0)                     # [N, heads]
    ex = np.exp(M1 - mx[dst])
    den = segment_sum(indptr, ex)
    den_safe = np.where(np.diff(indptr)[:, None] > 0, den, 1.0)
    M2 = ex / den_safe[dst]

    msg = M2[:, :, None] * Ht[src]                              # [E, heads, F] materialised
    Hn = segment_sum(indptr, msg)                               # reduce_sum
    return dict(Ht=Ht, src=src, dst=dst, a=a, cat=cat, M0=M0, M1=M1, M2=M2, mx=mx,
                den=den_safe, msg=msg, out=Hn.reshape(n, heads * F))


def gat_backward(indptr, indices, H, W, a_l, a_r, slope, gout, fwd=None):
    """Gradients of L = <gout, H'> w.r.t. H, W, a_l, a_r through the stashed tensors."""
    if fwd is None:
        fwd = gat_forward(indptr, indices, H, W, a_l, a_r, slope)
    Ht, src, dst, a, cat = fwd["Ht"], fwd["src"], fwd["dst"], fwd["a"], fwd["cat"]
    M0, M2 = fwd["M0"], fwd["M2"]
    n, heads, F = Ht.shape
    g = _f64(gout).reshape(n, heads, F)

    # backward of Gather(sum): Scatter(copy_v) of the vertex gradient to its in-edges
    dmsg = g[dst]                                               # [E, heads, F]
    # msg = M2 * Ht[u]
    dM2 = np.einsum("ehf,ehf->eh", dmsg, Ht[src])
    dHt_src = M2[:, :, None] * dmsg
    # edge-softmax backward: dM1 = M2 * (dM2 - sum_{e' into v} M2 dM2)
    t = segment_sum(indptr, M2 * dM2)
    dM1 = M2 * (dM2 - t[dst])
    dM0 = dM1 * np.where(M0 > 0, 1.0, slope)                    # LeakyReLU'
    # LP backward: M0 = cat . a
    da = np.einsum("eh,ehk->hk", dM0, cat)
    dcat = dM0[:, :, None] * a[None, :, :]                      # [E, heads, 2F]
    # backward of Scatter: Gather onto both endpoints
    dHt = np.zeros_like(Ht)
    np.add.at(dHt, src, dHt_src + dcat[:, :, :F])
    np.add.at(dHt, dst, dcat[:, :, F:])
    dHt2 = dHt.reshape(n, heads * F)
    gW = _f64(H).T @ dHt2
    gH = dHt2 @ _f64(W).T
    return dict(gx=gH, gw=gW, ga_l=da[:, :F], ga_r=da[:, F:], dHt=dHt2, dM0=dM0, dM1=dM1)
