"""MoNet / GMMConv layer, fp64, every per-edge tensor materialised.
Test infrastructure only.

Definition (App. A.2 "GMMConv"):

    m_e      = pseudo-coordinates of edge e = (u -> v)
    w_k(m)   = exp(-1/2 (m - mu_k)^T Sigma_k^-1 (m - mu_k))       k = 1..K   (ApplyEdge)
    H'[v]    = (1/K) sum over in-edges sum_k w_k(m_e) * Hk[u, k]             (Aggregate)

with Hk = H W_fc viewed as [N, K, Fout].  Readings the paper leaves open:
Sigma_k is diagonal and parameterised by its inverse square root,
Sigma_k^-1 = diag(inv_sigma[k]^2); the pseudo-coordinates are the constant
2-vector m_e = (c[u], c[v]) built from a per-vertex scalar c (1/sqrt(degree)
in the workloads) and carry no gradient.  mu and inv_sigma are learnable.
"""
import numpy as np

from .segments import edge_dst, segment_sum


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def gmm_forward(indptr, indices, H, W_fc, c, mu, inv_sigma):
    H, W_fc, c, mu, inv_sigma = map(_f64, (H, W_fc, c, mu, inv_sigma))
    K, r = mu.shape
    assert r == 2
    n = indptr.shape[0] - 1
    fout = W_fc.shape[1] // K
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)

    Hk = (H @ W_fc).reshape(n, K, fout)
    m = np.stack([c[src], c[dst]], axis=1)                     # [E, 2] pseudo-coordinates
    diff = m[:, None, :] - mu[None, :, :]                      # [E, K, 2]
    q = diff * inv_sigma[None, :, :]
    w = np.exp(-0.5 * (q * q).sum(axis=2))                     # [E, K] gaussian weights
    msg = (w[:, :, None] * Hk[src]).sum(axis=1) / K            # [E, Fout]
    out = segment_sum(indptr, msg)
    return dict(src=src, dst=dst, Hk=Hk, m=m, diff=diff, w=w, msg=msg, out=out)


def gmm_backward(indptr, indices, H, W_fc, c, mu, inv_sigma, gout, fwd=None):
    """Gradients of L = <gout, H'> w.r.t. H, W_fc, mu, inv_sigma."""
    if fwd is None:
        fwd = gmm_forward(indptr, indices, H, W_fc, c, mu, inv_sigma)
    H, W_fc, mu, inv_sigma, g = map(_f64, (H, W_fc, mu, inv_sigma, gout))
    src, dst, Hk, diff, w = fwd["src"], fwd["dst"], fwd["Hk"], fwd["diff"], fwd["w"]
    n, K, fout = Hk.shape

    dmsg = g[dst]                                               # [E, Fout]
    dw = np.einsum("ef,ekf->ek", dmsg, Hk[src]) / K             # [E, K]
    dHk_e = w[:, :, None] * dmsg[:, None, :] / K                # [E, K, Fout]
    dHk = np.zeros_like(Hk)
    np.add.at(dHk, src, dHk_e)
    # w = exp(-1/2 sum_d ((m_d - mu_kd) s_kd)^2)
    dlog = (dw * w)[:, :, None]                                 # [E, K, 1]
    gmu = (dlog * diff * inv_sigma[None] ** 2).sum(axis=0)
    ginv_sigma = (-dlog * diff ** 2 * inv_sigma[None]).sum(axis=0)
    dHk2 = dHk.reshape(n, K * fout)
    gW = H.T @ dHk2
    gH = dHk2 @ W_fc.T
    return dict(gx=gH, gw_fc=gW, gmu=gmu, ginv_sigma=ginv_sigma, dHk=dHk2, dw=dw)


# ---- general pseudo-coordinates ------------------------------------------------------------
# The paper's MoNet settings use pseudo-coordinates of dimension r = 1, 2, 3 obtained from the
# degrees by a learnable projection (Sec. 7.2; App. A.2: m_uv = f(x_u, x_v), f a projection).
# Here the pseudo-coordinates are a per-edge input [E, r] in CSR order, as in the definition of
# w_k(m); the projection that produces them is a separate, plain function below.
def gmm_pseudo_forward(indptr, indices, H, W_fc, pseudo, mu, inv_sigma):
    H, W_fc, m, mu, inv_sigma = map(_f64, (H, W_fc, pseudo, mu, inv_sigma))
    K, r = mu.shape
    n = indptr.shape[0] - 1
    fout = W_fc.shape[1] // K
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)
    m = m.reshape(src.shape[0], r)
    Hk = (H @ W_fc).reshape(n, K, fout)
    diff = m[:, None, :] - mu[None, :, :]                      # [E, K, r]
    q = diff * inv_sigma[None, :, :]
    w = np.exp(-0.5 * (q * q).sum(axis=2))                     # [E, K]
    msg = (w[:, :, None] * Hk[src]).sum(axis=1) / K            # [E, Fout]
    out = segment_sum(indptr, msg)
    return dict(src=src, dst=dst, Hk=Hk, m=m, diff=diff, w=w, msg=msg, out=out)


def gmm_pseudo_backward(indptr, indices, H, W_fc, pseudo, mu, inv_sigma, gout, fwd=None):
    """Gradients of L = <gout, H'> w.r.t. H, W_fc, mu, inv_sigma and the pseudo-coordinates."""
    if fwd is None:
        fwd = gmm_pseudo_forward(indptr, indices, H, W_fc, pseudo, mu, inv_sigma)
    H, W_fc, mu, inv_sigma, g = map(_f64, (H, W_fc, mu, inv_sigma, gout))
    src, dst, Hk, diff, w = fwd["src"], fwd["dst"], fwd["Hk"], fwd["diff"], fwd["w"]
    n, K, fout = Hk.shape
    dmsg = g[dst]
    dw = np.einsum("ef,ekf->ek", dmsg, Hk[src]) / K
    dHk_e = w[:, :, None] * dmsg[:, None, :] / K
    dHk = np.zeros_like(Hk)
    np.add.at(dHk, src, dHk_e)
    dlog = (dw * w)[:, :, None]                                 # d L / d (-1/2 |q|^2), per edge and kernel
    gmu = (dlog * diff * inv_sigma[None] ** 2).sum(axis=0)
    ginv_sigma = (-dlog * diff ** 2 * inv_sigma[None]).sum(axis=0)
    gpseudo = (-dlog * diff * inv_sigma[None] ** 2).sum(axis=1)  # [E, r]
    dHk2 = dHk.reshape(n, K * fout)
    return dict(gx=dHk2 @ W_fc.T, gw_fc=H.T @ dHk2, gmu=gmu, ginv_sigma=ginv_sigma, gpseudo=gpseudo,
                dHk=dHk2, dw=dw)


def pseudo_projection_forward(indptr, indices, c, P, pb):
    """pseudo[e, d] = tanh(P[d,0] c[u] + P[d,1] c[v] + pb[d]) for e = (u -> v): the learnable
    projection of the degree pair (c = 1/sqrt(degree) in the workloads) to r dimensions."""
    c, P, pb = map(_f64, (c, P, pb))
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)
    pre = c[src][:, None] * P[None, :, 0] + c[dst][:, None] * P[None, :, 1] + pb[None, :]
    return np.tanh(pre)


def pseudo_projection_backward(indptr, indices, c, P, pb, gpseudo):
    """Gradients of <gpseudo, pseudo> w.r.t. P [r,2] and pb [r]."""
    c, P, pb, g = map(_f64, (c, P, pb, gpseudo))
    src = np.asarray(indices, dtype=np.int64)
    dst = edge_dst(indptr)
    m = pseudo_projection_forward(indptr, indices, c, P, pb)
    dpre = g.reshape(m.shape) * (1.0 - m * m)
    gP = np.stack([(dpre * c[src][:, None]).sum(axis=0), (dpre * c[dst][:, None]).sum(axis=0)], axis=1)
    return gP, dpre.sum(axis=0)
