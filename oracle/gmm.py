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
