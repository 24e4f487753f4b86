"""Pins for the MoNet / GMMConv oracle (App. A.2 "GMMConv")."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

from oracle import gmm as om
from helpers import finite_difference, random_graph


def make_case(rng, n, m, fin, fout, K, duplicates=False):
    indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=duplicates)
    X = rng.standard_normal((n, fin))
    W = rng.standard_normal((fin, K * fout)) * 0.5
    deg = np.diff(indptr)
    c = 1.0 / np.sqrt(np.maximum(deg, 1))
    mu = rng.standard_normal((K, 2)) * 0.3
    inv_sigma = 0.5 + rng.random((K, 2))
    return indptr, indices, X, W, c, mu, inv_sigma


def brute_force(indptr, indices, X, W, c, mu, inv_sigma):
    n = len(indptr) - 1
    K = mu.shape[0]
    fout = W.shape[1] // K
    Hk = (X @ W).reshape(n, K, fout)
    out = np.zeros((n, fout))
    for v in range(n):
        for e in range(indptr[v], indptr[v + 1]):
            u = indices[e]
            m = np.array([c[u], c[v]])
            for k in range(K):
                Sinv = np.diag(inv_sigma[k] ** 2)                 # diagonal covariance inverse
                w = np.exp(-0.5 * (m - mu[k]) @ Sinv @ (m - mu[k]))
                out[v] += w * Hk[u, k] / K
    return out


def test_forward_matches_loop_brute_force():
    rng = np.random.default_rng(1)
    args = make_case(rng, 15, 50, 4, 3, 3, duplicates=True)
    np.testing.assert_allclose(om.gmm_forward(*args)["out"], brute_force(*args), rtol=1e-12, atol=1e-13)


def test_flat_kernels_reduce_to_sparse_matmul():
    # inv_sigma = 0 -> every gaussian weight is 1 -> out = (1/K) sum_k A Hk[:, k]
    rng = np.random.default_rng(2)
    indptr, indices, X, W, c, mu, inv_sigma = make_case(rng, 40, 220, 5, 4, 3)
    out = om.gmm_forward(indptr, indices, X, W, c, mu, 0 * inv_sigma)["out"]
    A = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(40, 40))
    Hk = (X @ W).reshape(40, 3, 4)
    ref = sum(A @ Hk[:, k, :] for k in range(3)) / 3
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_weight_is_one_at_the_kernel_mean():
    # regular graph: every degree equal -> all pseudo-coordinates equal; K = 1, mu = m
    n = 12
    edges_src = np.array([[v, (v + 1) % n, (v + 5) % n] for v in range(n)])
    indptr = (np.arange(n + 1) * 3).astype(np.int32)
    indices = np.sort(edges_src, axis=1).reshape(-1).astype(np.int32)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((n, 4))
    W = rng.standard_normal((4, 5))
    c = np.full(n, 1 / np.sqrt(3))
    mu = np.array([[c[0], c[0]]])
    fwd = om.gmm_forward(indptr, indices, X, W, c, mu, np.array([[2.0, 3.0]]))
    np.testing.assert_allclose(fwd["w"], 1.0, rtol=1e-15)
    A = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(n, n))
    np.testing.assert_allclose(fwd["out"], A @ (X @ W), rtol=1e-12, atol=1e-13)


def _loss(args, gout):
    return float((om.gmm_forward(*args)["out"] * gout).sum())


def test_backward_matches_finite_differences():
    rng = np.random.default_rng(4)
    indptr, indices, X, W, c, mu, inv_sigma = make_case(rng, 12, 40, 3, 4, 3)
    gout = rng.standard_normal((12, 4))
    bwd = om.gmm_backward(indptr, indices, X, W, c, mu, inv_sigma, gout)
    for name, theta, fun in [
        ("gx", X, lambda t: _loss((indptr, indices, t, W, c, mu, inv_sigma), gout)),
        ("gw_fc", W, lambda t: _loss((indptr, indices, X, t, c, mu, inv_sigma), gout)),
        ("gmu", mu, lambda t: _loss((indptr, indices, X, W, c, t, inv_sigma), gout)),
        ("ginv_sigma", inv_sigma, lambda t: _loss((indptr, indices, X, W, c, mu, t), gout)),
    ]:
        idx, g = finite_difference(fun, theta)
        np.testing.assert_allclose(bwd[name].reshape(-1)[idx], g, rtol=2e-6, atol=2e-7, err_msg=name)


def test_backward_matches_torch_autograd():
    rng = np.random.default_rng(5)
    n, K, fout = 18, 2, 3
    indptr, indices, X, W, c, mu, inv_sigma = make_case(rng, n, 70, 4, fout, K)
    gout = rng.standard_normal((n, fout))
    tX, tW, tmu, tis = (torch.tensor(a, dtype=torch.float64, requires_grad=True)
                        for a in (X, W, mu, inv_sigma))
    Hk = (tX @ tW).reshape(n, K, fout)
    src = torch.tensor(indices.astype(np.int64))
    dst = torch.tensor(np.repeat(np.arange(n), np.diff(indptr)))
    tc = torch.tensor(c)
    m = torch.stack([tc[src], tc[dst]], dim=1)
    q = (m[:, None, :] - tmu[None]) * tis[None]
    w = torch.exp(-0.5 * (q * q).sum(-1))
    msg = (w[:, :, None] * Hk[src]).sum(1) / K
    out = torch.zeros(n, fout, dtype=torch.float64).index_add(0, dst, msg)
    (out * torch.tensor(gout)).sum().backward()
    bwd = om.gmm_backward(indptr, indices, X, W, c, mu, inv_sigma, gout)
    np.testing.assert_allclose(bwd["gx"], tX.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["gw_fc"], tW.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["gmu"], tmu.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["ginv_sigma"], tis.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_kernels_are_exchangeable():
    """Permuting the K kernels (rows of mu / inv_sigma, column blocks of W_fc) leaves the
    output alone and permutes their gradients (App. A.2: a plain sum over k)."""
    rng = np.random.default_rng(51)
    K, fout = 3, 4
    indptr, indices, X, W, c, mu, inv_sigma = make_case(rng, 30, 140, 5, fout, K)
    gout = rng.standard_normal((30, fout))
    perm = np.array([1, 2, 0])
    cols = (perm[:, None] * fout + np.arange(fout)[None, :]).reshape(-1)
    f0 = om.gmm_forward(indptr, indices, X, W, c, mu, inv_sigma)
    f1 = om.gmm_forward(indptr, indices, X, W[:, cols], c, mu[perm], inv_sigma[perm])
    np.testing.assert_allclose(f1["out"], f0["out"], rtol=1e-12, atol=1e-12)
    b0 = om.gmm_backward(indptr, indices, X, W, c, mu, inv_sigma, gout, f0)
    b1 = om.gmm_backward(indptr, indices, X, W[:, cols], c, mu[perm], inv_sigma[perm], gout, f1)
    np.testing.assert_allclose(b1["gmu"], b0["gmu"][perm], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b1["ginv_sigma"], b0["ginv_sigma"][perm], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b1["gw_fc"], b0["gw_fc"][:, cols], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b1["gx"], b0["gx"], rtol=1e-10, atol=1e-12)


def test_far_away_kernels_contribute_nothing_and_scale_is_one_over_k():
    """A kernel whose mean is far from every pseudo-coordinate has weight exp(-large) = 0;
    with K identical kernels the 1/K factor makes the layer equal to the single-kernel one."""
    rng = np.random.default_rng(52)
    fout = 4
    indptr, indices, X, W1, c, mu1, is1 = make_case(rng, 25, 100, 5, fout, 1)
    f1 = om.gmm_forward(indptr, indices, X, W1, c, mu1, is1)
    # three copies of the same kernel
    f3 = om.gmm_forward(indptr, indices, X, np.tile(W1, (1, 3)), c, np.tile(mu1, (3, 1)), np.tile(is1, (3, 1)))
    np.testing.assert_allclose(f3["out"], f1["out"], rtol=1e-12, atol=1e-12)
    # one real kernel plus one far away: half of the single-kernel output
    mu2 = np.vstack([mu1, [[1e3, 1e3]]])
    f2 = om.gmm_forward(indptr, indices, X, np.hstack([W1, rng.standard_normal(W1.shape)]), c, mu2,
                        np.vstack([is1, [[1.0, 1.0]]]))
    np.testing.assert_allclose(f2["out"], 0.5 * f1["out"], rtol=1e-12, atol=1e-12)


# ---- general pseudo-coordinates and their projection ---------------------------------------
def _pcase(seed, n=30, m=110, fin=4, fout=3, K=2, r=3):
    rng = np.random.default_rng(seed)
    indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=True)
    E = len(indices)
    return dict(indptr=indptr, indices=indices, H=rng.standard_normal((n, fin)),
                W=rng.standard_normal((fin, K * fout)) * 0.5, pseudo=rng.uniform(-1, 1, (E, r)),
                mu=rng.standard_normal((K, r)) * 0.4, isg=0.5 + rng.random((K, r)),
                gout=rng.standard_normal((n, fout)), K=K, r=r, fout=fout)


def test_general_pseudo_reduces_to_the_degree_pair_layer():
    from oracle.segments import edge_dst
    rng = np.random.default_rng(21)
    n = 25
    indptr, indices = random_graph(rng, n, 90, self_loops=True, duplicates=True)
    H, W = rng.standard_normal((n, 5)), rng.standard_normal((5, 3 * 4))
    c = rng.uniform(0.2, 1.0, n)
    mu, isg = rng.standard_normal((3, 2)) * 0.3, 0.5 + rng.random((3, 2))
    gout = rng.standard_normal((n, 4))
    pseudo = np.stack([c[indices], c[edge_dst(indptr)]], axis=1)
    a = om.gmm_forward(indptr, indices, H, W, c, mu, isg)
    b = om.gmm_pseudo_forward(indptr, indices, H, W, pseudo, mu, isg)
    np.testing.assert_allclose(b["out"], a["out"], rtol=1e-13, atol=1e-13)
    ga = om.gmm_backward(indptr, indices, H, W, c, mu, isg, gout, a)
    gb = om.gmm_pseudo_backward(indptr, indices, H, W, pseudo, mu, isg, gout, b)
    for k in ("gx", "gw_fc", "gmu", "ginv_sigma"):
        np.testing.assert_allclose(gb[k], ga[k], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("r", [1, 3, 4])
def test_general_pseudo_against_loops_and_finite_differences(r):
    t = _pcase(30 + r, r=r)
    fwd = om.gmm_pseudo_forward(t["indptr"], t["indices"], t["H"], t["W"], t["pseudo"], t["mu"], t["isg"])
    # brute force: the definition edge by edge with an explicit diagonal covariance
    n, K, fout = len(t["indptr"]) - 1, t["K"], t["fout"]
    Hk = (t["H"] @ t["W"]).reshape(n, K, fout)
    ref = np.zeros((n, fout))
    for v in range(n):
        for e in range(t["indptr"][v], t["indptr"][v + 1]):
            u = t["indices"][e]
            for k in range(K):
                d = t["pseudo"][e] - t["mu"][k]
                cov_inv = np.diag(t["isg"][k] ** 2)
                ref[v] += np.exp(-0.5 * d @ cov_inv @ d) * Hk[u, k] / K
    np.testing.assert_allclose(fwd["out"], ref, rtol=1e-12, atol=1e-13)
    g = om.gmm_pseudo_backward(t["indptr"], t["indices"], t["H"], t["W"], t["pseudo"], t["mu"], t["isg"],
                               t["gout"], fwd)

    def loss(**kw):
        a = dict(H=t["H"], W=t["W"], pseudo=t["pseudo"], mu=t["mu"], isg=t["isg"])
        a.update(kw)
        o = om.gmm_pseudo_forward(t["indptr"], t["indices"], a["H"], a["W"], a["pseudo"], a["mu"], a["isg"])["out"]
        return float((t["gout"] * o).sum())
    rng = np.random.default_rng(0)
    for name, key in (("H", "gx"), ("W", "gw_fc"), ("mu", "gmu"), ("isg", "ginv_sigma"), ("pseudo", "gpseudo")):
        idx, fd = finite_difference(lambda x, name=name: loss(**{name: x}), t[name], h=1e-6, max_entries=10, rng=rng)
        np.testing.assert_allclose(g[key].reshape(-1)[idx], fd, rtol=2e-5, atol=1e-8, err_msg=name)


def test_pseudo_projection_values_and_gradients():
    rng = np.random.default_rng(40)
    n = 12
    indptr, indices = random_graph(rng, n, 30, self_loops=True, duplicates=False)
    c = rng.uniform(0.2, 1.0, n)
    P, pb = rng.standard_normal((3, 2)), rng.standard_normal(3) * 0.2
    m = om.pseudo_projection_forward(indptr, indices, c, P, pb)
    # one edge by hand
    v = int(np.flatnonzero(np.diff(indptr) > 0)[0])
    e = indptr[v]
    u = indices[e]
    np.testing.assert_allclose(m[e], np.tanh(P @ np.array([c[u], c[v]]) + pb), rtol=1e-14)
    # zero projection: every coordinate is tanh(bias)
    np.testing.assert_allclose(om.pseudo_projection_forward(indptr, indices, c, np.zeros((3, 2)), pb),
                               np.tanh(pb)[None, :].repeat(len(indices), 0), rtol=1e-14)
    g = rng.standard_normal(m.shape)
    gP, gpb = om.pseudo_projection_backward(indptr, indices, c, P, pb, g)
    _, fd = finite_difference(lambda x: float((g * om.pseudo_projection_forward(indptr, indices, c, x, pb)).sum()), P)
    np.testing.assert_allclose(gP.reshape(-1), fd, rtol=1e-6, atol=1e-9)
    _, fd = finite_difference(lambda x: float((g * om.pseudo_projection_forward(indptr, indices, c, P, x)).sum()), pb)
    np.testing.assert_allclose(gpb, fd, rtol=1e-6, atol=1e-9)
