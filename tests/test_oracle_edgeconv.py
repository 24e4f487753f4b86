"""Pins for the EdgeConv oracle (App. A.2 "EdgeConv")."""
import numpy as np
import pytest
import torch

from oracle import edgeconv as oe
from helpers import finite_difference, random_graph, tiny_graph


def make_case(rng, n, m, fin, fout, duplicates=False):
    indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=duplicates)
    X = rng.standard_normal((n, fin))
    Theta = rng.standard_normal((fin, fout)) * 0.5
    Phi = rng.standard_normal((fin, fout)) * 0.5
    return indptr, indices, X, Theta, Phi


def brute_force(indptr, indices, X, Theta, Phi):
    n, fout = len(indptr) - 1, Theta.shape[1]
    out = np.zeros((n, fout))
    arg = -np.ones((n, fout), dtype=np.int64)
    for v in range(n):
        for f in range(fout):
            best = None
            for e in range(indptr[v], indptr[v + 1]):
                u = indices[e]
                val = sum((X[u, i] - X[v, i]) * Theta[i, f] for i in range(X.shape[1])) \
                    + sum(X[v, i] * Phi[i, f] for i in range(X.shape[1]))
                if best is None or val > best:
                    best, arg[v, f] = val, e
            out[v, f] = 0.0 if best is None else best
    return out, arg


def test_forward_matches_loop_brute_force():
    rng = np.random.default_rng(1)
    indptr, indices, X, Theta, Phi = make_case(rng, 14, 40, 3, 4)
    fwd = oe.edgeconv_forward(indptr, indices, X, Theta, Phi)
    out, arg = brute_force(indptr, indices, X, Theta, Phi)
    np.testing.assert_allclose(fwd["out"], out, rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(fwd["argmax"], arg)


def test_reorganized_form_agrees_by_linearity():
    # Theta (h_u - h_v) + Phi h_v = (H Theta)[u] + (H (Phi - Theta))[v]   (Sec. 4)
    rng = np.random.default_rng(2)
    indptr, indices, X, Theta, Phi = make_case(rng, 40, 240, 6, 5)
    fwd = oe.edgeconv_forward(indptr, indices, X, Theta, Phi)
    P, Q = X @ Theta, X @ (Phi - Theta)
    ref = np.zeros_like(fwd["out"])
    for v in range(40):
        ref[v] = P[indices[indptr[v]:indptr[v + 1]]].max(axis=0) + Q[v]
    np.testing.assert_allclose(fwd["out"], ref, rtol=1e-12, atol=1e-12)


def test_special_cases_reduce_to_plain_products():
    rng = np.random.default_rng(3)
    indptr, indices, X, Theta, Phi = make_case(rng, 30, 150, 5, 4)
    # Theta = 0: the neighbourhood drops out
    out = oe.edgeconv_forward(indptr, indices, X, 0 * Theta, Phi)["out"]
    np.testing.assert_allclose(out, X @ Phi, rtol=1e-13, atol=1e-13)
    # Phi = Theta: out[v] = max_u (X Theta)[u]
    out = oe.edgeconv_forward(indptr, indices, X, Theta, Theta)["out"]
    P = X @ Theta
    ref = np.stack([P[indices[indptr[v]:indptr[v + 1]]].max(axis=0) for v in range(30)])
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    # self-loop only: out = X Phi
    ip = np.arange(31, dtype=np.int32)
    ix = np.arange(30, dtype=np.int32)
    out = oe.edgeconv_forward(ip, ix, X, Theta, Phi)["out"]
    np.testing.assert_allclose(out, X @ Phi, rtol=1e-13, atol=1e-13)


def test_first_edge_wins_an_exact_tie_and_empty_row():
    # duplicate edge (1 -> 0) twice: identical messages, the earlier CSR position wins
    indptr, indices = tiny_graph(3, [(1, 0), (1, 0), (2, 1)])
    X = np.array([[0.0, 1.0], [2.0, -1.0], [0.5, 0.5]])
    Theta = np.array([[1.0, -1.0], [0.5, 2.0]])
    Phi = np.array([[0.3, 0.1], [0.2, -0.4]])
    fwd = oe.edgeconv_forward(indptr, indices, X, Theta, Phi)
    np.testing.assert_array_equal(fwd["argmax"][0], [0, 0])
    np.testing.assert_array_equal(fwd["argmax"][2], [-1, -1])
    np.testing.assert_array_equal(fwd["out"][2], [0.0, 0.0])
    mask = oe.near_tie_mask(indptr, fwd, 1e-9)
    assert mask[0].all() and not mask[1].any() and not mask[2].any()


def _loss(indptr, indices, X, Theta, Phi, gout):
    return float((oe.edgeconv_forward(indptr, indices, X, Theta, Phi)["out"] * gout).sum())


def test_backward_matches_finite_differences():
    rng = np.random.default_rng(4)
    indptr, indices, X, Theta, Phi = make_case(rng, 12, 40, 3, 4)
    gout = rng.standard_normal((12, 4))
    fwd = oe.edgeconv_forward(indptr, indices, X, Theta, Phi)
    assert not oe.near_tie_mask(indptr, fwd, 1e-3).any()
    bwd = oe.edgeconv_backward(indptr, indices, X, Theta, Phi, gout, fwd)
    for name, theta, fun in [
        ("gx", X, lambda t: _loss(indptr, indices, t, Theta, Phi, gout)),
        ("gtheta", Theta, lambda t: _loss(indptr, indices, X, t, Phi, gout)),
        ("gphi", Phi, lambda t: _loss(indptr, indices, X, Theta, t, gout)),
    ]:
        idx, g = finite_difference(fun, theta)
        np.testing.assert_allclose(bwd[name].reshape(-1)[idx], g, rtol=1e-6, atol=1e-7, err_msg=name)


def test_backward_matches_torch_autograd():
    rng = np.random.default_rng(5)
    n = 20
    indptr, indices, X, Theta, Phi = make_case(rng, n, 90, 4, 3)
    gout = rng.standard_normal((n, 3))
    tX, tT, tP = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (X, Theta, Phi))
    rows = []
    for v in range(n):
        nb = torch.tensor(indices[indptr[v]:indptr[v + 1]].astype(np.int64))
        msg = (tX[nb] - tX[v]) @ tT + tX[v] @ tP
        rows.append(msg.max(dim=0).values)
    (torch.stack(rows) * torch.tensor(gout)).sum().backward()
    bwd = oe.edgeconv_backward(indptr, indices, X, Theta, Phi, gout)
    np.testing.assert_allclose(bwd["gx"], tX.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["gtheta"], tT.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["gphi"], tP.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_translating_all_points_moves_the_output_by_the_phi_image_only():
    """Theta sees differences of features, so a common shift t of every vertex only enters
    through Phi: out(x + t) = out(x) + t Phi, with the same winners."""
    rng = np.random.default_rng(41)
    indptr, indices, X, Theta, Phi = make_case(rng, 30, 150, 5, 6)
    t = rng.standard_normal(5)
    f0 = oe.edgeconv_forward(indptr, indices, X, Theta, Phi)
    f1 = oe.edgeconv_forward(indptr, indices, X + t[None, :], Theta, Phi)
    has_edges = np.diff(indptr) > 0
    np.testing.assert_allclose(f1["out"][has_edges], (f0["out"] + (t @ Phi)[None, :])[has_edges], rtol=1e-10, atol=1e-10)
    assert np.array_equal(f1["argmax"], f0["argmax"])


def test_backward_is_linear_in_the_upstream_gradient():
    rng = np.random.default_rng(42)
    indptr, indices, X, Theta, Phi = make_case(rng, 25, 100, 4, 5)
    g1, g2 = rng.standard_normal((25, 5)), rng.standard_normal((25, 5))
    fwd = oe.edgeconv_forward(indptr, indices, X, Theta, Phi)
    b = lambda g: oe.edgeconv_backward(indptr, indices, X, Theta, Phi, g, fwd)
    b1, b2, b12 = b(g1), b(g2), b(0.5 * g1 + 4.0 * g2)
    for k in ("gx", "gtheta", "gphi"):
        np.testing.assert_allclose(b12[k], 0.5 * b1[k] + 4.0 * b2[k], rtol=1e-10, atol=1e-10)
