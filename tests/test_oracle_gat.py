"""Pins for the GAT oracle: things fixed by the paper's definition and by
mathematics, none of which re-use the oracle's own code path."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

from oracle import gat as og
from helpers import finite_difference, random_graph, tiny_graph


def dense_gat(indptr, indices, X, W, a_l, a_r, slope):
    """Masked dense attention (App. A.2 GAT with the Eq. 1 score), per head, with
    an adjacency COUNT matrix so duplicate edges weigh as distinct edges."""
    n = len(indptr) - 1
    heads, F = a_l.shape
    C = np.zeros((n, n))
    for v in range(n):
        for e in range(indptr[v], indptr[v + 1]):
            C[v, indices[e]] += 1.0
    Z = (X.astype(np.float64) @ W.astype(np.float64)).reshape(n, heads, F)
    out = np.zeros((n, heads, F))
    alphas = []
    for h in range(heads):
        sl = Z[:, h, :] @ a_l[h].astype(np.float64)      # source half
        sr = Z[:, h, :] @ a_r[h].astype(np.float64)      # destination half
        S = sr[:, None] + sl[None, :]                    # S[v, u]
        S = np.where(S > 0, S, slope * S)
        A = np.zeros((n, n))
        for v in range(n):
            if C[v].sum() == 0:
                continue
            mask = C[v] > 0
            ex = np.zeros(n)
            ex[mask] = C[v, mask] * np.exp(S[v, mask] - S[v, mask].max())
            A[v] = ex / ex.sum()
        out[:, h, :] = A @ Z[:, h, :]
        alphas.append(A)
    return out.reshape(n, heads * F), alphas


def make_case(rng, n, m, fin, heads, F, duplicates=False, self_loops=True):
    indptr, indices = random_graph(rng, n, m, self_loops=self_loops, duplicates=duplicates)
    X = rng.standard_normal((n, fin))
    W = rng.standard_normal((fin, heads * F)) * 0.4
    a_l = rng.standard_normal((heads, F)) * 0.5
    a_r = rng.standard_normal((heads, F)) * 0.5
    return indptr, indices, X, W, a_l, a_r


@pytest.mark.parametrize("heads,F,dups", [(1, 4, False), (3, 5, False), (2, 3, True)])
def test_forward_matches_dense_masked_attention(heads, F, dups):
    rng = np.random.default_rng(10 + heads)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 23, 90, 7, heads, F, duplicates=dups,
                                                self_loops=False)
    fwd = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    ref, _ = dense_gat(indptr, indices, X, W, a_l, a_r, 0.2)
    np.testing.assert_allclose(fwd["out"], ref, rtol=1e-12, atol=1e-12)


def test_two_vertex_closed_form():
    # v0 receives edges from v0 and v1; one head, F = 1, W = 1.
    indptr, indices = tiny_graph(2, [(0, 0), (1, 0)])
    X = np.array([[1.0], [2.0]])
    W = np.array([[1.0]])
    e = np.e
    # a = [a_l || a_r] = [1, 0]: scores 1 and 2, positive -> LeakyReLU is identity
    out = og.gat_forward(indptr, indices, X, W, np.array([[1.0]]), np.array([[0.0]]), 0.2)["out"]
    assert out[0, 0] == pytest.approx((1 + 2 * e) / (1 + e), rel=1e-14)
    assert out[1, 0] == 0.0
    # a = [-1, 0]: scores -1, -2 -> LeakyReLU gives -0.2, -0.4
    out = og.gat_forward(indptr, indices, X, W, np.array([[-1.0]]), np.array([[0.0]]), 0.2)["out"]
    w0, w1 = np.exp(-0.2), np.exp(-0.4)
    assert out[0, 0] == pytest.approx((w0 + 2 * w1) / (w0 + w1), rel=1e-14)
    # a = [0, 3]: the destination half is common to all in-edges -> uniform weights
    out = og.gat_forward(indptr, indices, X, W, np.array([[0.0]]), np.array([[3.0]]), 0.2)["out"]
    assert out[0, 0] == pytest.approx(1.5, rel=1e-14)


def test_source_and_destination_halves_are_not_interchangeable():
    # star into vertex 0: the score must depend on the SOURCE through a_l
    indptr, indices = tiny_graph(3, [(1, 0), (2, 0)])
    X = np.array([[0.0], [1.0], [5.0]])
    W = np.array([[1.0]])
    out = og.gat_forward(indptr, indices, X, W, np.array([[1.0]]), np.array([[0.0]]), 0.2)["out"]
    w1, w2 = 1.0, np.exp(4.0)
    assert out[0, 0] == pytest.approx((1 * w1 + 5 * w2) / (w1 + w2), rel=1e-13)


def test_zero_attention_vector_is_mean_aggregation():
    rng = np.random.default_rng(3)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 40, 200, 6, 2, 4)
    fwd = og.gat_forward(indptr, indices, X, W, 0 * a_l, 0 * a_r, 0.2)
    n = 40
    A = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(n, n))
    deg = np.asarray(A.sum(axis=1)).ravel()
    ref = sp.diags(1.0 / deg) @ A @ (X @ W)
    np.testing.assert_allclose(fwd["out"], ref, rtol=1e-12, atol=1e-13)


def test_softmax_weights_sum_to_one_and_ranges():
    rng = np.random.default_rng(4)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 50, 300, 5, 3, 4)
    fwd = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    dst = fwd["dst"]
    sums = np.zeros((50, 3))
    np.add.at(sums, dst, fwd["M2"])
    np.testing.assert_allclose(sums, 1.0, rtol=1e-13)
    assert (fwd["M2"] > 0).all() and (fwd["M2"] <= 1).all()
    # the saved maximum is the largest activated score of the row
    for v in (0, 7, 31):
        seg = fwd["M1"][indptr[v]:indptr[v + 1]]
        np.testing.assert_array_equal(fwd["mx"][v], seg.max(axis=0))


def test_in_degree_one_copies_the_source_row_and_empty_row_is_zero():
    indptr, indices = tiny_graph(4, [(2, 0), (3, 1), (0, 1)])
    rng = np.random.default_rng(5)
    X = rng.standard_normal((4, 3))
    W = rng.standard_normal((3, 8))
    a_l = rng.standard_normal((2, 4))
    a_r = rng.standard_normal((2, 4))
    fwd = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    np.testing.assert_allclose(fwd["out"][0], (X @ W)[2], rtol=1e-14)
    np.testing.assert_array_equal(fwd["out"][2], 0.0)
    np.testing.assert_array_equal(fwd["out"][3], 0.0)
    np.testing.assert_array_equal(fwd["mx"][2], 0.0)
    np.testing.assert_array_equal(fwd["den"][2], 1.0)


def test_edge_order_inside_a_row_does_not_matter():
    rng = np.random.default_rng(6)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 30, 150, 5, 2, 4)
    out = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)["out"]
    perm = indices.copy()
    for v in range(30):
        seg = perm[indptr[v]:indptr[v + 1]]
        perm[indptr[v]:indptr[v + 1]] = seg[::-1]
    out2 = og.gat_forward(indptr, perm, X, W, a_l, a_r, 0.2)["out"]
    np.testing.assert_allclose(out, out2, rtol=1e-12, atol=1e-13)


def test_split_score_identity_of_the_reorganization():
    # a^T [h_u || h_v] = a_l^T h_u + a_r^T h_v   (Sec. 4, text after Eq. 1)
    rng = np.random.default_rng(7)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 25, 100, 5, 2, 4)
    fwd = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    Z = (X @ W).reshape(25, 2, 4)
    A_l = np.einsum("nhf,hf->nh", Z, a_l)
    A_r = np.einsum("nhf,hf->nh", Z, a_r)
    np.testing.assert_allclose(fwd["M0"], A_l[fwd["src"]] + A_r[fwd["dst"]], rtol=1e-12, atol=1e-13)


def _loss(indptr, indices, X, W, a_l, a_r, slope, gout):
    return float((og.gat_forward(indptr, indices, X, W, a_l, a_r, slope)["out"] * gout).sum())


@pytest.mark.parametrize("heads,F,dups", [(1, 4, False), (2, 3, True)])
def test_backward_matches_finite_differences(heads, F, dups):
    rng = np.random.default_rng(20 + heads)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 12, 40, 4, heads, F, duplicates=dups)
    gout = rng.standard_normal((12, heads * F))
    fwd = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    assert np.abs(fwd["M0"]).min() > 1e-4          # stay away from the LeakyReLU kink
    bwd = og.gat_backward(indptr, indices, X, W, a_l, a_r, 0.2, gout, fwd)
    checks = [
        ("gx", X, lambda t: _loss(indptr, indices, t, W, a_l, a_r, 0.2, gout)),
        ("gw", W, lambda t: _loss(indptr, indices, X, t, a_l, a_r, 0.2, gout)),
        ("ga_l", a_l, lambda t: _loss(indptr, indices, X, W, t, a_r, 0.2, gout)),
        ("ga_r", a_r, lambda t: _loss(indptr, indices, X, W, a_l, t, 0.2, gout)),
    ]
    for name, theta, fun in checks:
        idx, g = finite_difference(fun, theta)
        np.testing.assert_allclose(bwd[name].reshape(-1)[idx], g, rtol=2e-6, atol=2e-7,
                                   err_msg=name)


def test_backward_matches_torch_autograd_on_the_dense_formula():
    rng = np.random.default_rng(30)
    n, fin, heads, F = 15, 5, 2, 4
    indptr, indices, X, W, a_l, a_r = make_case(rng, n, 60, fin, heads, F)
    gout = rng.standard_normal((n, heads * F))
    mask = np.zeros((n, n), dtype=bool)
    for v in range(n):
        mask[v, indices[indptr[v]:indptr[v + 1]]] = True
    tX, tW, tal, tar = (torch.tensor(a, dtype=torch.float64, requires_grad=True)
                        for a in (X, W, a_l, a_r))
    Z = (tX @ tW).reshape(n, heads, F)
    sl = (Z * tal[None]).sum(-1)           # [n, heads] source half
    sr = (Z * tar[None]).sum(-1)
    S = torch.nn.functional.leaky_relu(sr[:, None, :] + sl[None, :, :], 0.2)   # [v, u, h]
    S = S.masked_fill(~torch.tensor(mask)[:, :, None], float("-inf"))
    A = torch.softmax(S, dim=1)
    out = torch.einsum("vuh,uhf->vhf", A, Z).reshape(n, heads * F)
    (out * torch.tensor(gout)).sum().backward()
    bwd = og.gat_backward(indptr, indices, X, W, a_l, a_r, 0.2, gout)
    np.testing.assert_allclose(bwd["gx"], tX.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["gw"], tW.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["ga_l"], tal.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(bwd["ga_r"], tar.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_slope_one_kills_the_destination_half_gradient():
    # with slope 1 LeakyReLU is the identity, a_r^T h_v is a per-row constant and
    # cancels inside the softmax: no gradient reaches a_r through the scores
    rng = np.random.default_rng(31)
    indptr, indices, X, W, a_l, a_r = make_case(rng, 20, 80, 4, 2, 3)
    gout = rng.standard_normal((20, 6))
    bwd = og.gat_backward(indptr, indices, X, W, a_l, a_r, 1.0, gout)
    np.testing.assert_allclose(bwd["ga_r"], 0.0, atol=1e-12)
    # softmax Jacobian: the score gradients of a row sum to zero
    s = np.zeros((20, 2))
    np.add.at(s, og.edge_dst(indptr), bwd["dM1"])
    np.testing.assert_allclose(s, 0.0, atol=1e-12)


def test_heads_are_independent_and_laid_out_head_major():
    """Permuting the heads (column blocks of W, rows of a_l and a_r) permutes the output's
    column blocks and nothing else (App. A.2: heads are concatenated)."""
    rng = np.random.default_rng(31)
    indptr, indices = random_graph(rng, 25, 90, self_loops=True, duplicates=True)
    H, F, fin = 3, 4, 5
    X = rng.standard_normal((25, fin))
    W = rng.standard_normal((fin, H * F))
    a_l, a_r = rng.standard_normal((H, F)), rng.standard_normal((H, F))
    gout = rng.standard_normal((25, H * F))
    perm = np.array([2, 0, 1])
    cols = (perm[:, None] * F + np.arange(F)[None, :]).reshape(-1)
    f0 = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    f1 = og.gat_forward(indptr, indices, X, W[:, cols], a_l[perm], a_r[perm], 0.2)
    np.testing.assert_allclose(f1["out"], f0["out"][:, cols], rtol=1e-12, atol=1e-12)
    b0 = og.gat_backward(indptr, indices, X, W, a_l, a_r, 0.2, gout, f0)
    b1 = og.gat_backward(indptr, indices, X, W[:, cols], a_l[perm], a_r[perm], 0.2, gout[:, cols], f1)
    np.testing.assert_allclose(b1["gx"], b0["gx"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b1["gw"], b0["gw"][:, cols], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(b1["ga_l"], b0["ga_l"][perm], rtol=1e-10, atol=1e-12)


def test_backward_is_linear_in_the_upstream_gradient_and_local():
    """Every gradient is a linear map of gout; a destination with zero upstream gradient and
    no out-edges contributes nothing."""
    rng = np.random.default_rng(32)
    indptr, indices = random_graph(rng, 30, 120, self_loops=True, duplicates=False)
    H, F, fin = 2, 4, 6
    X, W = rng.standard_normal((30, fin)), rng.standard_normal((fin, H * F))
    a_l, a_r = rng.standard_normal((H, F)), rng.standard_normal((H, F))
    g1, g2 = rng.standard_normal((30, H * F)), rng.standard_normal((30, H * F))
    fwd = og.gat_forward(indptr, indices, X, W, a_l, a_r, 0.2)
    b = lambda g: og.gat_backward(indptr, indices, X, W, a_l, a_r, 0.2, g, fwd)
    b1, b2, b12 = b(g1), b(g2), b(2.0 * g1 - 3.0 * g2)
    for k in ("gx", "gw", "ga_l", "ga_r"):
        np.testing.assert_allclose(b12[k], 2.0 * b1[k] - 3.0 * b2[k], rtol=1e-10, atol=1e-10)
    z = b(np.zeros_like(g1))
    for k in ("gx", "gw", "ga_l", "ga_r"):
        assert np.abs(z[k]).max() == 0.0


def test_a_uniform_shift_of_the_scores_changes_nothing():
    """Softmax is shift-invariant: adding a constant feature direction that raises every
    destination score by the same amount leaves the attention weights alone."""
    rng = np.random.default_rng(33)
    indptr, indices = random_graph(rng, 20, 80, self_loops=True, duplicates=False)
    F, fin = 4, 3
    X, W = rng.standard_normal((20, fin)), rng.standard_normal((fin, F))
    a_l, a_r = rng.standard_normal((1, F)), rng.standard_normal((1, F))
    f0 = og.gat_forward(indptr, indices, X, W, a_l, a_r, 1.0)            # slope 1: scores are linear
    # with slope 1 the destination half is constant along a row and cancels in the softmax
    f1 = og.gat_forward(indptr, indices, X, W, a_l, 5.0 * a_r, 1.0)
    np.testing.assert_allclose(f1["out"], f0["out"], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(f1["M2"], f0["M2"], rtol=1e-10, atol=1e-12)
