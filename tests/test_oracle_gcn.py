"""Pins of the GCN oracle: a sparse-matrix product from a library, closed forms, finite
differences.  None of them reuses the oracle's own formula."""
import numpy as np
import scipy.sparse as sp

from helpers import finite_difference, random_graph
from oracle import gcn as og


def _case(seed=0, n=40, m=160, fin=5, fout=6):
    rng = np.random.default_rng(seed)
    indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=True)
    H = rng.standard_normal((n, fin))
    W = rng.standard_normal((fin, fout))
    c_src, c_dst = rng.uniform(0.2, 1.5, n), rng.uniform(0.2, 1.5, n)
    gout = rng.standard_normal((n, fout))
    return indptr, indices, H, W, c_src, c_dst, gout


def _adjacency(indptr, indices, n):
    # A[v, u] = number of edges u -> v (duplicates add up)
    data = np.ones(len(indices))
    return sp.csr_matrix((data, indices, indptr), shape=(n, n))


def test_forward_is_a_scaled_sparse_product():
    indptr, indices, H, W, c_src, c_dst, _ = _case(1)
    n = len(indptr) - 1
    A = _adjacency(indptr, indices, n)
    ref = sp.diags(c_dst) @ A @ sp.diags(c_src) @ (H @ W)
    out = og.gcn_forward(indptr, indices, H, W, c_src, c_dst)["out"]
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)


def test_symmetric_normalisation_and_mean_aggregation():
    rng = np.random.default_rng(2)
    n = 30
    indptr, indices = random_graph(rng, n, 120, self_loops=True, duplicates=False)
    deg = np.diff(indptr).astype(np.float64)
    H, W = rng.standard_normal((n, 4)), np.eye(4)
    # mean aggregation: constant features stay constant
    ones = np.ones((n, 4))
    out = og.gcn_forward(indptr, indices, ones, W, np.ones(n), 1.0 / deg)["out"]
    np.testing.assert_allclose(out, ones, rtol=1e-12)
    # sum aggregation of ones counts the in-degree
    out = og.gcn_forward(indptr, indices, ones, W, np.ones(n), np.ones(n))["out"]
    np.testing.assert_allclose(out[:, 0], deg, rtol=1e-12)
    # a vertex whose only in-edge is its self-loop keeps its own (scaled) row
    indptr2 = np.arange(n + 1, dtype=np.int32)
    indices2 = np.arange(n, dtype=np.int32)
    c = rng.uniform(0.5, 2.0, n)
    out = og.gcn_forward(indptr2, indices2, H, W, c, c)["out"]
    np.testing.assert_allclose(out, (c * c)[:, None] * H, rtol=1e-12)


def test_source_and_destination_scales_are_not_interchangeable():
    indptr, indices, H, W, c_src, c_dst, _ = _case(3)
    a = og.gcn_forward(indptr, indices, H, W, c_src, c_dst)["out"]
    b = og.gcn_forward(indptr, indices, H, W, c_dst, c_src)["out"]
    assert np.abs(a - b).max() > 1e-3


def test_backward_matches_finite_differences():
    indptr, indices, H, W, c_src, c_dst, gout = _case(4)
    bwd = og.gcn_backward(indptr, indices, H, W, c_src, c_dst, gout)
    loss_H = lambda t: float((gout * og.gcn_forward(indptr, indices, t, W, c_src, c_dst)["out"]).sum())
    loss_W = lambda t: float((gout * og.gcn_forward(indptr, indices, H, t, c_src, c_dst)["out"]).sum())
    rng = np.random.default_rng(5)
    idx, g = finite_difference(loss_H, H, max_entries=60, rng=rng)
    np.testing.assert_allclose(bwd["gx"].reshape(-1)[idx], g, rtol=1e-6, atol=1e-7)
    idx, g = finite_difference(loss_W, W, max_entries=30, rng=rng)
    np.testing.assert_allclose(bwd["gw"].reshape(-1)[idx], g, rtol=1e-6, atol=1e-7)


def test_backward_is_the_transposed_product():
    indptr, indices, H, W, c_src, c_dst, gout = _case(6)
    n = len(indptr) - 1
    A = _adjacency(indptr, indices, n)
    dZ = sp.diags(c_src) @ A.T @ sp.diags(c_dst) @ gout
    bwd = og.gcn_backward(indptr, indices, H, W, c_src, c_dst, gout)
    np.testing.assert_allclose(bwd["dZ"], dZ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(bwd["gw"], H.T @ dZ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(bwd["gx"], dZ @ W.T, rtol=1e-12, atol=1e-12)


# ---- general static edge weights ----------------------------------------------------------------
def _weighted_adjacency(indptr, indices, ew, n):
    # A[v, u] = sum of the weights of the edges u -> v (scipy adds duplicates when it multiplies)
    return sp.csr_matrix((np.asarray(ew, dtype=np.float64), indices, indptr), shape=(n, n))


def test_edge_weighted_forward_and_backward_are_sparse_products():
    indptr, indices, H, W, _, _, gout = _case(11)
    n = len(indptr) - 1
    rng = np.random.default_rng(12)
    ew = rng.standard_normal(len(indices))                 # both signs, duplicates weighted separately
    A = _weighted_adjacency(indptr, indices, ew, n)
    fwd = og.gcn_edge_forward(indptr, indices, H, W, ew)
    np.testing.assert_allclose(fwd["out"], A @ (H @ W), rtol=1e-12, atol=1e-12)
    bwd = og.gcn_edge_backward(indptr, indices, H, W, ew, gout, fwd)
    dZ = A.T @ gout
    np.testing.assert_allclose(bwd["gw"], H.T @ dZ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(bwd["gx"], dZ @ W.T, rtol=1e-12, atol=1e-12)


def test_edge_weighted_layer_reduces_to_the_separable_one():
    indptr, indices, H, W, c_src, c_dst, gout = _case(13)
    dst = np.repeat(np.arange(len(indptr) - 1), np.diff(indptr))
    ew = c_src[indices] * c_dst[dst]
    a = og.gcn_forward(indptr, indices, H, W, c_src, c_dst)["out"]
    b = og.gcn_edge_forward(indptr, indices, H, W, ew)["out"]
    np.testing.assert_allclose(b, a, rtol=1e-12, atol=1e-12)
    ga = og.gcn_backward(indptr, indices, H, W, c_src, c_dst, gout)
    gb = og.gcn_edge_backward(indptr, indices, H, W, ew, gout)
    for k in ("gx", "gw"):
        np.testing.assert_allclose(gb[k], ga[k], rtol=1e-12, atol=1e-12)


def test_edge_weighted_closed_forms_and_finite_differences():
    # two vertices, edges 0 -> 1 (weight 2), 1 -> 1 (weight -3), 1 -> 0 (weight 5); W = identity
    indptr, indices = np.array([0, 1, 3], dtype=np.int32), np.array([1, 0, 1], dtype=np.int32)
    H = np.array([[1.0, 10.0], [100.0, 1000.0]])
    out = og.gcn_edge_forward(indptr, indices, H, np.eye(2), np.array([5.0, 2.0, -3.0]))["out"]
    np.testing.assert_allclose(out, [[500.0, 5000.0], [2.0 - 300.0, 20.0 - 3000.0]])
    # zero weights switch edges off; a weight on a missing gradient path leaves the others alone
    indptr, indices, H, W, _, _, gout = _case(14)
    rng = np.random.default_rng(15)
    ew = rng.uniform(-1.0, 1.0, len(indices))
    assert not og.gcn_edge_forward(indptr, indices, H, W, np.zeros_like(ew))["out"].any()
    bwd = og.gcn_edge_backward(indptr, indices, H, W, ew, gout)
    loss_H = lambda t: float((gout * og.gcn_edge_forward(indptr, indices, t, W, ew)["out"]).sum())
    loss_W = lambda t: float((gout * og.gcn_edge_forward(indptr, indices, H, t, ew)["out"]).sum())
    idx, g = finite_difference(loss_H, H, max_entries=60, rng=rng)
    np.testing.assert_allclose(bwd["gx"].reshape(-1)[idx], g, rtol=1e-6, atol=1e-7)
    idx, g = finite_difference(loss_W, W, max_entries=30, rng=rng)
    np.testing.assert_allclose(bwd["gw"].reshape(-1)[idx], g, rtol=1e-6, atol=1e-7)
