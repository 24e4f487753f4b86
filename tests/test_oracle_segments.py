"""Pins for the per-destination reductions and the row restriction the sampled full-size
comparisons rely on (the Gather operator of App. A.1 over CSR-by-destination edge tensors).
None of them re-uses the code under test: plain Python loops, scipy's sparse slicing, and the
layer oracles evaluated on the whole graph."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import gat as og
from oracle import gcn as ogcn
from oracle import gmm as ogmm
from oracle.segments import edge_dst, restrict_rows, segment_max, segment_sum
from helpers import tiny_graph


def graph_with_empty_rows(rng, n=17, m=60):
    """Random multigraph in which every fourth vertex has no in-edge."""
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    edges = [(int(s), int(d)) for s, d in zip(src, dst) if d % 4 != 1]
    return tiny_graph(n, edges)


def test_edge_dst_and_segment_reductions_against_loops():
    rng = np.random.default_rng(3)
    ip, ix = graph_with_empty_rows(rng)
    n = len(ip) - 1
    assert (np.diff(ip) == 0).any() and (np.diff(ip) > 1).any()
    vals = rng.standard_normal((len(ix), 3))
    dst = edge_dst(ip)
    s_ref, m_ref = np.zeros((n, 3)), np.full((n, 3), -7.0)
    for v in range(n):
        for e in range(ip[v], ip[v + 1]):
            assert dst[e] == v
        if ip[v + 1] > ip[v]:
            s_ref[v] = sum(vals[e] for e in range(ip[v], ip[v + 1]))
            m_ref[v] = np.max(vals[ip[v]:ip[v + 1]], axis=0)
    np.testing.assert_allclose(segment_sum(ip, vals), s_ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(segment_max(ip, vals, empty=-7.0), m_ref)


def test_restrict_rows_on_a_hand_worked_graph():
    # rows: 0 <- {1, 2}, 1 <- {}, 2 <- {0, 0, 3} (a duplicate edge), 3 <- {3}
    ip, ix = tiny_graph(4, [(1, 0), (2, 0), (0, 2), (0, 2), (3, 2), (3, 3)])
    rip, rix, pos = restrict_rows(ip, ix, [2])
    assert rip.tolist() == [0, 0, 0, 3, 3]
    assert rix.tolist() == [0, 0, 3]
    assert pos.tolist() == [2, 3, 4]
    rip, rix, pos = restrict_rows(ip, ix, [3, 0])            # order and type of `rows` do not matter
    assert rip.tolist() == [0, 2, 2, 2, 3]
    assert rix.tolist() == [1, 2, 3]
    assert pos.tolist() == [0, 1, 5]
    rip, rix, pos = restrict_rows(ip, ix, np.array([1], dtype=np.int32))   # an empty row
    assert rip.tolist() == [0, 0, 0, 0, 0] and rix.size == 0 and pos.size == 0
    rip, rix, pos = restrict_rows(ip, ix, [0, 1, 2, 3])      # everything: the identity
    assert np.array_equal(rip, ip) and np.array_equal(rix, ix) and pos.tolist() == list(range(6))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_restrict_rows_is_scipys_row_mask(seed):
    """Kept rows keep their in-edges in CSR order, every other row becomes empty, `pos` names
    the kept CSR positions: the same as zeroing the other rows of the sparse matrix whose data
    are the CSR positions."""
    rng = np.random.default_rng(seed)
    ip, ix = graph_with_empty_rows(rng, n=40, m=300)
    n, E = len(ip) - 1, len(ix)
    rows = rng.choice(n, size=11, replace=False)
    rip, rix, pos = restrict_rows(ip, ix, rows)
    A = sp.csr_matrix((np.arange(1, E + 1), ix, ip), shape=(n, n))   # has_canonical_format is not assumed
    keep = np.zeros(n, dtype=bool)
    keep[rows] = True
    for v in range(n):
        got_src = rix[rip[v]:rip[v + 1]].tolist()
        got_pos = pos[rip[v]:rip[v + 1]].tolist()
        if keep[v]:
            assert got_src == A.indices[A.indptr[v]:A.indptr[v + 1]].tolist()
            assert got_pos == (A.data[A.indptr[v]:A.indptr[v + 1]] - 1).tolist()
        else:
            assert got_src == [] and got_pos == []
    assert rip[0] == 0 and rip[-1] == len(rix) == len(pos)
    assert np.array_equal(ix[pos], rix)


def test_layer_oracles_on_a_restricted_graph_give_the_full_graphs_rows():
    """What the sampled comparisons assume: a destination row depends on its own in-edges only, so
    the oracle on the restricted graph reproduces the kept rows of the oracle on the whole graph,
    and with the upstream gradient zeroed outside the kept rows the backward pass of the whole
    graph equals the backward pass of the restricted one, for every gradient."""
    rng = np.random.default_rng(5)
    ip, ix = graph_with_empty_rows(rng, n=60, m=500)
    n = len(ip) - 1
    fin, H, F = 6, 2, 4
    X = rng.standard_normal((n, fin))
    W = rng.standard_normal((fin, H * F)) * 0.4
    a_l, a_r = rng.standard_normal((H, F)) * 0.5, rng.standard_normal((H, F)) * 0.5
    rows = rng.choice(n, size=13, replace=False)
    keep = np.zeros(n, dtype=bool)
    keep[rows] = True
    gout = rng.standard_normal((n, H * F)) * keep[:, None]
    rip, rix, pos = restrict_rows(ip, ix, rows)

    full = og.gat_forward(ip, ix, X, W, a_l, a_r, 0.2)
    part = og.gat_forward(rip, rix, X, W, a_l, a_r, 0.2)
    np.testing.assert_allclose(part["out"][rows], full["out"][rows], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(part["M2"], full["M2"][pos], rtol=1e-13, atol=1e-13)
    assert not part["out"][~keep].any()
    bf = og.gat_backward(ip, ix, X, W, a_l, a_r, 0.2, gout, full)
    bp = og.gat_backward(rip, rix, X, W, a_l, a_r, 0.2, gout, part)
    for k in ("gx", "gw", "ga_l", "ga_r"):
        np.testing.assert_allclose(bp[k], bf[k], rtol=1e-11, atol=1e-12, err_msg=k)

    c_src, c_dst = rng.uniform(0.5, 1.5, n), rng.uniform(0.5, 1.5, n)
    Wg = rng.standard_normal((fin, 8)) * 0.4
    gfull = ogcn.gcn_forward(ip, ix, X, Wg, c_src, c_dst)
    gpart = ogcn.gcn_forward(rip, rix, X, Wg, c_src, c_dst)
    np.testing.assert_allclose(gpart["out"][rows], gfull["out"][rows], rtol=1e-13, atol=1e-13)
    bf = ogcn.gcn_backward(ip, ix, X, Wg, c_src, c_dst, gout)
    bp = ogcn.gcn_backward(rip, rix, X, Wg, c_src, c_dst, gout)
    for k in ("gx", "gw"):
        np.testing.assert_allclose(bp[k], bf[k], rtol=1e-11, atol=1e-12, err_msg=k)

    K, R = 2, 1
    w_fc = rng.standard_normal((fin, K * 4)) * 0.4
    pseudo = rng.standard_normal((len(ix), R))
    mu, isg = rng.standard_normal((K, R)) * 0.3, rng.uniform(0.5, 1.5, (K, R))
    go4 = rng.standard_normal((n, 4)) * keep[:, None]
    mfull = ogmm.gmm_pseudo_forward(ip, ix, X, w_fc, pseudo, mu, isg)
    mpart = ogmm.gmm_pseudo_forward(rip, rix, X, w_fc, pseudo[pos], mu, isg)
    np.testing.assert_allclose(mpart["out"][rows], mfull["out"][rows], rtol=1e-13, atol=1e-13)
    bf = ogmm.gmm_pseudo_backward(ip, ix, X, w_fc, pseudo, mu, isg, go4, mfull)
    bp = ogmm.gmm_pseudo_backward(rip, rix, X, w_fc, pseudo[pos], mu, isg, go4, mpart)
    for k in ("gx", "gw_fc", "gmu", "ginv_sigma"):
        np.testing.assert_allclose(bp[k], bf[k], rtol=1e-11, atol=1e-12, err_msg=k)
    np.testing.assert_allclose(bp["gpseudo"], bf["gpseudo"][pos], rtol=1e-11, atol=1e-12)
