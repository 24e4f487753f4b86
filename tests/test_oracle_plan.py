"""Pins for the integer plan tables and the closed-form cost model."""
import numpy as np
import scipy.sparse as sp

from oracle import cost_model as cm
from oracle import plan as op
from helpers import random_graph, tiny_graph
from workloads import graphs


def test_csc_matches_scipy_transpose_on_simple_graphs():
    rng = np.random.default_rng(1)
    indptr, indices = random_graph(rng, 60, 400, self_loops=True)
    n = 60
    A = sp.csr_matrix((np.arange(1, len(indices) + 1), indices, indptr), shape=(n, n))
    T = A.tocsc()            # column u lists the destinations of u, ascending
    T.sort_indices()
    indptr_t, indices_t, eid_t = op.csc_transpose(indptr, indices)
    np.testing.assert_array_equal(indptr_t, T.indptr)
    np.testing.assert_array_equal(indices_t, T.indices)
    np.testing.assert_array_equal(eid_t, T.data - 1)


def test_csc_keeps_csr_order_among_duplicates_and_is_a_permutation():
    indptr, indices = tiny_graph(4, [(1, 0), (1, 0), (3, 0), (1, 2), (0, 2), (1, 2)])
    indptr_t, indices_t, eid_t = op.csc_transpose(indptr, indices)
    assert sorted(eid_t.tolist()) == list(range(6))
    dst = graphs.dst_of_edges(indptr)
    np.testing.assert_array_equal(indices[eid_t], np.repeat(np.arange(4), np.diff(indptr_t)))
    np.testing.assert_array_equal(dst[eid_t], indices_t)
    for u in range(4):
        seg = eid_t[indptr_t[u]:indptr_t[u + 1]]
        assert (np.diff(seg) > 0).all()
    np.testing.assert_array_equal(indptr_t, [0, 1, 5, 5, 6])


def test_degree_buckets():
    # degrees: v0=3, v1=0, v2=1, v3=3, v4=8
    indptr = np.array([0, 3, 3, 4, 7, 15], dtype=np.int32)
    bucket, order, offsets = op.degree_buckets(indptr)
    np.testing.assert_array_equal(bucket, [30, 32, 31, 30, 28])
    np.testing.assert_array_equal(order, [4, 0, 3, 2, 1])
    assert offsets[28] == 0 and offsets[29] == 1 and offsets[30] == 1
    assert offsets[31] == 3 and offsets[32] == 4 and offsets[33] == 5
    assert op.clz32(1) == 31 and op.clz32(2**31 - 1) == 1 and op.clz32(0) == 32
    # ascending bucket along the order
    assert (np.diff(bucket[order]) >= 0).all()


def test_closed_form_operation_counts():
    indptr, _ = graphs.erdos_renyi(200, 900, 5)
    n, e = 200, int(indptr[-1])
    for f in (1, 8, 64):
        assert cm.count_gat_score_ops_by_walking(indptr, f, False) == cm.gat_score_ops_original(n, e, f)
        assert cm.count_gat_score_ops_by_walking(indptr, f, True) == cm.gat_score_ops_reorganized(n, e, f)
    # the Sec. 5 example: fusing saves 2|E|h + |E|hf elements of IO
    v, e, h, f = 232965, 114_000_000, 4, 64
    assert cm.gat_graph_io_unfused(v, e, h, f) - cm.gat_graph_io_fused(v, e, h, f) == 2 * e * h + e * h * f
    ratio = cm.gat_graph_io_unfused(v, e, h, f) / cm.gat_graph_io_fused(v, e, h, f)
    assert 1.45 < ratio < 1.55


def test_closed_forms_equal_the_printed_ones():
    """tests/golden/closed_forms.txt holds the polynomials as the paper prints them; the cost
    model's functions must evaluate to the same numbers."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")
    forms = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        name, _cite, terms = [t.strip() for t in line.split(";")]
        forms[name] = [t.strip().split("*") for t in terms.split("+")]
    assert set(forms) == {"gat_score_ops_original", "gat_score_ops_reorganized", "gat_graph_io_unfused",
                          "gat_graph_io_fused"}

    def evaluate(terms, env):
        total = 0
        for t in terms:
            prod = int(t[0])
            for sym in t[1:]:
                prod *= env[sym]
            total += prod
        return total

    for V, E, h, f in ((7, 31, 1, 1), (200, 900, 3, 8), (232965, 114_000_000, 4, 64)):
        env = dict(V=V, E=E, h=h, f=f)
        assert cm.gat_score_ops_original(V, E, f) == evaluate(forms["gat_score_ops_original"], env)
        assert cm.gat_score_ops_reorganized(V, E, f) == evaluate(forms["gat_score_ops_reorganized"], env)
        assert cm.gat_graph_io_unfused(V, E, h, f) == evaluate(forms["gat_graph_io_unfused"], env)
        assert cm.gat_graph_io_fused(V, E, h, f) == evaluate(forms["gat_graph_io_fused"], env)


def test_generators_shapes_and_degrees():
    ip, ix = graphs.erdos_renyi(2000, 10_000, 1)
    assert ip[-1] == 12_000 and ix.shape == (12_000,)
    dst = graphs.dst_of_edges(ip)
    assert (np.diff(ip) >= 1).all() and ((ix == dst).sum() == 2000)
    key = dst.astype(np.int64) * 2000 + ix
    assert (np.diff(key) > 0).all()                     # sorted, no duplicates
    ip, ix, xyz = graphs.knn_point_clouds(2, 64, 5, 3)
    assert (np.diff(ip) == 5).all() and xyz.shape == (128, 3)
    for v in (0, 70, 127):
        nb = ix[ip[v]:ip[v + 1]]
        assert v in nb and (nb // 64 == v // 64).all()
        d2 = ((xyz[nb].astype(np.float64) - xyz[v]) ** 2).sum(1)
        cloud = np.arange(64) + 64 * (v // 64)
        all_d2 = ((xyz[cloud].astype(np.float64) - xyz[v]) ** 2).sum(1)
        assert d2.max() <= np.sort(all_d2)[4] + 1e-15
    ip, ix = graphs.chung_lu(3000, 30_000, 2.1, 7)
    deg = np.diff(ip)
    assert deg.min() >= 1 and deg.max() > 20 * np.median(deg) / 2
    ip2, ix2 = graphs.chung_lu(3000, 30_000, 2.1, 7)
    np.testing.assert_array_equal(ix, ix2)


def test_blocked_edge_list_is_a_partition_by_column_block():
    rng = np.random.default_rng(8)
    indptr, indices = random_graph(rng, 50, 400, self_loops=True, duplicates=True)
    nblk, bptr, bcol = op.blocked_edges(indptr, indices, 16)
    assert nblk == 4 and bptr[0] == 0 and bptr[-1] == len(indices)
    n = 50
    for b in range(nblk):
        for r in (0, 7, 49):
            seg = bcol[bptr[b * n + r]:bptr[b * n + r + 1]]
            assert ((seg // 16) == b).all()
            want = [c for c in indices[indptr[r]:indptr[r + 1]] if c // 16 == b]
            assert seg.tolist() == want          # original order kept inside a (block, row) cell
    # every edge appears exactly once
    assert sorted(bcol.tolist()) == sorted(indices.tolist())
