"""Plan tables from the HIP library, bit-exact against the brute-force oracle."""
import numpy as np
import pytest
import torch

from oracle import plan as oplan
from helpers import random_graph, tiny_graph
from workloads import make

pytestmark = pytest.mark.gpu


def _check(indptr, indices):
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    g = pk.Graph(dev(indptr), dev(indices))
    ip_t, ix_t, eid_t = (t.cpu().numpy() for t in g.csc())
    r_ip, r_ix, r_eid = oplan.csc_transpose(indptr, indices)
    np.testing.assert_array_equal(ip_t, r_ip)
    np.testing.assert_array_equal(ix_t, r_ix)
    np.testing.assert_array_equal(eid_t, r_eid)
    for side, ptr in ((0, indptr), (1, r_ip)):
        b, o, off = (t.cpu().numpy() for t in g.buckets(side))
        rb, ro, roff = oplan.degree_buckets(ptr)
        np.testing.assert_array_equal(b, rb)
        np.testing.assert_array_equal(o, ro)
        np.testing.assert_array_equal(off, roff)
    g.close()


def test_tiny_graph_with_duplicates_and_empty_rows():
    print("plan: tiny", flush=True)
    _check(*tiny_graph(6, [(1, 0), (1, 0), (3, 0), (1, 2), (0, 2), (1, 2), (5, 5)]))


def test_single_vertex_and_no_edges():
    print("plan: degenerate", flush=True)
    _check(np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32))
    _check(np.zeros(5, dtype=np.int32), np.zeros(0, dtype=np.int32))


def test_random_multigraph():
    print("plan: random multigraph", flush=True)
    rng = np.random.default_rng(2)
    _check(*random_graph(rng, 300, 5000, self_loops=False, duplicates=True))


@pytest.mark.parametrize("name", ["gat_c1", "gat_c2", "ec_c3_mid"])
def test_workload_graphs(name):
    print("plan:", name, flush=True)
    c = make(name)
    _check(c["indptr"], c["indices"])


def test_malformed_graphs_are_rejected():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    print("plan: malformed", flush=True)
    good_ptr = np.array([0, 2, 3], dtype=np.int32)
    with pytest.raises(pk.GnnError) as e:
        pk.Graph(dev(good_ptr), dev(np.array([0, 1, 2], dtype=np.int32)))       # source id 2 >= n
    assert e.value.status == 2
    with pytest.raises(pk.GnnError) as e:
        pk.Graph(dev(np.array([0, 3, 2], dtype=np.int32)), dev(np.array([0, 1], dtype=np.int32)))
    assert e.value.status == 2
    with pytest.raises(pk.GnnError) as e:
        pk.Graph(dev(np.array([1, 2, 3], dtype=np.int32)), dev(np.array([0, 1, 1], dtype=np.int32)))
    assert e.value.status == 2
    with pytest.raises(pk.GnnError) as e:
        pk.Graph(dev(good_ptr), dev(np.array([0, -1, 1], dtype=np.int32)))
    assert e.value.status == 2


@pytest.mark.parametrize("block_cols", [16, 100])
def test_blocked_edge_lists(block_cols):
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    print("plan: blocked lists, block_cols =", block_cols, flush=True)
    rng = np.random.default_rng(4)
    indptr, indices = random_graph(rng, 333, 4000, self_loops=True, duplicates=True)
    pk.gnn_config_set("block_cols", block_cols)
    try:
        g = pk.Graph(dev(indptr), dev(indices))
    finally:
        pk.gnn_config_set("block_cols", 12288)
    ip_t, ix_t, _ = (t.cpu().numpy() for t in g.csc())
    for side, ptr, cols in ((0, indptr, indices), (1, ip_t, ix_t)):
        nb, bc, bptr, bcol = g.blocked(side)
        r_nb, r_bptr, r_bcol = oplan.blocked_edges(ptr, cols, block_cols)
        assert nb == r_nb and bc == block_cols
        np.testing.assert_array_equal(bptr.cpu().numpy(), r_bptr)
        np.testing.assert_array_equal(bcol.cpu().numpy(), r_bcol)
    g.close()
    g = pk.Graph(dev(indptr), dev(indices))          # default block size: one block, no tables
    assert g.blocked(0)[0] == 1
    g.close()


def test_no_blocked_lists_for_graphs_too_sparse_to_use_them():
    """With fewer than "blocked_min_edges" edges per (row, block) the column-blocked kernels are never
    chosen, so gnn_graph_create does not build their lists (most of the launches of a small plan);
    the rest of the plan is the same and the layers run on the single-launch kernels."""
    import paper_2110_09524_amd as pk
    import test_gpu_gat as TG
    from gpu_harness import dev, run_gat
    rng = np.random.default_rng(41)
    indptr, indices = random_graph(rng, 400, 4000, self_loops=True, duplicates=False)   # 11 edges per row
    pk.gnn_config_set("block_cols", 100)                                                # 4 blocks: 2.7 per (row, block)
    try:
        dense_enough = pk.Graph(dev(indptr), dev(indices))      # the suite runs with blocked_min_edges = 0
        pk.gnn_config_set("blocked_min_edges", 16)
        try:
            sparse = pk.Graph(dev(indptr), dev(indices))
        finally:
            pk.gnn_config_set("blocked_min_edges", 0)
    finally:
        pk.gnn_config_set("block_cols", 12288)
    assert dense_enough.blocked(0)[0] == 4 and dense_enough.blocked(1)[0] == 4
    assert sparse.blocked(0)[0] == 1 and sparse.blocked(1)[0] == 1
    for a, b in zip(dense_enough.csc(), sparse.csc()):
        assert bool((a == b).all())
    for side in (0, 1):
        for a, b in zip(dense_enough.buckets(side), sparse.buckets(side)):
            assert bool((a == b).all())
    c = TG.synth(rng, indptr, indices, 12, 2, 16)
    fwd, bwd = TG.oracle_all(c)
    TG.compare(c, run_gat(c, graph=sparse), fwd, bwd)
    dense_enough.close()
    sparse.close()


def _group_cost(begin, n, block_cols, groups, fixed):
    """Modelled cost of a partition of the block sequence into launches (units: one gathered edge per
    row): per launch a fixed part plus its edges per row, dearer by 32 % per doubling of the gathered
    columns beyond 24576."""
    cost = 0.0
    for a, b in zip(groups[:-1], groups[1:]):
        d = (begin[b] - begin[a]) / n
        over = max(0.0, np.log2((b - a) * block_cols / 24576.0))
        cost += fixed + d * (1.0 + 0.32 * over)
    return cost


def _all_partitions(nb, max_width):
    def rec(start):
        if start == nb:
            yield [nb]
            return
        for w in range(1, min(max_width, nb - start) + 1):
            for rest in rec(start + w):
                yield [start] + rest
    return rec(0)


def test_launch_groups_merge_the_sparse_tail_and_keep_dense_blocks_alone():
    """A graph whose first column block holds 150 edges per row and whose other two hold one each:
    the launches of a column-blocked kernel are the dense block alone and the tail merged.  On a
    small graph with ten narrow blocks the library's choice is the cheapest of all partitions under
    the cost model it documents; without merging every block has its own launch."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    print("plan: launch groups", flush=True)
    rng = np.random.default_rng(12)
    n, bc = 60000, 20480
    cols = np.concatenate([rng.integers(0, bc, size=(n, 150)), rng.integers(bc, 2 * bc, size=(n, 1)),
                           rng.integers(2 * bc, n, size=(n, 1))], axis=1)
    indices = np.sort(cols, axis=1).astype(np.int32).ravel()
    indptr = (np.arange(n + 1, dtype=np.int64) * cols.shape[1]).astype(np.int32)
    pk.gnn_config_set("block_cols", bc)
    try:
        g = pk.Graph(dev(indptr), dev(indices))
    finally:
        pk.gnn_config_set("block_cols", 12288)
    assert g.blocked(0)[:2] == (3, bc)
    assert g.launch_groups(0, 1) == [0, 1, 3] == g.launch_groups(0, 2)
    g.close()

    n, bc = 3000, 300
    cols = np.concatenate([rng.integers(0, bc, size=(n, 40))] +
                          [rng.integers(b * bc, (b + 1) * bc, size=(n, int(k))) for b, k in
                           zip(range(1, n // bc), rng.integers(0, 12, size=n // bc))], axis=1)
    indices = np.sort(cols, axis=1).astype(np.int32).ravel()
    indptr = (np.arange(n + 1, dtype=np.int64) * cols.shape[1]).astype(np.int32)
    pk.gnn_config_set("block_cols", bc)
    try:
        g = pk.Graph(dev(indptr), dev(indices))
        pk.gnn_config_set("merge_blocks", 0)
        g_plain = pk.Graph(dev(indptr), dev(indices))
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("merge_blocks", 1)
    nb = g.blocked(0)[0]
    assert nb == 10
    assert g_plain.launch_groups(0, 1) == list(range(nb + 1)) == g_plain.launch_groups(1, 2)
    begin = np.zeros(nb + 1, dtype=np.int64)
    np.add.at(begin, indices // bc + 1, 1)
    begin = np.cumsum(begin)
    for sums, fixed in ((1, 6.0), (2, 10.0)):
        groups = g.launch_groups(0, sums)
        assert groups[0] == 0 and groups[-1] == nb and all(0 < b - a <= 8 for a, b in zip(groups[:-1], groups[1:]))
        assert len(groups) < nb + 1, groups
        best = min(_group_cost(begin, n, bc, p, fixed) for p in _all_partitions(nb, 8))
        assert abs(_group_cost(begin, n, bc, groups, fixed) - best) <= 1e-9 * best, groups
    g.close()
    g_plain.close()
    g = pk.Graph(dev(indptr), dev(indices))          # one block: no groups
    assert g.launch_groups(0, 1) == []
    for side, sums in ((2, 1), (0, 3), (0, 0)):
        with pytest.raises(pk.GnnError) as e:
            g.launch_groups(side, sums)
        assert e.value.status == 1
    g.close()


def test_plans_reuse_cached_memory_and_release_it():
    """Rebuilding a plan of the same size takes its tables from the library's free list (no new device
    memory), and gnn_release_cached_memory hands the idle blocks back to the driver."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    from workloads import make
    c = make("ec_c3_mid")
    ip, ix = dev(c["indptr"]), dev(c["indices"])
    g = pk.Graph(ip, ix)
    csc = g.csc()                                   # also warms torch's own allocator
    g.close()                                       # fills the library's free list
    del csc
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for _ in range(5):
        g = pk.Graph(ip, ix)
        csc = g.csc()
        g.close()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free0    # nothing new was taken from the driver
    pk.gnn_release_cached_memory()
    assert torch.cuda.mem_get_info()[0] > free0     # and the idle blocks went back
    g = pk.Graph(ip, ix)                            # still works afterwards, same tables
    again = g.csc()
    for a, b in zip(csc, again):
        assert torch.equal(a, b)
    g.close()
