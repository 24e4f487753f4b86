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
        pk.gnn_config_set("block_cols", 24576)
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
