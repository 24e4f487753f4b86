"""GCN layer: HIP path (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest

from helpers import random_graph, tiny_graph
from oracle import gcn as og
from workloads import make

pytestmark = pytest.mark.gpu


def synth(rng, indptr, indices, fin, fout):
    n = len(indptr) - 1
    return dict(n=n, nnz=len(indices), fin=fin, fout=fout, indptr=indptr, indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                w=(rng.standard_normal((fin, fout)) * np.sqrt(2.0 / (fin + fout))).astype(np.float32),
                c_src=rng.uniform(0.2, 1.5, n).astype(np.float32),
                c_dst=rng.uniform(0.2, 1.5, n).astype(np.float32),
                gout=rng.standard_normal((n, fout)).astype(np.float32))


def check(c, **kw):
    from gpu_harness import assert_close, run_gcn
    fwd = og.gcn_forward(c["indptr"], c["indices"], c["x"], c["w"], c["c_src"], c["c_dst"])
    bwd = og.gcn_backward(c["indptr"], c["indices"], c["x"], c["w"], c["c_src"], c["c_dst"], c["gout"], fwd)
    res = run_gcn(c, **kw)
    assert_close("zs", res["zs"], c["c_src"].astype(np.float64)[:, None] * fwd["Z"])
    assert_close("out", res["out"], fwd["out"])
    assert_close("gw", res["gw"], bwd["gw"], reduce_scale=True)
    if "gx" in res:
        assert_close("gx", res["gx"], bwd["gx"])
    return res


def test_mid_workload():
    print("gcn: gcn_mid", flush=True)
    check(make("gcn_mid"))


@pytest.mark.parametrize("fin,fout", [(3, 4), (9, 20), (64, 64), (17, 128), (8, 512), (5, 1024)])
def test_shapes(fin, fout):
    print(f"gcn: shapes fin={fin} fout={fout}", flush=True)
    rng = np.random.default_rng(fin * 100 + fout)
    indptr, indices = random_graph(rng, 300, 3000, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout))


def test_empty_rows_hub_and_skipped_input_gradient():
    print("gcn: empty rows + hub", flush=True)
    rng = np.random.default_rng(8)
    n = 600
    edges = [(u, 0) for u in range(n)]                      # vertex 0 hears from everyone
    edges += [(0, v) for v in range(1, n, 3)]               # and speaks to many
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(20, n) for _ in range(int(v) % 3)]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, 12, 32)
    res = check(c)
    empty_rows = np.flatnonzero(np.diff(indptr) == 0)
    assert empty_rows.size > 0 and (res["out"][empty_rows] == 0).all()
    check(c, want_gx=False)


def test_graph_without_edges():
    print("gcn: no edges", flush=True)
    rng = np.random.default_rng(9)
    n = 33
    res = check(synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16))
    assert (res["out"] == 0).all() and (res["gw"] == 0).all() and (res["gx"] == 0).all()


@pytest.mark.parametrize("block_cols,fout", [(256, 256), (500, 128), (300, 512), (128, 1024), (256, 64), (300, 36), (200, 4)])
@pytest.mark.parametrize("merge", [0, 1, 2, 3])
def test_column_blocked_path(block_cols, fout, merge):
    """merge 0 / 1: one launch per block / merged launches; 2: all blocks in one persistent launch
    (running sums in LDS); 3: the same with the workgroups' bounded wait for each other cut to zero
    polls, which must not change any result."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    print(f"gcn: blocked path block_cols={block_cols} fout={fout} merge={merge}", flush=True)
    rng = np.random.default_rng(block_cols + fout)
    indptr, indices = random_graph(rng, 1500, 30000, self_loops=False, duplicates=True)
    c = synth(rng, indptr, indices, 24, fout)
    pk.gnn_config_set("block_cols", block_cols)
    pk.gnn_config_set("merge_blocks", int(merge == 1))
    pk.gnn_config_set("resident_sums", int(merge >= 2))
    pk.gnn_config_set("resident_spin", 0 if merge == 3 else 4096)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        nb = g.blocked(0)[0]
        assert nb == -(-c["n"] // block_cols)
        launches = len(g.launch_groups(0, 1)) - 1
        print(f"  {nb} blocks in {launches} launches", flush=True)
        assert launches == nb if merge != 1 else 1 <= launches <= nb
        check(c, graph=g)
        g.close()
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("merge_blocks", 1)
        pk.gnn_config_set("resident_sums", 1)
        pk.gnn_config_set("resident_spin", 4096)


def test_bad_arguments_raise():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    rng = np.random.default_rng(10)
    indptr, indices = random_graph(rng, 50, 200)
    c = synth(rng, indptr, indices, 8, 16)
    g = pk.Graph(dev(indptr), dev(indices))
    x, w, cs, cd = dev(c["x"]), dev(c["w"]), dev(c["c_src"]), dev(c["c_dst"])
    with pytest.raises(pk.GnnError) as e:          # fout not a multiple of 4
        pk.gnn_gcn_fwd(g, 8, 18, x, w, cs, cd, empty((50, 18)), empty((50, 18)))
    assert e.value.status == 4
    with pytest.raises(pk.GnnError) as e:          # workspace too small
        pk.gnn_gcn_bwd(g, 8, 16, x, w, cs, cd, dev(c["gout"]), None, empty((8, 16)),
                       workspace(pk.gnn_gcn_workspace_bytes(g, 8, 16) - 256))
    assert e.value.status == 3
    g.close()


def test_many_vertices_few_edges_on_the_blocked_path():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    print("gcn: 70000 vertices, sparse", flush=True)
    rng = np.random.default_rng(4243)
    n = 70_000
    src = rng.integers(0, n, size=150_000)
    dst = rng.integers(0, n // 2, size=150_000)
    order = np.lexsort((src, dst))
    src, dst = src[order], dst[order]
    indptr = np.zeros(n + 1, dtype=np.int32)
    np.add.at(indptr, dst + 1, 1)
    indptr = np.cumsum(indptr).astype(np.int32)
    c = synth(rng, indptr, src.astype(np.int32), 6, 128)
    g = pk.Graph(dev(indptr), dev(c["indices"]))
    assert g.blocked(0)[0] == -(-n // 12288)
    res = check(c, graph=g)
    assert (res["out"][n // 2:] == 0).all()
    g.close()


# ---- edge-balanced mapping (Sec. 5) and the profile-driven choice -------------------------
@pytest.fixture
def edge_balanced():
    import paper_2110_09524_amd as pk
    pk.gnn_config_set("gcn_mapping", 1)
    yield
    pk.gnn_config_set("gcn_mapping", 2)


def test_edge_balanced_mid_workload(edge_balanced):
    print("gcn: edge-balanced gcn_mid", flush=True)
    check(make("gcn_mid"))


@pytest.mark.parametrize("fin,fout", [(3, 4), (9, 20), (64, 64), (17, 128), (8, 512), (5, 1024)])
def test_edge_balanced_shapes(edge_balanced, fin, fout):
    print(f"gcn: edge-balanced shapes fin={fin} fout={fout}", flush=True)
    rng = np.random.default_rng(fin * 100 + fout + 1)
    indptr, indices = random_graph(rng, 300, 3000, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout))


def test_edge_balanced_empty_rows_hub_and_ragged_tail(edge_balanced):
    """Rows without edges between rows with edges, a row of 600 edges that spans ten runs, rows that
    start or end exactly on a run boundary, and an edge count that is not a multiple of the run."""
    print("gcn: edge-balanced empty rows + hub", flush=True)
    rng = np.random.default_rng(18)
    n = 600
    edges = [(u, 0) for u in range(n)]
    edges += [(int(rng.integers(0, n)), 5) for _ in range(64 - (n % 64))]      # row 5 ends on a boundary
    edges += [(int(rng.integers(0, n)), 9) for _ in range(64)]                   # row 9 is exactly one run
    edges += [(0, v) for v in range(12, n, 3)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(20, n) for _ in range(int(v) % 3)]
    indptr, indices = tiny_graph(n, edges)
    assert len(indices) % 64 != 0
    c = synth(rng, indptr, indices, 12, 32)
    res = check(c)
    empty_rows = np.flatnonzero(np.diff(indptr) == 0)
    assert empty_rows.size > 0 and (res["out"][empty_rows] == 0).all()


def test_edge_balanced_graph_without_edges(edge_balanced):
    rng = np.random.default_rng(19)
    n = 33
    res = check(synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16))
    assert (res["out"] == 0).all() and (res["gw"] == 0).all()


def test_tune_records_a_choice_and_results_stay_right():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, workspace
    print("gcn: tune", flush=True)
    c = make("gcn_mid")
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    ms = pk.gnn_gcn_tune(g, c["fout"], workspace(pk.gnn_gcn_workspace_bytes(g, 1, c["fout"])))
    assert len(ms) == 4 and all(t > 0 for t in ms)
    check(c, graph=g)        # whichever mapping was recorded per side
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_gcn_tune(g, c["fout"], workspace(256))
    assert e.value.status == 3
    with pytest.raises(pk.GnnError):
        pk.gnn_config_set("gcn_mapping", 3)
    g.close()


# ---- general static weight per edge --------------------------------------------------------------
def run_gcn_edge(c, want_gx=True):
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    n, fin, fout = c["n"], c["fin"], c["fout"]
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    ew = pk.EdgeWeights(g, dev(c["ew"]))
    x, w = dev(c["x"]), dev(c["w"])
    z, out = empty((n, fout)), empty((n, fout))
    pk.gnn_gcn_edge_fwd(g, ew, fin, fout, x, w, z, out)
    ws = workspace(pk.gnn_gcn_workspace_bytes(g, fin, fout))
    ws.fill_(0xFF)
    gx = empty((n, fin)) if want_gx else None
    gw = empty((fin, fout))
    pk.gnn_gcn_edge_bwd(g, ew, fin, fout, x, w, dev(c["gout"]), gx, gw, ws)
    torch.cuda.synchronize()
    res = dict(z=z.cpu().numpy(), out=out.cpu().numpy(), gw=gw.cpu().numpy())
    if want_gx:
        res["gx"] = gx.cpu().numpy()
    nblk = g.blocked(0)[0]
    ew.close()
    g.close()
    return res, nblk


def check_edge(c, **kw):
    from gpu_harness import assert_close
    fwd = og.gcn_edge_forward(c["indptr"], c["indices"], c["x"], c["w"], c["ew"])
    bwd = og.gcn_edge_backward(c["indptr"], c["indices"], c["x"], c["w"], c["ew"], c["gout"], fwd)
    res, nblk = run_gcn_edge(c, **kw)
    assert_close("z", res["z"], fwd["Z"])
    assert_close("out", res["out"], fwd["out"])
    assert_close("gw", res["gw"], bwd["gw"], reduce_scale=True)
    if "gx" in res:
        assert_close("gx", res["gx"], bwd["gx"])
    return res, nblk


@pytest.mark.parametrize("fin,fout", [(3, 4), (9, 20), (64, 64), (17, 128), (8, 512), (5, 1024)])
def test_edge_weighted_shapes(fin, fout):
    """A general static scalar per edge (both signs, duplicates weighted separately, empty rows,
    a hub): single-launch kernels, CSR side and CSC side."""
    print(f"gcn: per-edge weights fin={fin} fout={fout}", flush=True)
    rng = np.random.default_rng(fin * 100 + fout + 1)
    n = 400
    src = rng.integers(0, n, size=4000)
    dst = rng.integers(0, n, size=4000)
    edges = [(int(s), int(d)) for s, d in zip(src, dst) if d % 7 != 3]        # every 7th row empty
    edges += [(u, 0) for u in range(n)] + [(0, v) for v in range(1, n, 2) if v % 7 != 3]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, fin, fout)
    c["ew"] = rng.standard_normal(len(indices)).astype(np.float32)
    res, _ = check_edge(c)
    assert (res["out"][np.diff(indptr) == 0] == 0).all()
    check_edge(c, want_gx=False)


@pytest.mark.parametrize("block_cols,fout", [(256, 256), (1000, 128), (300, 512), (128, 1024), (256, 44)])
@pytest.mark.parametrize("resident", [0, 1])
def test_edge_weighted_column_blocked_path(block_cols, fout, resident):
    """The same on the column-blocked kernels: the weights travel in the order of the blocked edge
    lists (sorted once with the plan's keys), both sides, merged launches included; resident = 1:
    all blocks in one persistent launch."""
    import paper_2110_09524_amd as pk
    print(f"gcn: per-edge weights, blocked, block_cols={block_cols} fout={fout} resident={resident}", flush=True)
    rng = np.random.default_rng(block_cols + fout)
    indptr, indices = random_graph(rng, 1500, 30000, self_loops=False, duplicates=True)
    c = synth(rng, indptr, indices, 24, fout)
    c["ew"] = rng.uniform(-2.0, 2.0, len(indices)).astype(np.float32)
    pk.gnn_config_set("block_cols", block_cols)
    pk.gnn_config_set("resident_sums", resident)
    try:
        _, nblk = check_edge(c)
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("resident_sums", 1)
    assert nblk == -(-1500 // block_cols)


def test_edge_weighted_mid_workload_and_separable_case():
    """On the Reddit-shaped mid-size workload; with e_uv = c_src[u] c_dst[v] the general layer
    reproduces the separable one."""
    from gpu_harness import assert_close, run_gcn
    print("gcn: per-edge weights, gcn_mid", flush=True)
    c = dict(make("gcn_mid"))
    dst = np.repeat(np.arange(c["n"]), np.diff(c["indptr"]))
    c["ew"] = (c["c_src"][c["indices"]] * c["c_dst"][dst]).astype(np.float32)
    res, _ = check_edge(c)
    sep = run_gcn(c)
    assert_close("out vs separable", res["out"], sep["out"].astype(np.float64))
    assert_close("gx vs separable", res["gx"], sep["gx"].astype(np.float64))


def test_edge_weights_belong_to_their_graph():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty
    rng = np.random.default_rng(3)
    ip1, ix1 = random_graph(rng, 50, 200, self_loops=True)
    ip2, ix2 = random_graph(rng, 50, 210, self_loops=True)
    g1, g2 = pk.Graph(dev(ip1), dev(ix1)), pk.Graph(dev(ip2), dev(ix2))
    ew = pk.EdgeWeights(g1, dev(rng.standard_normal(len(ix1)).astype(np.float32)))
    a = empty((50, 8))
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_gcn_edge_fwd(g2, ew, 8, 8, a, a, a, a)
    assert e.value.status == 1
    ew.close()
    g1.close()
    g2.close()


@pytest.mark.parametrize("fin,fout", [(9, 20), (64, 64), (8, 512)])
def test_edge_weighted_edge_balanced_mapping(edge_balanced, fin, fout):
    """The general edge-weight layer in the edge-balanced mapping (runs of 64 edge positions, the
    weights read next to the indices): rows spanning several runs, empty rows, a ragged tail."""
    print(f"gcn: per-edge weights, edge-balanced fin={fin} fout={fout}", flush=True)
    rng = np.random.default_rng(fin * 31 + fout)
    n = 600
    edges = [(u, 0) for u in range(n)] + [(0, v) for v in range(12, n, 3)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(20, n) for _ in range(int(v) % 5)]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, fin, fout)
    c["ew"] = rng.uniform(-2.0, 2.0, len(indices)).astype(np.float32)
    res, _ = check_edge(c)
    assert (res["out"][np.diff(indptr) == 0] == 0).all()
