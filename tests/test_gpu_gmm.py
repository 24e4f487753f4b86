"""MoNet / GMMConv layer: HIP path against the fp64 oracle."""
import numpy as np
import pytest

from oracle import gmm as om
from helpers import random_graph, tiny_graph
from workloads import make

pytestmark = pytest.mark.gpu


def check(c, **kw):
    from gpu_harness import assert_close, run_gmm
    args = (c["indptr"], c["indices"], c["x"], c["w_fc"], c["c"], c["mu"], c["inv_sigma"])
    fwd = om.gmm_forward(*args)
    bwd = om.gmm_backward(*args, c["gout"], fwd)
    res = run_gmm(c, **kw)
    n = c["n"]
    aggregate_first = kw.get("fwd_workspace", True) and c["fin"] % 4 == 0 and c["fin"] <= 256 and \
        c["fin"] < c["k"] * c["fout"]
    if not aggregate_first:      # hk is only written when the layer projects before it aggregates
        assert_close("hk", res["hk"], fwd["Hk"].reshape(n, -1))
    assert_close("out", res["out"], fwd["out"])
    assert_close("gx", res["gx"], bwd["gx"])
    assert_close("gw_fc", res["gw_fc"], bwd["gw_fc"], reduce_scale=True)
    assert_close("gmu", res["gmu"], bwd["gmu"])
    assert_close("ginv_sigma", res["ginv_sigma"], bwd["ginv_sigma"])


def synth(rng, indptr, indices, fin, fout, K):
    n = len(indptr) - 1
    deg = np.diff(indptr)
    return dict(n=n, fin=fin, fout=fout, k=K, indptr=indptr, indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                w_fc=(rng.standard_normal((fin, K * fout)) * 0.3).astype(np.float32),
                c=(1.0 / np.sqrt(np.maximum(deg, 1))).astype(np.float32),
                mu=(rng.standard_normal((K, 2)) * 0.3).astype(np.float32),
                inv_sigma=(0.5 + rng.random((K, 2))).astype(np.float32),
                gout=rng.standard_normal((n, fout)).astype(np.float32))


@pytest.mark.parametrize("name", ["gmm_c5_mid", "gmm_c5"])
def test_workloads(name):
    print("gmm:", name, flush=True)
    check(make(name))


@pytest.mark.parametrize("fin,fout,K", [(6, 4, 8), (3, 16, 5), (5, 16, 1), (9, 16, 4), (64, 64, 3), (12, 32, 8), (7, 256, 5),
                                        (20, 24, 2)])
def test_shapes(fin, fout, K):
    print(f"gmm: shape {fin}->{fout} K={K}", flush=True)
    rng = np.random.default_rng(fin + fout + K)
    indptr, indices = random_graph(rng, 263, 2600, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout, K))


@pytest.mark.parametrize("fin,fout,K", [(64, 64, 3), (16, 16, 2), (8, 256, 4), (100, 64, 8), (4, 4, 2), (252, 100, 3)])
def test_aggregate_first_and_project_first_agree_with_the_oracle(fin, fout, K):
    """Input rows narrower than the K projected rows: the forward call aggregates x per kernel and
    projects afterwards when it has a workspace, and projects first without one; the backward
    call gathers x on the destination side.  Hub rows included (cooperative path)."""
    print(f"gmm: aggregate first {fin}->{fout} K={K}", flush=True)
    rng = np.random.default_rng(fin * 7 + fout + K)
    n = 500
    edges = [(u, 3) for u in range(n)] + [(int(rng.integers(0, n)), int(v)) for v in range(n) for _ in range(int(v) % 9)]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, fin, fout, K)
    check(c)
    check(c, fwd_workspace=False)


def test_graph_without_edges():
    print("gmm: no edges", flush=True)
    rng = np.random.default_rng(62)
    n = 41
    check(synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16, 3))


def test_empty_rows_and_hub():
    print("gmm: empty rows + hub", flush=True)
    rng = np.random.default_rng(3)
    n = 500
    edges = [(u, 0) for u in range(n)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(10, n) for _ in range(2)]
    indptr, indices = tiny_graph(n, edges)
    check(synth(rng, indptr, indices, 10, 32, 3))


# ---- edge-balanced mapping of forward and both backward halves (Sec. 5), profile-driven choice ----
@pytest.fixture
def edge_balanced():
    import paper_2110_09524_amd as pk
    pk.gnn_config_set("gmm_mapping", 1)
    yield
    pk.gnn_config_set("gmm_mapping", 2)


@pytest.mark.parametrize("name", ["gmm_c5_mid", "gmm_c5"])
def test_edge_balanced_workloads(edge_balanced, name):
    print("gmm: edge-balanced", name, flush=True)
    check(make(name))


@pytest.mark.parametrize("fin,fout,K", [(5, 16, 1), (9, 16, 4), (64, 64, 3), (6, 4, 2), (7, 256, 3), (20, 24, 2),
                                        (12, 32, 8)])   # K = 8 > 4: stays vertex-balanced
def test_edge_balanced_shapes(edge_balanced, fin, fout, K):
    print(f"gmm: edge-balanced shape {fin}->{fout} K={K}", flush=True)
    rng = np.random.default_rng(fin + fout + K + 1)
    indptr, indices = random_graph(rng, 263, 2601, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout, K))


def test_edge_balanced_empty_rows_and_a_row_spanning_many_runs(edge_balanced):
    print("gmm: edge-balanced hub + empty rows", flush=True)
    rng = np.random.default_rng(77)
    n = 400
    edges = [(u, 3) for u in range(n)]                       # row 3 spans 13 runs of 32
    edges += [(int(rng.integers(0, n)), 7) for _ in range(32 - (n % 32))]   # row 7 ends on a run boundary
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(30, n) for _ in range(int(v) % 4)]
    indptr, indices = tiny_graph(n, edges)
    assert (np.diff(indptr) == 0).any() and len(indices) % 32 != 0
    check(synth(rng, indptr, indices, 10, 32, 3))
    check(synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16, 3))


def test_tune_records_a_choice_and_results_stay_right():
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty
    print("gmm: tune", flush=True)
    c = make("gmm_c5_mid")
    n, fin, fout, K = c["n"], c["fin"], c["fout"], c["k"]
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    x, w_fc, cc, mu, isg = dev(c["x"]), dev(c["w_fc"]), dev(c["c"]), dev(c["mu"]), dev(c["inv_sigma"])
    hk, out = empty((n, K * fout)), empty((n, fout))
    pk.gnn_gmm_fwd(g, fin, fout, K, x, w_fc, cc, mu, isg, hk, out)
    ms = pk.gnn_gmm_tune(g, fout, K, hk, cc, mu, isg, out)
    assert len(ms) == 2 and all(t > 0 for t in ms)
    ref = om.gmm_forward(c["indptr"], c["indices"], c["x"], c["w_fc"], c["c"], c["mu"], c["inv_sigma"])["out"]
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-4, atol=1e-5)     # the tuner leaves the result
    pk.gnn_gmm_fwd(g, fin, fout, K, x, w_fc, cc, mu, isg, hk, out)                # the recorded mapping
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-4, atol=1e-5)
    with pytest.raises(pk.GnnError):
        pk.gnn_config_set("gmm_mapping", 5)
    g.close()


def test_backward_tune_records_a_choice_and_results_stay_right():
    """gnn_gmm_tune_bwd times both halves of backward in both mappings; whatever it records, a
    following backward call matches the oracle."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, empty, workspace
    print("gmm: tune backward", flush=True)
    c = make("gmm_c5_mid")
    n, fin, fout, K = c["n"], c["fin"], c["fout"], c["k"]
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    x, w_fc, cc, mu, isg = dev(c["x"]), dev(c["w_fc"]), dev(c["c"]), dev(c["mu"]), dev(c["inv_sigma"])
    gout = dev(c["gout"])
    hk, out = empty((n, K * fout)), empty((n, fout))
    ws = workspace(pk.gnn_gmm_workspace_bytes(g, fin, fout, K))
    pk.gnn_gmm_fwd(g, fin, fout, K, x, w_fc, cc, mu, isg, hk, out)      # no workspace: projects first, writes hk
    ms = pk.gnn_gmm_tune_bwd(g, fin, fout, K, hk, cc, mu, isg, gout, ws)
    print("  ms: dst vertex/edge", ms[:2], "src vertex/edge", ms[2:], flush=True)
    assert len(ms) == 4 and all(t > 0 for t in ms)
    args = (c["indptr"], c["indices"], c["x"], c["w_fc"], c["c"], c["mu"], c["inv_sigma"])
    fwd = om.gmm_forward(*args)
    bwd = om.gmm_backward(*args, c["gout"], fwd)
    for mapping in (2, 1, 0):       # the recorded choice, edge-balanced forced, vertex-balanced forced
        pk.gnn_config_set("gmm_mapping", mapping)
        try:
            gx, gw_fc, gmu, gis = empty((n, fin)), empty((fin, K * fout)), empty((K, 2)), empty((K, 2))
            ws.fill_(0xFF)
            pk.gnn_gmm_bwd(g, fin, fout, K, x, w_fc, cc, mu, isg, hk, gout, gx, gw_fc, gmu, gis, ws)
            torch.cuda.synchronize()
        finally:
            pk.gnn_config_set("gmm_mapping", 2)
        assert_close(f"gx mapping={mapping}", gx.cpu().numpy(), bwd["gx"])
        assert_close(f"gw_fc mapping={mapping}", gw_fc.cpu().numpy(), bwd["gw_fc"], reduce_scale=True)
        assert_close(f"gmu mapping={mapping}", gmu.cpu().numpy(), bwd["gmu"])
        assert_close(f"ginv_sigma mapping={mapping}", gis.cpu().numpy(), bwd["ginv_sigma"])
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_gmm_tune_bwd(g, fin, fout, K, hk, cc, mu, isg, gout, workspace(256))
    assert e.value.status == 3
    g.close()


def test_edge_balanced_destination_side_is_bit_reproducible(edge_balanced):
    """The edge-balanced destination side of backward adds a row's pieces in a fixed order (no
    atomics): gmu and ginv_sigma repeat bit for bit."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    print("gmm: edge-balanced dst side twice", flush=True)
    c = make("gmm_c5_mid")
    n, fin, fout, K = c["n"], c["fin"], c["fout"], c["k"]
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    x, w_fc, cc, mu, isg = dev(c["x"]), dev(c["w_fc"]), dev(c["c"]), dev(c["mu"]), dev(c["inv_sigma"])
    hk, out = empty((n, K * fout)), empty((n, fout))
    ws = workspace(pk.gnn_gmm_workspace_bytes(g, fin, fout, K))
    pk.gnn_gmm_fwd(g, fin, fout, K, x, w_fc, cc, mu, isg, hk, out, ws)
    runs = []
    for _ in range(2):
        gw_fc, gmu, gis = empty((fin, K * fout)), empty((K, 2)), empty((K, 2))
        pk.gnn_gmm_bwd(g, fin, fout, K, x, w_fc, cc, mu, isg, hk, dev(c["gout"]), None, gw_fc, gmu, gis, ws)
        torch.cuda.synchronize()
        runs.append((gmu.cpu().numpy().copy(), gis.cpu().numpy().copy()))
    assert np.array_equal(runs[0][0], runs[1][0]) and np.array_equal(runs[0][1], runs[1][1])
    g.close()
