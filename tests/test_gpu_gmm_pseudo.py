"""GMM layer with general per-edge pseudo-coordinates and the projection that produces them:
HIP path against the fp64 oracle."""
import numpy as np
import pytest

from helpers import random_graph, tiny_graph
from oracle import gmm as om

pytestmark = pytest.mark.gpu


def synth(rng, indptr, indices, fin, fout, K, r):
    n, E = len(indptr) - 1, len(indices)
    return dict(n=n, fin=fin, fout=fout, k=K, r=r, indptr=indptr, indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                w_fc=(rng.standard_normal((fin, K * fout)) * 0.3).astype(np.float32),
                pseudo=rng.uniform(-1, 1, (E, r)).astype(np.float32),
                mu=(rng.standard_normal((K, r)) * 0.3).astype(np.float32),
                inv_sigma=(0.5 + rng.random((K, r))).astype(np.float32),
                gout=rng.standard_normal((n, fout)).astype(np.float32))


def transposed_order(indices):
    """CSR positions in the order of the transposed edge list: by source, then by CSR position."""
    return np.argsort(indices, kind="stable")


def run(c, want_gx=True, want_gpseudo=True, transposed=False):
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    n, fin, fout, K, r, E = c["n"], c["fin"], c["fout"], c["k"], c["r"], len(c["indices"])
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    x, w_fc, mu, isg = dev(c["x"]), dev(c["w_fc"]), dev(c["mu"]), dev(c["inv_sigma"])
    pseudo = dev(c["pseudo"]) if E else empty((1, r))
    hk, out = empty((n, K * fout)), empty((n, fout))
    pk.gnn_gmmp_fwd(g, fin, fout, K, r, x, w_fc, pseudo, mu, isg, hk, out)
    ws = workspace(pk.gnn_gmmp_workspace_bytes(g, fin, fout, K))
    ws.fill_(0xFF)
    gx = empty((n, fin)) if want_gx else None
    gps = empty((max(E, 1), r)) if want_gpseudo else None
    gw, gmu, gis = empty((fin, K * fout)), empty((K, r)), empty((K, r))
    pseudo_t = dev(c["pseudo"][transposed_order(c["indices"])]) if transposed and E else None
    pk.gnn_gmmp_bwd(g, fin, fout, K, r, x, w_fc, pseudo, mu, isg, hk, dev(c["gout"]), gx, gw, gmu, gis, gps, ws,
                    pseudo_t=pseudo_t)
    torch.cuda.synchronize()
    res = dict(hk=hk, out=out, gw_fc=gw, gmu=gmu, ginv_sigma=gis)
    if want_gx:
        res["gx"] = gx
    if want_gpseudo:
        res["gpseudo"] = gps[:E]
    g.close()
    return {k: v.cpu().numpy() for k, v in res.items()}


def check(c, **kw):
    from gpu_harness import assert_close
    args = (c["indptr"], c["indices"], c["x"], c["w_fc"], c["pseudo"], c["mu"], c["inv_sigma"])
    fwd = om.gmm_pseudo_forward(*args)
    bwd = om.gmm_pseudo_backward(*args, c["gout"], fwd)
    res = run(c, **kw)
    assert_close("hk", res["hk"], fwd["Hk"].reshape(c["n"], -1))
    assert_close("out", res["out"], fwd["out"])
    assert_close("gw_fc", res["gw_fc"], bwd["gw_fc"], reduce_scale=True)
    assert_close("gmu", res["gmu"], bwd["gmu"])
    assert_close("ginv_sigma", res["ginv_sigma"], bwd["ginv_sigma"])
    if "gx" in res:
        assert_close("gx", res["gx"], bwd["gx"])
    if "gpseudo" in res:
        assert_close("gpseudo", res["gpseudo"], bwd["gpseudo"].reshape(res["gpseudo"].shape))
    return res


@pytest.mark.parametrize("fin,fout,K,r", [(16, 16, 3, 2), (16, 16, 3, 3), (16, 16, 2, 1), (5, 4, 1, 4), (40, 64, 4, 3),
                                          (7, 256, 2, 2), (9, 100, 3, 1), (3, 24, 4, 4)])
def test_shapes(fin, fout, K, r):
    print(f"gmmp: {fin}->{fout} K={K} r={r}", flush=True)
    rng = np.random.default_rng(fin + fout + 10 * K + r)
    indptr, indices = random_graph(rng, 400, 5000, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout, K, r))


@pytest.mark.parametrize("fout,K,r", [(16, 2, 1), (16, 3, 3), (64, 4, 2)])
def test_coordinates_in_the_transposed_order_give_the_same_bits(fout, K, r):
    """pseudo_t only changes where the source side of backward reads its coordinates from."""
    from workloads import graphs
    print(f"gmmp: pseudo_t fout={fout} K={K} r={r}", flush=True)
    indptr, indices = graphs.chung_lu(3000, 60_000, 2.1, 17)
    c = synth(np.random.default_rng(fout + K), indptr, indices, 24, fout, K, r)
    a, b = check(c), check(c, transposed=True)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_single_edge_kernels_agree_with_the_chunked_ones():
    """Rows of up to 64 projected floats take the chunked kernels; force_simple_kernels selects the
    one-edge-at-a-time kernels that wider rows use.  Both against the oracle."""
    import paper_2110_09524_amd as pk
    from workloads import graphs
    indptr, indices = graphs.chung_lu(4000, 90_000, 2.1, 23)
    c = synth(np.random.default_rng(3), indptr, indices, 20, 16, 3, 2)
    check(c)
    pk.gnn_config_set("force_simple_kernels", 1)
    try:
        check(c)
    finally:
        pk.gnn_config_set("force_simple_kernels", 0)


def test_the_papers_settings_on_a_power_law_graph():
    """k = 3, r = 3 and k = 2, r = 1 with 16 hidden features (Sec. 7.2) on a graph with hub rows."""
    from workloads import graphs
    print("gmmp: paper settings", flush=True)
    n = 5000
    indptr, indices = graphs.chung_lu(n, 100_000, 2.1, 99)
    rng = np.random.default_rng(5)
    for K, r in ((3, 3), (2, 1)):
        check(synth(rng, indptr, indices, 32, 16, K, r))


def test_hub_empty_rows_no_edges_and_optional_outputs():
    print("gmmp: hub / empty / optional", flush=True)
    rng = np.random.default_rng(6)
    n = 500
    edges = [(u, 0) for u in range(n)] + [(0, v) for v in range(1, n, 2)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(20, n) for _ in range(int(v) % 3)]
    indptr, indices = tiny_graph(n, edges)
    assert (np.diff(indptr) == 0).any()
    c = synth(rng, indptr, indices, 12, 32, 3, 2)
    res = check(c)
    assert (res["out"][np.diff(indptr) == 0] == 0).all()
    check(c, want_gx=False, want_gpseudo=False)
    check(synth(rng, np.zeros(34, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16, 2, 2))


def test_degree_pair_coordinates_agree_with_the_dedicated_layer():
    """pseudo = (c[u], c[v]) reproduces gnn_gmm_fwd (same oracle, two kernels paths)."""
    from gpu_harness import assert_close, run_gmm
    from workloads import make
    c = dict(make("gmm_c5_mid"))
    dst = np.repeat(np.arange(c["n"]), np.diff(c["indptr"]))
    c2 = dict(c, r=2, pseudo=np.stack([c["c"][c["indices"]], c["c"][dst]], axis=1).astype(np.float32))
    a, b = run_gmm(c), run(c2)
    for k in ("out", "gmu", "ginv_sigma", "gw_fc"):      # (hk is not written by the dedicated layer here)
        assert_close(k, b[k], a[k].astype(np.float64), reduce_scale=k == "gw_fc")


def test_projection_forward_backward_and_bad_arguments():
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, empty, workspace
    from workloads import graphs
    print("gmmp: projection", flush=True)
    n = 3000
    indptr, indices = graphs.chung_lu(n, 40_000, 2.1, 7)
    rng = np.random.default_rng(8)
    E = len(indices)
    c = (1.0 / np.sqrt(np.maximum(np.diff(indptr), 1))).astype(np.float32)
    g = pk.Graph(dev(indptr), dev(indices))
    for r in (1, 2, 3):
        P, pb = rng.standard_normal((r, 2)).astype(np.float32), (0.2 * rng.standard_normal(r)).astype(np.float32)
        gps = rng.standard_normal((E, r)).astype(np.float32)
        pseudo, pseudo_t, gP, gpb = empty((E, r)), empty((E, r)), empty((r, 2)), empty((r,))
        pk.gnn_pseudo_proj_fwd(g, r, dev(c), dev(P), dev(pb), pseudo, pseudo_t=pseudo_t)
        pk.gnn_pseudo_proj_bwd(g, r, dev(c), pseudo, dev(gps), gP, gpb, workspace(pk.gnn_pseudo_proj_workspace_bytes(g)))
        torch.cuda.synchronize()
        assert_close("pseudo", pseudo.cpu().numpy(), om.pseudo_projection_forward(indptr, indices, c, P, pb))
        assert np.array_equal(pseudo_t.cpu().numpy(), pseudo.cpu().numpy()[transposed_order(indices)])
        rP, rpb = om.pseudo_projection_backward(indptr, indices, c, P, pb, gps)
        assert_close("gproj_w", gP.cpu().numpy(), rP)
        assert_close("gproj_b", gpb.cpu().numpy(), rpb)
    a = empty((4, 4))
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_gmmp_fwd(g, 4, 16, 5, 2, a, a, a, a, a, a, a)          # 5 kernels
    assert e.value.status == 4
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_pseudo_proj_fwd(g, 5, a, a, a, a)                        # 5 dimensions
    assert e.value.status == 4
    g.close()
