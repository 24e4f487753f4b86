"""MoNet layer with the projection of the degree pair fused into the gather kernels (gnn_monet_fwd/bwd):
HIP path against the fp64 oracle chain projection -> GMM layer -> projection's backward, and against the
two-call form of the library, which it must reproduce bit for bit wherever the summation order is the same."""
import numpy as np
import pytest

from helpers import random_graph, tiny_graph
from oracle import gmm as om

pytestmark = pytest.mark.gpu


def synth(rng, indptr, indices, fin, fout, K, r):
    n = len(indptr) - 1
    return dict(n=n, fin=fin, fout=fout, k=K, r=r, indptr=indptr, indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                w_fc=(rng.standard_normal((fin, K * fout)) * 0.3).astype(np.float32),
                c=(1.0 / np.sqrt(np.maximum(np.diff(indptr), 1))).astype(np.float32),
                proj_w=rng.standard_normal((r, 2)).astype(np.float32),
                proj_b=(0.2 * rng.standard_normal(r)).astype(np.float32),
                mu=(rng.standard_normal((K, r)) * 0.3).astype(np.float32),
                inv_sigma=(0.5 + rng.random((K, r))).astype(np.float32),
                gout=rng.standard_normal((n, fout)).astype(np.float32))


def run(c, fused=True, want_gx=True):
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    n, fin, fout, K, r, E = c["n"], c["fin"], c["fout"], c["k"], c["r"], len(c["indices"])
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    x, w_fc, mu, isg, cc = dev(c["x"]), dev(c["w_fc"]), dev(c["mu"]), dev(c["inv_sigma"]), dev(c["c"])
    P, pb, gout = dev(c["proj_w"]), dev(c["proj_b"]), dev(c["gout"])
    hk, out = empty((n, K * fout)), empty((n, fout))
    gx = empty((n, fin)) if want_gx else None
    gw, gmu, gis, gP, gpb = empty((fin, K * fout)), empty((K, r)), empty((K, r)), empty((r, 2)), empty((r,))
    ws = workspace(max(pk.gnn_monet_workspace_bytes(g, fin, fout, K), pk.gnn_pseudo_proj_workspace_bytes(g)))
    ws.fill_(0xFF)
    if fused:
        pk.gnn_monet_fwd(g, fin, fout, K, r, x, w_fc, cc, P, pb, mu, isg, hk, out)
        pk.gnn_monet_bwd(g, fin, fout, K, r, x, w_fc, cc, P, pb, mu, isg, hk, gout, gx, gw, gmu, gis, gP, gpb, ws)
    else:
        pseudo, gps = empty((max(E, 1), r)), empty((max(E, 1), r))
        pk.gnn_pseudo_proj_fwd(g, r, cc, P, pb, pseudo)
        pk.gnn_gmmp_fwd(g, fin, fout, K, r, x, w_fc, pseudo, mu, isg, hk, out)
        pk.gnn_gmmp_bwd(g, fin, fout, K, r, x, w_fc, pseudo, mu, isg, hk, gout, gx, gw, gmu, gis, gps, ws)
        pk.gnn_pseudo_proj_bwd(g, r, cc, pseudo, gps, gP, gpb, ws)
    torch.cuda.synchronize()
    res = dict(hk=hk, out=out, gw_fc=gw, gmu=gmu, ginv_sigma=gis, gproj_w=gP, gproj_b=gpb)
    if want_gx:
        res["gx"] = gx
    g.close()
    return {k: v.cpu().numpy() for k, v in res.items()}


def oracle(c):
    ip, ix = c["indptr"], c["indices"]
    ps = om.pseudo_projection_forward(ip, ix, c["c"], c["proj_w"], c["proj_b"])
    args = (ip, ix, c["x"], c["w_fc"], ps, c["mu"], c["inv_sigma"])
    fwd = om.gmm_pseudo_forward(*args)
    bwd = om.gmm_pseudo_backward(*args, c["gout"], fwd)
    gP, gpb = om.pseudo_projection_backward(ip, ix, c["c"], c["proj_w"], c["proj_b"], bwd["gpseudo"])
    return fwd, bwd, gP, gpb


def check(c, **kw):
    from gpu_harness import assert_close
    fwd, bwd, gP, gpb = oracle(c)
    res = run(c, **kw)
    assert_close("hk", res["hk"], fwd["Hk"].reshape(c["n"], -1))
    assert_close("out", res["out"], fwd["out"])
    assert_close("gw_fc", res["gw_fc"], bwd["gw_fc"], reduce_scale=True)
    assert_close("gmu", res["gmu"], bwd["gmu"])
    assert_close("ginv_sigma", res["ginv_sigma"], bwd["ginv_sigma"])
    assert_close("gproj_w", res["gproj_w"], gP)
    assert_close("gproj_b", res["gproj_b"], gpb)
    if "gx" in res:
        assert_close("gx", res["gx"], bwd["gx"])
    return res


@pytest.mark.parametrize("fin,fout,K,r", [(16, 16, 2, 1), (16, 16, 3, 3), (9, 8, 4, 2), (5, 4, 1, 4), (12, 16, 4, 4),
                                          (7, 64, 1, 2), (6, 12, 3, 1)])
def test_shapes(fin, fout, K, r):
    print(f"monet: {fin}->{fout} K={K} r={r}", flush=True)
    rng = np.random.default_rng(100 + fin + fout + 10 * K + r)
    indptr, indices = random_graph(rng, 400, 5000, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout, K, r))


def test_the_papers_settings_on_a_power_law_graph_and_the_two_call_form():
    """k = 3, r = 3 and k = 2, r = 1 with 16 hidden features (Sec. 7.2, 7.3) on a graph with hub rows.  The
    fused kernels evaluate the same expressions in the same order as projection + general layer, so
    everything but the projection's own gradient (summed in another order there) is bit-equal."""
    from gpu_harness import assert_close
    from workloads import graphs
    print("monet: paper settings", flush=True)
    indptr, indices = graphs.chung_lu(5000, 100_000, 2.1, 99)
    rng = np.random.default_rng(5)
    for K, r in ((3, 3), (2, 1)):
        c = synth(rng, indptr, indices, 32, 16, K, r)
        a = check(c)
        b = run(c, fused=False)
        for k in ("hk", "out", "gx", "gw_fc", "gmu", "ginv_sigma"):
            assert np.array_equal(a[k], b[k]), k
        assert_close("gproj_w", a["gproj_w"], b["gproj_w"].astype(np.float64))
        assert_close("gproj_b", a["gproj_b"], b["gproj_b"].astype(np.float64))


def test_hub_empty_rows_no_edges_optional_gx_and_limits():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty
    print("monet: hub / empty / optional / limits", flush=True)
    rng = np.random.default_rng(6)
    n = 500
    edges = [(u, 0) for u in range(n)] + [(0, v) for v in range(1, n, 2)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(20, n) for _ in range(int(v) % 3)]
    indptr, indices = tiny_graph(n, edges)
    assert (np.diff(indptr) == 0).any()
    c = synth(rng, indptr, indices, 12, 16, 3, 2)
    res = check(c)
    assert (res["out"][np.diff(indptr) == 0] == 0).all()
    check(c, want_gx=False)
    res = check(synth(rng, np.zeros(34, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16, 2, 2))
    assert not res["gproj_w"].any() and not res["gmu"].any()
    g = pk.Graph(dev(indptr), dev(indices))
    a = empty((4, 4))
    with pytest.raises(pk.GnnError) as e:                 # 3 x 32 projected floats: the two-call form's range
        pk.gnn_monet_fwd(g, 4, 32, 3, 2, a, a, a, a, a, a, a, a, a)
    assert e.value.status == 4 and "64" in str(e.value)
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_monet_bwd(g, 4, 16, 2, 1, a, a, a, a, a, a, a, a, a, None, a, a, a, a, a, None)
    assert e.value.status == 3                           # no workspace
    assert pk.gnn_monet_workspace_bytes(g, 4, 16, 2) > 0
    g.close()
