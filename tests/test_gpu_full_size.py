"""Full-size GAT workload (the one bench.py times, same launch configuration):
sampled outputs against the oracle, and properties that hold at any size."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c4():
    from workloads import make
    print("full size: generating gat_c4", flush=True)
    return make("gat_c4")


def test_gat_c4_plan_is_the_stable_transpose(c4):
    """At this size the oracle's sort of Python tuples is out of reach; the CSC transpose is
    instead pinned by the properties that define it uniquely: eid_t is a permutation of the
    CSR positions, grouped by source in ascending source order, ascending inside a source
    (stability), and indices_t / indptr_t follow from it."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    ip, ix = c4["indptr"], c4["indices"]
    n, nnz = ip.shape[0] - 1, ix.shape[0]
    print("full size: plan", flush=True)
    g = pk.Graph(dev(ip), dev(ix))
    indptr_t, indices_t, eid_t = (a.cpu().numpy() for a in g.csc())
    g.close()
    assert indptr_t[0] == 0 and indptr_t[-1] == nnz
    assert np.array_equal(np.diff(indptr_t), np.bincount(ix, minlength=n))
    seen = np.zeros(nnz, dtype=bool)
    seen[eid_t] = True
    assert seen.all()                                              # a permutation
    src_of_slot = np.repeat(np.arange(n, dtype=np.int32), np.diff(indptr_t))
    assert np.array_equal(ix[eid_t], src_of_slot)                  # grouped by source, sources ascending
    inner = np.ones(nnz, dtype=bool)
    inner[indptr_t[:-1][np.diff(indptr_t) > 0]] = False            # first slot of every non-empty row
    assert (np.diff(eid_t.astype(np.int64))[inner[1:]] > 0).all()  # CSR order kept inside a source
    dst_of = np.repeat(np.arange(n, dtype=np.int32), np.diff(ip))
    assert np.array_equal(indices_t, dst_of[eid_t])


def test_gat_c4_sampled_rows_and_consistency(c4):
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, gat_kink_masks, run_gat
    from oracle import gat as og
    from oracle.segments import restrict_rows, segment_sum
    c = c4
    n, H, F = c["n"], c["heads"], c["f"]
    HF = H * F
    ip, ix = c["indptr"], c["indices"]
    g = pk.Graph(dev(ip), dev(ix))
    assert g.blocked(0)[0] > 1                      # the column-blocked kernels are in use
    print("full size: GPU fwd+bwd", flush=True)
    res = run_gat(c, graph=g)

    deg = np.diff(ip)
    outdeg = np.bincount(ix, minlength=n)
    rng = np.random.default_rng(99)
    # destinations: the biggest hub, the smallest row, and a seeded sample
    dst_rows = np.unique(np.concatenate([[int(np.argmax(deg)), int(np.argmin(deg))],
                                         rng.choice(n, size=30, replace=False)]))
    # sources whose full backward neighbourhood the oracle can afford: small out-degree
    cand = np.flatnonzero(outdeg <= np.partition(outdeg, 2000)[2000])
    src_rows = rng.choice(cand, size=3, replace=False)
    # every destination that a sampled source points to, plus the sampled sources themselves
    dst_of = np.repeat(np.arange(n, dtype=np.int64), deg)
    hit = np.isin(ix, src_rows)
    rows = np.unique(np.concatenate([dst_rows, dst_of[hit], src_rows]))
    print(f"full size: oracle on the in-edges of {rows.size} rows", flush=True)
    rip, rix, _ = restrict_rows(ip, ix, rows)
    Ht = c["x"].astype(np.float64) @ c["w"].astype(np.float64)
    fwd = og.gat_forward(rip, rix, c["x"], c["w"], c["a_l"], c["a_r"], c["slope"], Ht=Ht)
    bwd = og.gat_backward(rip, rix, c["x"], c["w"], c["a_l"], c["a_r"], c["slope"], c["gout"], fwd)

    print("full size: comparing sampled rows", flush=True)
    assert_close("z", res["z"][rows], Ht[rows])
    assert_close("out", res["out"][rows], fwd["out"][rows])
    assert_close("m", res["m"][rows], fwd["mx"][rows])
    assert_close("d", res["d"][rows], fwd["den"][rows])
    ag = fwd["M2"] * np.where(fwd["M0"] > 0, 1.0, c["slope"])
    amb_vh, amb_vertex = gat_kink_masks(rip, fwd)
    print(f"full size: {int(amb_vh.sum())} (row, head) pairs sit on the LeakyReLU kink", flush=True)
    keep_vh = ~amb_vh[rows]
    sg_ref = segment_sum(rip, ag)[rows]
    assert_close("sg", np.where(keep_vh, res["sg"][rows], sg_ref), sg_ref)
    t_ref = segment_sum(rip, ag[:, :, None] * fwd["Ht"][fwd["src"]]).reshape(n, HF)[rows]
    assert_close("t", np.where(np.repeat(keep_vh, F, axis=1), res["t"][rows], t_ref), t_ref)
    src_rows = src_rows[~amb_vertex[src_rows]]
    assert src_rows.size >= 1
    # input gradient of the sampled sources: all their out-edges and those edges' whole
    # destination rows are inside the restricted graph, so the oracle's rows are complete
    assert_close("gx", res["gx"][src_rows], bwd["gx"][src_rows], row_scale=True)

    print("full size: properties", flush=True)
    # <gw, w> = <dz, z> = <gx, x>: both products contract the same dz
    gw_w = float((res["gw"].astype(np.float64) * c["w"]).sum())
    gx_x = float((res["gx"].astype(np.float64) * c["x"]).sum())
    assert abs(gw_w - gx_x) <= 1e-4 * max(abs(gw_w), abs(gx_x)) + 1e-3
    # softmax weights sum to one: out is a convex combination, so it is bounded by z
    assert (np.abs(res["out"]).max(axis=0) <= np.abs(res["z"]).max(axis=0) * (1 + 1e-5)).all()
    assert (res["d"] >= 1.0 - 1e-6).all()
    # the single-launch kernels and the stash-free backward are independent routes to the
    # same numbers: every output, including the |V|-long parameter reductions, must agree
    pk.gnn_config_set("force_simple_kernels", 1)
    try:
        res2 = run_gat(c, graph=g, stash=False)
    finally:
        pk.gnn_config_set("force_simple_kernels", 0)
    for k in ("out", "m", "d", "gw", "ga_l", "ga_r"):
        assert_close(k + " (two kernel paths)", res[k], res2[k],
                     reduce_scale=k in ("gw", "ga_l", "ga_r"))
    assert_close("gx (two kernel paths)", res["gx"], res2["gx"], row_scale=True)
    # the hub block's LDS-table variant adds the same terms in the same order as the plain one
    pk.gnn_config_set("lds_scalar_table", 0)
    try:
        res3 = run_gat(c, graph=g, backward=False)
    finally:
        pk.gnn_config_set("lds_scalar_table", 1)
    for k in ("out", "t", "sg", "m", "d"):
        assert np.array_equal(res[k], res3[k]), f"{k}: LDS-table and plain variants differ at full size"
    g.close()


def test_gcn_on_the_c4_graph_sampled_rows_and_consistency(c4):
    """The GCN layer on the same graph and feature widths (602 -> 256), in the launch
    configuration bench.py times for gcn_c4: sampled rows against the oracle, and
    properties that hold at any size."""
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, run_gcn
    from oracle import gcn as og
    from oracle.segments import restrict_rows
    c = dict(c4)
    n = c["n"]
    ip, ix = c["indptr"], c["indices"]
    indeg = np.diff(ip).astype(np.float64)
    outdeg = np.bincount(ix, minlength=n).astype(np.float64)
    c.update(kind="gcn", fout=c["heads"] * c["f"],
             c_src=(1.0 / np.sqrt(np.maximum(outdeg, 1.0))).astype(np.float32),
             c_dst=(1.0 / np.sqrt(np.maximum(indeg, 1.0))).astype(np.float32))
    g = pk.Graph(dev(ip), dev(ix))
    assert g.blocked(0)[0] > 1
    print("full size gcn: GPU fwd+bwd", flush=True)
    res = run_gcn(c, graph=g)

    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[int(np.argmax(indeg)), int(np.argmin(indeg))],
                                     rng.choice(n, size=40, replace=False)]))
    print(f"full size gcn: oracle on the in-edges of {rows.size} rows", flush=True)
    rip, rix, _ = restrict_rows(ip, ix, rows)
    fwd = og.gcn_forward(rip, rix, c["x"], c["w"], c["c_src"], c["c_dst"])
    assert_close("zs", res["zs"][rows], (c["c_src"].astype(np.float64)[:, None] * fwd["Z"])[rows])
    assert_close("out", res["out"][rows], fwd["out"][rows])
    # backward on sampled sources: their out-edges reach into many rows, so compare through the
    # transposed graph restricted to those sources: dZ[u] = c_src[u] sum_v c_dst[v] gout[v]
    srcs = rng.choice(np.flatnonzero(outdeg <= np.partition(outdeg, 2000)[2000]), size=5, replace=False)
    dst_of = np.repeat(np.arange(n, dtype=np.int64), np.diff(ip))
    W64 = c["w"].astype(np.float64)
    for u in srcs:
        vs = dst_of[ix == u]
        dz_u = c["c_src"][u].astype(np.float64) * (c["c_dst"][vs].astype(np.float64)[:, None]
                                                   * c["gout"][vs].astype(np.float64)).sum(axis=0)
        assert_close(f"gx[{u}]", res["gx"][u][None, :], (dz_u @ W64.T)[None, :], row_scale=True)
    print("full size gcn: properties", flush=True)
    gw_w = float((res["gw"].astype(np.float64) * c["w"]).sum())
    gx_x = float((res["gx"].astype(np.float64) * c["x"]).sum())
    assert abs(gw_w - gx_x) <= 1e-4 * max(abs(gw_w), abs(gx_x)) + 1e-3
    pk.gnn_config_set("force_simple_kernels", 1)
    try:
        res2 = run_gcn(c, graph=g)
    finally:
        pk.gnn_config_set("force_simple_kernels", 0)
    assert_close("out (two kernel paths)", res["out"], res2["out"])
    assert_close("gw (two kernel paths)", res["gw"], res2["gw"], reduce_scale=True)
    assert_close("gx (two kernel paths)", res["gx"], res2["gx"], row_scale=True)
    g.close()


def test_monet_on_the_c4_graph_sampled_rows_and_consistency(c4):
    """The general GMM layer with projected 1-D pseudo-coordinates (the ablation setting of Sec. 7.3:
    k = 2, r = 1, 16 features) on the Reddit-scale graph: sampled rows, hub row included, against the
    oracle, and the bilinearity identity <gx, x> = <gw_fc, w_fc> = <gout, out> over the whole graph."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, empty, workspace
    from oracle import gmm as om
    from oracle.segments import restrict_rows
    n, fin, fout, K, R = c4["n"], c4["fin"], 16, 2, 1
    ip, ix = c4["indptr"], c4["indices"]
    E = len(ix)
    rng = np.random.default_rng(11)
    indeg = np.diff(ip)
    cvec = (1.0 / np.sqrt(np.maximum(indeg, 1))).astype(np.float32)
    w_fc = (rng.standard_normal((fin, K * fout)) * np.sqrt(2.0 / (fin + K * fout))).astype(np.float32)
    P, pb = rng.standard_normal((R, 2)).astype(np.float32), (0.1 * rng.standard_normal(R)).astype(np.float32)
    mu, isg = (0.3 * rng.standard_normal((K, R))).astype(np.float32), np.ones((K, R), dtype=np.float32)
    gout = rng.standard_normal((n, fout)).astype(np.float32)
    g = pk.Graph(dev(ip), dev(ix))
    x, dw, dc, dmu, dis, dgo = dev(c4["x"]), dev(w_fc), dev(cvec), dev(mu), dev(isg), dev(gout)
    pseudo, gps = empty((E, R)), empty((E, R))
    hk, out = empty((n, K * fout)), empty((n, fout))
    gx, gw, gmu, gis = empty((n, fin)), empty((fin, K * fout)), empty((K, R)), empty((K, R))
    ws = workspace(max(pk.gnn_gmmp_workspace_bytes(g, fin, fout, K), pk.gnn_pseudo_proj_workspace_bytes(g)))
    print("full size monet: GPU fwd+bwd", flush=True)
    pk.gnn_pseudo_proj_fwd(g, R, dc, dev(P), dev(pb), pseudo)
    pk.gnn_gmmp_fwd(g, fin, fout, K, R, x, dw, pseudo, dmu, dis, hk, out)
    pk.gnn_gmmp_bwd(g, fin, fout, K, R, x, dw, pseudo, dmu, dis, hk, dgo, gx, gw, gmu, gis, gps, ws)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[int(np.argmax(indeg)), int(np.argmin(indeg))],
                                     rng.choice(n, size=60, replace=False)]))
    print(f"full size monet: oracle on the in-edges of {rows.size} rows", flush=True)
    rip, rix, pos = restrict_rows(ip, ix, rows)
    ps_ref = om.pseudo_projection_forward(rip, rix, cvec, P, pb)
    assert_close("pseudo", pseudo.cpu().numpy()[pos], ps_ref)
    fwd = om.gmm_pseudo_forward(rip, rix, c4["x"], w_fc, ps_ref, mu, isg)
    assert_close("out", out.cpu().numpy()[rows], fwd["out"][rows])
    bwd = om.gmm_pseudo_backward(rip, rix, c4["x"], w_fc, ps_ref, mu, isg, gout, fwd)
    assert_close("gpseudo", gps.cpu().numpy()[pos], bwd["gpseudo"])
    print("full size monet: bilinearity", flush=True)
    a = float((gx.double() * x.double()).sum())
    b = float((gw.double() * dw.double()).sum())
    o = float((dgo.double() * out.double()).sum())
    assert abs(a - o) <= 1e-4 * abs(o) + 1e-2 and abs(b - o) <= 1e-4 * abs(o) + 1e-2, (a, b, o)
    g.close()
