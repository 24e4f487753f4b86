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


@pytest.fixture(scope="module")
def sample(c4):
    """Seeded destination sample S: 4096 rows, every row of the top in-degree bucket (the hubs),
    and the shortest row; cut into chunks of at most ~0.8 M in-edges, the most the oracle's
    materialised per-edge tensors should hold at a time."""
    ip = c4["indptr"]
    n = ip.shape[0] - 1
    deg = np.diff(ip).astype(np.int64)
    rng = np.random.default_rng(99)
    top = np.flatnonzero(deg >= 1 << int(np.log2(deg.max())))       # the plan's top degree bucket
    rows = np.unique(np.concatenate([rng.choice(n, size=4096, replace=False), top, [int(np.argmin(deg))]]))
    rows = rows[rng.permutation(rows.size)]                         # hubs spread over the chunks
    bounds = np.searchsorted(np.cumsum(deg[rows]), np.arange(1, 64) * 800_000)
    chunks = [ch for ch in np.split(rows, np.unique(bounds[bounds < rows.size])) if ch.size]
    return dict(rows=np.sort(rows), chunks=chunks, top=top, edges=int(deg[rows].sum()))


def test_gat_c4_sampled_rows_and_consistency(c4, sample, capsys):
    """The layer bench.py times, in the launch configuration it times.  Forward: every output row of
    the sample S against the oracle on S's in-edges.  Backward: the upstream gradient is zero outside
    S, so only S's in-edges carry gradient and the oracle on them yields the COMPLETE gw, ga_l, ga_r
    and gx (all |V| source rows, hub sources included), compared element by element."""
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, gat_kink_masks, run_gat
    from oracle import gat as og
    from oracle.segments import restrict_rows, segment_sum
    c = c4
    n, H, F, fin = c["n"], c["heads"], c["f"], c["fin"]
    HF = H * F
    ip, ix = c["indptr"], c["indices"]

    def say(msg):
        with capsys.disabled():
            print("full size gat: " + msg, flush=True)

    g = pk.Graph(dev(ip), dev(ix))
    assert g.blocked(0)[0] > 1                      # the column-blocked kernels are in use
    rows = sample["rows"]
    say(f"oracle on the {sample['edges']} in-edges of {rows.size} rows ({sample['top'].size} hubs), "
        f"{len(sample['chunks'])} chunks")
    Ht = c["x"].astype(np.float64) @ c["w"].astype(np.float64)
    ref = {k: np.zeros((n, w)) for k, w in (("out", HF), ("t", HF), ("m", H), ("d", H), ("sg", H))}
    grads = dict(gx=np.zeros((n, fin)), gw=np.zeros((fin, HF)), ga_l=np.zeros((H, F)), ga_r=np.zeros((H, F)))
    amb_vh = np.zeros((n, H), dtype=bool)
    keep = np.zeros(n, dtype=bool)                  # S minus the rows with an edge on the LeakyReLU kink
    gout = c["gout"]
    for i, ch in enumerate(sample["chunks"]):
        rip, rix, _ = restrict_rows(ip, ix, ch)
        fwd = og.gat_forward(rip, rix, c["x"], c["w"], c["a_l"], c["a_r"], c["slope"], Ht=Ht)
        ref["out"][ch], ref["m"][ch], ref["d"][ch] = fwd["out"][ch], fwd["mx"][ch], fwd["den"][ch]
        ag = fwd["M2"] * np.where(fwd["M0"] > 0, 1.0, c["slope"])
        ref["sg"][ch] = segment_sum(rip, ag)[ch]
        ref["t"][ch] = segment_sum(rip, ag[:, :, None] * fwd["Ht"][fwd["src"]]).reshape(n, HF)[ch]
        a_vh, _ = gat_kink_masks(rip, fwd)
        amb_vh |= a_vh
        # a row holding an edge whose raw score is within 1e-5 of 0 may take either slope in fp32
        # (and then moves the shared-parameter gradients): it gets no upstream gradient, on both sides
        ok = ch[~a_vh[ch].any(axis=1)]
        keep[ok] = True
        go = np.zeros_like(gout)
        go[ok] = gout[ok]
        bwd = og.gat_backward(rip, rix, c["x"], c["w"], c["a_l"], c["a_r"], c["slope"], go, fwd)
        for k in grads:
            grads[k] += bwd[k]
        del fwd, bwd
        say(f"chunk {i + 1}/{len(sample['chunks'])} done")
    say(f"{int((~keep[rows]).sum())} of {rows.size} sampled rows sit on the LeakyReLU kink")
    assert (~keep[rows]).sum() <= rows.size // 20

    say("GPU fwd+bwd, upstream gradient zero outside the sample")
    cm = dict(c)
    cm["gout"] = np.where(keep[:, None], gout, np.float32(0))
    res = run_gat(cm, graph=g)
    assert_close("z", res["z"][rows], Ht[rows])
    for k in ("out", "m", "d"):
        assert_close(k, res[k][rows], ref[k][rows])
    keep_vh = ~amb_vh[rows]
    assert_close("sg", np.where(keep_vh, res["sg"][rows], ref["sg"][rows]), ref["sg"][rows])
    assert_close("t", np.where(np.repeat(keep_vh, F, axis=1), res["t"][rows], ref["t"][rows]), ref["t"][rows])
    assert_close("gx", res["gx"], grads["gx"])      # every source row of the graph
    for k in ("gw", "ga_l", "ga_r"):
        assert_close(k, res[k], grads[k], reduce_scale=True)

    say("properties")
    # <gw, w> = <dz, z> = <gx, x>: both products contract the same dz
    gw_w = float((res["gw"].astype(np.float64) * c["w"]).sum())
    gx_x = float((res["gx"].astype(np.float64) * c["x"]).sum())
    assert abs(gw_w - gx_x) <= 1e-4 * max(abs(gw_w), abs(gx_x)) + 1e-3
    # softmax weights sum to one: out is a convex combination, so it is bounded by z
    assert (np.abs(res["out"]).max(axis=0) <= np.abs(res["z"]).max(axis=0) * (1 + 1e-5)).all()
    assert (res["d"] >= 1.0 - 1e-6).all()
    # the single-launch kernels and the stash-free backward are independent routes to the
    # same numbers (full upstream gradient here): every output must agree
    res = run_gat(c, graph=g)
    pk.gnn_config_set("force_simple_kernels", 1)
    try:
        res2 = run_gat(c, graph=g, stash=False)
    finally:
        pk.gnn_config_set("force_simple_kernels", 0)
    for k in ("out", "m", "d", "gw", "ga_l", "ga_r"):
        assert_close(k + " (two kernel paths)", res[k], res2[k],
                     reduce_scale=k in ("gw", "ga_l", "ga_r"))
    assert_close("gx (two kernel paths)", res["gx"], res2["gx"])
    # the launch-per-block kernels (one launch per column block, the dense blocks with the score table
    # in LDS) add the same terms in the same order as the persistent kernel: every output bit for bit
    say("launch-per-block kernels against the persistent launch")
    pk.gnn_config_set("resident_sums", 0)
    pk.gnn_config_set("merge_blocks", 0)
    try:
        g2 = pk.Graph(dev(ip), dev(ix))
        res3 = run_gat(c, graph=g2)
        g2.close()
    finally:
        pk.gnn_config_set("resident_sums", 1)
        pk.gnn_config_set("merge_blocks", 1)
    for k in ("out", "t", "sg", "m", "d", "gx", "gw", "ga_l", "ga_r"):
        assert np.array_equal(res[k], res3[k]), f"{k}: persistent and launch-per-block kernels differ at full size"
    # the optional fp16 copy of the gathered rows (outside the 1e-4 contract) on the persistent kernels,
    # all batches of rows: within the rounding of an fp16 operand of the fp32 results above
    say("fp16 gather storage on the persistent launch")
    pk.gnn_config_set("gather_precision", 1)
    try:
        res16 = run_gat(c, graph=g)
    finally:
        pk.gnn_config_set("gather_precision", 0)
    for k in ("out", "gx", "gw", "ga_l", "ga_r"):
        a, b = res16[k].astype(np.float64), res[k].astype(np.float64)
        scale = max(float(np.sqrt(np.mean(b * b))), 1e-30)
        # an entry is held to the larger of the tensor's rms and its own row's largest entry (hub rows of gx
        # are sums over ~10^4 edges, far above the rms)
        row = np.maximum(np.abs(b).max(axis=1, keepdims=True), scale)
        worst, rms = float((np.abs(a - b) / row).max()), float(np.sqrt(np.mean((a - b) ** 2)) / scale)
        say(f"  {k}: fp16 gather against fp32, worst {worst:.1e} of its row's scale, rms {rms:.1e} of the tensor's rms")
        assert worst < 1.5e-2 and rms < 2e-3, f"{k}: fp16 gather error worst {worst:.2e} rms {rms:.2e}"
    assert np.array_equal(res16["m"], res["m"]) and not np.array_equal(res16["out"], res["out"])
    g.close()


def test_gcn_on_the_c4_graph_sampled_rows_and_consistency(c4, sample, capsys):
    """The GCN layer on the same graph and feature widths (602 -> 256), in the launch configuration
    bench.py times for gcn_c4.  Forward: every row of the sample against the oracle.  Backward: with
    the upstream gradient zero outside the sample the oracle on the sample's in-edges yields the
    complete gw and gx (every source row), compared element by element."""
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, run_gcn
    from oracle import gcn as og
    from oracle.segments import restrict_rows
    c = dict(c4)
    n, fin = c["n"], c["fin"]
    ip, ix = c["indptr"], c["indices"]
    indeg = np.diff(ip).astype(np.float64)
    outdeg = np.bincount(ix, minlength=n).astype(np.float64)
    c.update(kind="gcn", fout=c["heads"] * c["f"],
             c_src=(1.0 / np.sqrt(np.maximum(outdeg, 1.0))).astype(np.float32),
             c_dst=(1.0 / np.sqrt(np.maximum(indeg, 1.0))).astype(np.float32))

    def say(msg):
        with capsys.disabled():
            print("full size gcn: " + msg, flush=True)

    g = pk.Graph(dev(ip), dev(ix))
    assert g.blocked(0)[0] > 1
    rows = sample["rows"]
    keep = np.zeros(n, dtype=bool)
    keep[rows] = True
    gout = np.where(keep[:, None], c["gout"], np.float32(0))
    say(f"oracle on the in-edges of {rows.size} rows, {len(sample['chunks'])} chunks")
    out_ref = np.zeros((n, c["fout"]))
    grads = dict(gx=np.zeros((n, fin)), gw=np.zeros((fin, c["fout"])))
    Z = None
    for i, ch in enumerate(sample["chunks"]):
        rip, rix, _ = restrict_rows(ip, ix, ch)
        fwd = og.gcn_forward(rip, rix, c["x"], c["w"], c["c_src"], c["c_dst"])
        out_ref[ch], Z = fwd["out"][ch], fwd["Z"]
        go = np.zeros_like(gout)
        go[ch] = gout[ch]
        bwd = og.gcn_backward(rip, rix, c["x"], c["w"], c["c_src"], c["c_dst"], go, fwd)
        for k in grads:
            grads[k] += bwd[k]
        del fwd, bwd
        say(f"chunk {i + 1}/{len(sample['chunks'])} done")
    say("GPU fwd+bwd, upstream gradient zero outside the sample")
    res = run_gcn(dict(c, gout=gout), graph=g)
    assert_close("zs", res["zs"], c["c_src"].astype(np.float64)[:, None] * Z)
    assert_close("out", res["out"][rows], out_ref[rows])
    assert_close("gx", res["gx"], grads["gx"])
    assert_close("gw", res["gw"], grads["gw"], reduce_scale=True)
    say("general static weight per edge, first two chunks of the sample")
    import torch
    from gpu_harness import empty, workspace
    rng = np.random.default_rng(5)
    ew = (rng.uniform(-1.0, 1.0, len(ix)) / np.repeat(np.sqrt(np.maximum(indeg, 1.0)), np.diff(ip))).astype(np.float32)
    sub = np.concatenate(sample["chunks"][:2])
    keep2 = np.zeros(n, dtype=bool)
    keep2[sub] = True
    gout2 = np.where(keep2[:, None], c["gout"], np.float32(0))
    handle = pk.EdgeWeights(g, dev(ew))
    dx, dw = dev(c["x"]), dev(c["w"])
    z_w, out_w = empty((n, c["fout"])), empty((n, c["fout"]))
    gx_w, gw_w_ = empty((n, fin)), empty((fin, c["fout"]))
    ws = workspace(pk.gnn_gcn_workspace_bytes(g, fin, c["fout"]))
    pk.gnn_gcn_edge_fwd(g, handle, fin, c["fout"], dx, dw, z_w, out_w)
    pk.gnn_gcn_edge_bwd(g, handle, fin, c["fout"], dx, dw, dev(gout2), gx_w, gw_w_, ws)
    torch.cuda.synchronize()
    handle.close()
    ref_out = np.zeros((n, c["fout"]))
    ref = dict(gx=np.zeros((n, fin)), gw=np.zeros((fin, c["fout"])))
    for ch in sample["chunks"][:2]:
        rip, rix, pos = restrict_rows(ip, ix, ch)
        fwd = og.gcn_edge_forward(rip, rix, c["x"], c["w"], ew[pos])
        ref_out[ch] = fwd["out"][ch]
        go = np.zeros_like(gout2)
        go[ch] = gout2[ch]
        bwd = og.gcn_edge_backward(rip, rix, c["x"], c["w"], ew[pos], go, fwd)
        for k in ref:
            ref[k] += bwd[k]
        del fwd, bwd
    assert_close("out (edge weights)", out_w.cpu().numpy()[sub], ref_out[sub])
    assert_close("gx (edge weights)", gx_w.cpu().numpy(), ref["gx"])
    assert_close("gw (edge weights)", gw_w_.cpu().numpy(), ref["gw"], reduce_scale=True)
    del z_w, out_w, gx_w, gw_w_, ws

    say("properties")
    res = run_gcn(c, graph=g)
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
    assert_close("gx (two kernel paths)", res["gx"], res2["gx"])
    g.close()


def test_monet_on_the_c4_graph_sampled_rows_and_consistency(c4, sample, capsys):
    """The general GMM layer with projected 1-D pseudo-coordinates (the ablation setting of Sec. 7.3:
    k = 2, r = 1, 16 features) on the Reddit-scale graph.  Forward: every row of the sample.  Backward:
    upstream gradient zero outside the sample, so the oracle on the sample's in-edges yields the
    complete gx, gw_fc, gmu, ginv_sigma, the projection's gradients and gpseudo of those edges."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, empty, workspace
    from oracle import gmm as om
    from oracle.segments import restrict_rows
    n, fin, fout, K, R = c4["n"], c4["fin"], 16, 2, 1
    ip, ix = c4["indptr"], c4["indices"]
    E = len(ix)

    def say(msg):
        with capsys.disabled():
            print("full size monet: " + msg, flush=True)

    rng = np.random.default_rng(11)
    indeg = np.diff(ip)
    cvec = (1.0 / np.sqrt(np.maximum(indeg, 1))).astype(np.float32)
    w_fc = (rng.standard_normal((fin, K * fout)) * np.sqrt(2.0 / (fin + K * fout))).astype(np.float32)
    P, pb = rng.standard_normal((R, 2)).astype(np.float32), (0.1 * rng.standard_normal(R)).astype(np.float32)
    mu, isg = (0.3 * rng.standard_normal((K, R))).astype(np.float32), np.ones((K, R), dtype=np.float32)
    rows = sample["rows"]
    keep = np.zeros(n, dtype=bool)
    keep[rows] = True
    gout = np.where(keep[:, None], rng.standard_normal((n, fout)).astype(np.float32), np.float32(0))
    g = pk.Graph(dev(ip), dev(ix))
    x, dw, dc, dmu, dis, dgo = dev(c4["x"]), dev(w_fc), dev(cvec), dev(mu), dev(isg), dev(gout)
    dP, dpb = dev(P), dev(pb)
    pseudo, gps = empty((E, R)), empty((E, R))
    hk, out = empty((n, K * fout)), empty((n, fout))
    gx, gw, gmu, gis = empty((n, fin)), empty((fin, K * fout)), empty((K, R)), empty((K, R))
    gP, gpb = empty((R, 2)), empty((R,))
    ws = workspace(max(pk.gnn_gmmp_workspace_bytes(g, fin, fout, K), pk.gnn_pseudo_proj_workspace_bytes(g)))
    say("GPU fwd+bwd, upstream gradient zero outside the sample")
    pseudo_t = empty((E, R))   # the launch configuration bench.py times: coordinates in both edge orders
    pk.gnn_pseudo_proj_fwd(g, R, dc, dP, dpb, pseudo, pseudo_t=pseudo_t)
    pk.gnn_gmmp_fwd(g, fin, fout, K, R, x, dw, pseudo, dmu, dis, hk, out)
    pk.gnn_gmmp_bwd(g, fin, fout, K, R, x, dw, pseudo, dmu, dis, hk, dgo, gx, gw, gmu, gis, gps, ws,
                    pseudo_t=pseudo_t)
    pk.gnn_pseudo_proj_bwd(g, R, dc, pseudo, gps, gP, gpb, ws)
    torch.cuda.synchronize()
    say(f"oracle on the {sample['edges']} in-edges of {rows.size} rows")
    rip, rix, pos = restrict_rows(ip, ix, rows)
    ps_ref = om.pseudo_projection_forward(rip, rix, cvec, P, pb)
    assert_close("pseudo", pseudo.cpu().numpy()[pos], ps_ref)
    fwd = om.gmm_pseudo_forward(rip, rix, c4["x"], w_fc, ps_ref, mu, isg)
    assert_close("hk", hk.cpu().numpy(), fwd["Hk"].reshape(n, K * fout))
    # unnormalised sums: a hub row adds ~10^4 terms of order 1 and its entries are of order 30, so an
    # fp32 sum carries rounding of the order of 1e-5 whatever the entry cancels to (row-scaled bound)
    assert_close("out", out.cpu().numpy()[rows], fwd["out"][rows], row_scale=True)
    bwd = om.gmm_pseudo_backward(rip, rix, c4["x"], w_fc, ps_ref, mu, isg, gout, fwd)
    gps_all = gps.cpu().numpy()
    assert_close("gpseudo", gps_all[pos], bwd["gpseudo"])
    rest = np.ones(E, dtype=bool)
    rest[pos] = False
    assert not gps_all[rest].any()                   # edges into rows without upstream gradient
    assert_close("gx", gx.cpu().numpy(), bwd["gx"])
    for k, t in (("gw_fc", gw), ("gmu", gmu), ("ginv_sigma", gis)):
        assert_close(k, t.cpu().numpy(), bwd[k], reduce_scale=k == "gw_fc")
    rP, rpb = om.pseudo_projection_backward(rip, rix, cvec, P, pb, bwd["gpseudo"])
    assert_close("gproj_w", gP.cpu().numpy(), rP)
    assert_close("gproj_b", gpb.cpu().numpy(), rpb)
    say("the fused calls (what bench.py times): no per-edge array")
    hk2, out2 = empty((n, K * fout)), empty((n, fout))
    gx2, gw2, gmu2, gis2 = empty((n, fin)), empty((fin, K * fout)), empty((K, R)), empty((K, R))
    gP2, gpb2 = empty((R, 2)), empty((R,))
    pk.gnn_monet_fwd(g, fin, fout, K, R, x, dw, dc, dP, dpb, dmu, dis, hk2, out2)
    pk.gnn_monet_bwd(g, fin, fout, K, R, x, dw, dc, dP, dpb, dmu, dis, hk2, dgo, gx2, gw2, gmu2, gis2, gP2, gpb2, ws)
    torch.cuda.synchronize()
    # same expressions in the same order as the two-call form above, which was checked against the oracle
    for k, t2, t in (("hk", hk2, hk), ("out", out2, out), ("gx", gx2, gx), ("gw_fc", gw2, gw), ("gmu", gmu2, gmu),
                     ("ginv_sigma", gis2, gis)):
        assert torch.equal(t2, t), k
    assert_close("gproj_w", gP2.cpu().numpy(), rP)      # summed in another order than gnn_pseudo_proj_bwd
    assert_close("gproj_b", gpb2.cpu().numpy(), rpb)
    say("bilinearity")
    a = float((gx.double() * x.double()).sum())
    b = float((gw.double() * dw.double()).sum())
    o = float((dgo.double() * out.double()).sum())
    assert abs(a - o) <= 1e-4 * abs(o) + 1e-2 and abs(b - o) <= 1e-4 * abs(o) + 1e-2, (a, b, o)
    g.close()
