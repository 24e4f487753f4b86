"""Vertex operators, loss, SGD and the two-layer GAT step: HIP path against the fp64 oracle."""
import numpy as np
import pytest

from oracle import apply_vertex as av
from oracle import two_layer as ot
from workloads import make

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("act", ["identity", "relu", "elu", "leaky"])
@pytest.mark.parametrize("n,f", [(1, 4), (77, 20), (1000, 64), (5000, 256), (300, 1024)])
def test_bias_act_forward_backward(act, n, f):
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, empty, workspace
    print(f"bias_act: {act} n={n} f={f}", flush=True)
    rng = np.random.default_rng(n * 7 + f)
    x = rng.standard_normal((n, f)).astype(np.float32)
    b = (0.3 * rng.standard_normal(f)).astype(np.float32)
    pre = x.astype(np.float64) + b.astype(np.float64)
    x[np.abs(pre) < 1e-3] += 0.01          # the kink is tested on its own below
    gout = rng.standard_normal((n, f)).astype(np.float32)
    y, gin, gb = empty((n, f)), empty((n, f)), empty((f,))
    pk.gnn_bias_act_fwd(n, f, act, 0.2, dev(x), dev(b), y)
    pk.gnn_bias_act_bwd(n, f, act, 0.2, y, dev(gout), gin, gb, workspace(pk.gnn_bias_act_workspace_bytes(n, f)))
    ref_y = av.bias_act_forward(x, b, act, 0.2)
    ref_gx, ref_gb = av.bias_act_backward(x, b, act, gout, 0.2)
    assert_close("y", y.cpu().numpy(), ref_y)
    assert_close("gin", gin.cpu().numpy(), ref_gx)
    assert_close("gbias", gb.cpu().numpy(), ref_gb)
    # without a bias, in place, no bias gradient
    y2 = dev(x)
    pk.gnn_bias_act_fwd(n, f, act, 0.2, y2, None, y2)
    assert_close("y in place", y2.cpu().numpy(), av.bias_act_forward(x, None, act, 0.2))
    g2 = dev(gout)
    pk.gnn_bias_act_bwd(n, f, act, 0.2, y2, g2, g2, None)
    assert_close("gin in place", g2.cpu().numpy(), av.bias_act_backward(x, None, act, gout, 0.2)[0])


def test_activation_kinks_follow_the_conventions():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty
    z, one = dev(np.zeros((1, 4), dtype=np.float32)), dev(np.ones((1, 4), dtype=np.float32))
    for act, want in (("relu", 0.0), ("leaky", 0.2), ("elu", 1.0), ("identity", 1.0)):
        y, g = empty((1, 4)), empty((1, 4))
        pk.gnn_bias_act_fwd(1, 4, act, 0.2, z, None, y)
        pk.gnn_bias_act_bwd(1, 4, act, 0.2, y, one, g, None)
        assert (g.cpu().numpy() == np.float32(want)).all(), act


@pytest.mark.parametrize("n,c", [(1, 2), (300, 4), (2000, 41), (70000, 7)])
def test_softmax_xent(n, c):
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev, empty, workspace
    print(f"xent: n={n} c={c}", flush=True)
    rng = np.random.default_rng(n + c)
    z = (4 * rng.standard_normal((n, c))).astype(np.float32)
    if n > 10:
        z[3] += 80.0           # large logits must not overflow
    labels = rng.integers(0, c, n).astype(np.int32)
    labels[rng.random(n) < 0.3] = -1
    if n > 10:
        labels[5] = c          # out of range counts as unlabelled
    ref_labels = np.where(labels >= c, -1, labels)
    L = int((ref_labels >= 0).sum())
    loss, g = empty((1,)), empty((n, c))
    pk.gnn_softmax_xent(n, c, L, dev(z), dev(labels), loss, g, workspace(pk.gnn_softmax_xent_workspace_bytes(n)))
    ref_loss, ref_g = av.softmax_xent(z, ref_labels)
    assert abs(float(loss.cpu()[0]) - ref_loss) <= 1e-5 + 1e-4 * abs(ref_loss)
    got = g.cpu().numpy()
    assert np.abs(got - ref_g).max() <= 1e-5 / max(L, 1) + 1e-4 * np.abs(ref_g).max()
    assert (got[ref_labels < 0] == 0).all()


def test_sgd_update():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    rng = np.random.default_rng(3)
    p, g = rng.standard_normal(1001).astype(np.float32), rng.standard_normal(1001).astype(np.float32)
    dp = dev(p)
    pk.gnn_sgd_update(0.05, dev(g), dp)
    np.testing.assert_allclose(dp.cpu().numpy(), p.astype(np.float64) - 0.05 * g.astype(np.float64), rtol=1e-6, atol=1e-7)


def test_bad_arguments_raise():
    import paper_2110_09524_amd as pk
    from gpu_harness import empty, workspace
    a = empty((10, 6))
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_bias_act_fwd(10, 6, "relu", 0.0, a, None, a)          # f % 4 != 0
    assert e.value.status == 4
    b = empty((10, 8))
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_bias_act_bwd(10, 8, "relu", 0.0, b, b, b, empty((8,)), None)   # bias gradient without workspace
    assert e.value.status == 3
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_bias_act_fwd(10, 8, "leaky", -0.5, b, None, b)
    assert e.value.status == 1


def run_gat2(c, lr=None):
    import torch
    import paper_2110_09524_amd as pk
    from paper_2110_09524_amd.steps import Gat2Step
    from gpu_harness import dev
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    params = {k: dev(v) for k, v in c["params"].items()}
    step = Gat2Step(g, c["fin"], c["heads1"], c["f1"], c["classes"], c["slope"], params, dev(c["labels"]),
                    int((c["labels"] >= 0).sum()), need_gx=False)
    x = dev(c["x"])
    step.step(x, lr)
    torch.cuda.synchronize()
    res = dict(loss=float(step.loss.cpu()[0]), logits=step.logits.cpu().numpy(), a1=step.a1.cpu().numpy())
    res.update({"g" + k: v.cpu().numpy() for k, v in step.grads.items()})
    res.update({"new_" + k: v.cpu().numpy() for k, v in params.items()})
    g.close()
    return res


def test_two_layer_gat_step_matches_the_composed_oracle():
    from gpu_harness import assert_close
    print("gat2: gat2_mid", flush=True)
    c = make("gat2_mid")
    fwd = ot.gat2_forward(c["indptr"], c["indices"], c["x"], c["params"], c["labels"], c["slope"])
    bwd = ot.gat2_backward(c["indptr"], c["indices"], c["x"], c["params"], c["labels"], c["slope"], fwd)
    res = run_gat2(c, lr=0.1)
    assert_close("a1", res["a1"], fwd["a1"])
    assert_close("logits", res["logits"], fwd["z"])
    assert abs(res["loss"] - fwd["loss"]) <= 1e-5 + 1e-4 * abs(fwd["loss"])
    for k in ("w1", "al1", "ar1", "b1", "w2", "al2", "ar2", "b2"):
        assert_close("g" + k, res["g" + k], bwd["g" + k])
        want = c["params"][k].astype(np.float64) - 0.1 * bwd["g" + k]
        np.testing.assert_allclose(res["new_" + k], want, rtol=1e-4, atol=1e-5, err_msg="sgd " + k)


def _two_layer_case(kind, seed):
    """A seeded two-layer node classifier of the given layer type on a graph the oracle handles."""
    from helpers import random_graph
    from oracle import knn as ok
    rng = np.random.default_rng(seed)
    consts, extra = {}, {}
    if kind == "edgeconv":
        clouds, points, k = 3, 400, 12
        coords = rng.random((clouds * points, 3), dtype=np.float32)
        indptr, indices = ok.knn_graph(coords, clouds, points, k)
        n, fin, hid, c = clouds * points, 3, 32, 8
        x = coords                                  # the first layer works on the coordinates
        extra = dict(coords=coords, clouds=clouds, points=points, k=k)
    else:
        n, fin, hid, c = 1500, 24, 32, 8
        indptr, indices = random_graph(rng, n, 20000, self_loops=True, duplicates=False)
        x = rng.standard_normal((n, fin)).astype(np.float32)
    deg = np.maximum(np.diff(indptr), 1)
    f32 = lambda a: np.asarray(a, dtype=np.float32)

    def params(fi, fo):
        s = np.sqrt(2.0 / (fi + fo))
        if kind == "edgeconv":
            return dict(theta=f32(rng.standard_normal((fi, fo)) * s), phi=f32(rng.standard_normal((fi, fo)) * s))
        if kind == "gmm":
            return dict(w_fc=f32(rng.standard_normal((fi, 3 * fo)) * s), mu=f32(rng.standard_normal((3, 2)) * 0.3),
                        inv_sigma=f32(0.5 + rng.random((3, 2))))
        if kind == "monet":
            return dict(w_fc=f32(rng.standard_normal((fi, 3 * fo)) * s), mu=f32(rng.standard_normal((3, 3)) * 0.3),
                        inv_sigma=f32(0.5 + rng.random((3, 3))), proj_w=f32(rng.standard_normal((3, 2))),
                        proj_b=f32(0.2 * rng.standard_normal(3)))
        return dict(w=f32(rng.standard_normal((fi, fo)) * s))
    if kind in ("gmm", "monet"):
        consts["c"] = f32(1.0 / np.sqrt(deg))
    if kind == "gcn":
        consts["c_src"] = f32(1.0 / np.sqrt(np.maximum(np.bincount(indices, minlength=n), 1)))
        consts["c_dst"] = f32(1.0 / np.sqrt(deg))
    labels = rng.integers(0, c, n).astype(np.int32)
    labels[rng.random(n) < 0.4] = -1
    return dict(kind=kind, n=n, fin=fin, hid=hid, c=c, indptr=indptr, indices=indices, x=x, consts=consts,
                p1=params(fin, hid), p2=params(hid, c), b1=f32(0.1 * rng.standard_normal(hid)),
                b2=f32(0.1 * rng.standard_normal(c)), labels=labels, **extra)


@pytest.mark.parametrize("kind", ["edgeconv", "gmm", "gcn", "monet"])
def test_two_layer_step_of_every_layer_type(kind):
    """EdgeConv: the graph itself is built on the GPU from the coordinates (gnn_knn_graph)."""
    import torch
    import paper_2110_09524_amd as pk
    from paper_2110_09524_amd import steps
    from gpu_harness import assert_close, dev
    print(f"two-layer step: {kind}", flush=True)
    t = _two_layer_case(kind, 2024)
    n, fin, hid, c = t["n"], t["fin"], t["hid"], t["c"]
    act, slope = ("leaky", 0.2) if kind == "edgeconv" else ("relu", 0.0)
    fwd = ot.two_layer_forward(kind, t["indptr"], t["indices"], t["x"], t["p1"], t["b1"], t["p2"], t["b2"],
                               t["consts"], t["labels"], act, slope)
    g1, gb1, g2, gb2 = ot.two_layer_backward(kind, t["indptr"], t["indices"], t["x"], t["p1"], t["b1"], t["p2"],
                                             t["b2"], t["consts"], t["labels"], act, slope, fwd)
    if kind == "edgeconv":
        from oracle import edgeconv as oe
        for f, name in ((fwd["f1"], "layer 1"), (fwd["f2"], "layer 2")):     # the comparison needs a clear winner
            assert not oe.near_tie_mask(t["indptr"], f, 1e-6).any(), f"seed gives a near-tie in {name}"
        ip = torch.empty(n + 1, dtype=torch.int32, device="cuda:0")
        ix = torch.empty(n * t["k"], dtype=torch.int32, device="cuda:0")
        pk.gnn_knn_graph(t["clouds"], t["points"], 3, t["k"], dev(t["coords"]), ip, ix)
        assert (ix.cpu().numpy() == t["indices"]).all()
        g = pk.Graph(ip, ix)
    else:
        g = pk.Graph(dev(t["indptr"]), dev(t["indices"]))
    P1, P2 = {k: dev(v) for k, v in t["p1"].items()}, {k: dev(v) for k, v in t["p2"].items()}
    if kind == "edgeconv":
        l1, l2 = steps.EdgeConvLayer(g, fin, hid, P1), steps.EdgeConvLayer(g, hid, c, P2)
    elif kind == "gmm":
        cc = dev(t["consts"]["c"])
        l1, l2 = steps.GmmLayer(g, fin, hid, 3, P1, cc), steps.GmmLayer(g, hid, c, 3, P2, cc)
    elif kind == "monet":
        cc = dev(t["consts"]["c"])
        l1, l2 = steps.MonetLayer(g, fin, hid, 3, 3, P1, cc), steps.MonetLayer(g, hid, c, 3, 3, P2, cc)
    else:
        cs, cd = dev(t["consts"]["c_src"]), dev(t["consts"]["c_dst"])
        l1, l2 = steps.GcnLayer(g, fin, hid, P1, cs, cd), steps.GcnLayer(g, hid, c, P2, cs, cd)
    step = steps.TwoLayerStep(l1, l2, dev(t["b1"]), dev(t["b2"]), dev(t["labels"]), int((t["labels"] >= 0).sum()),
                              act=act, act_slope=slope)
    step.step(dev(t["x"]))
    torch.cuda.synchronize()
    assert_close("a1", step.a1.cpu().numpy(), fwd["a1"])
    assert_close("logits", step.logits.cpu().numpy(), fwd["z"])
    assert abs(float(step.loss.cpu()[0]) - fwd["loss"]) <= 1e-5 + 1e-4 * abs(fwd["loss"])
    for name in t["p1"]:
        assert_close(f"layer 1 g{name}", l1.grads[name].cpu().numpy(), g1[name])
        assert_close(f"layer 2 g{name}", l2.grads[name].cpu().numpy(), g2[name])
    assert_close("gb1", step.gb1.cpu().numpy(), gb1)
    assert_close("gb2", step.gb2.cpu().numpy(), gb2)
    g.close()
