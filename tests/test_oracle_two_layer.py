"""Pins of the two-layer composition: finite differences of the whole loss, and a case that
reduces to a plain softmax regression."""
import numpy as np

from helpers import finite_difference, random_graph, tiny_graph
from oracle import apply_vertex as av
from oracle import two_layer as ot


def _case(seed=0, n=14, m=50, fin=5, h1=2, f1=3, c=4):
    rng = np.random.default_rng(seed)
    indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=True)
    x = rng.standard_normal((n, fin))
    p = dict(w1=rng.standard_normal((fin, h1 * f1)) * 0.5, al1=rng.standard_normal((h1, f1)) * 0.5,
             ar1=rng.standard_normal((h1, f1)) * 0.5, b1=rng.standard_normal(h1 * f1) * 0.1,
             w2=rng.standard_normal((h1 * f1, c)) * 0.5, al2=rng.standard_normal((1, c)) * 0.5,
             ar2=rng.standard_normal((1, c)) * 0.5, b2=rng.standard_normal(c) * 0.1)
    labels = rng.integers(0, c, n)
    labels[::5] = -1
    return indptr, indices, x, p, labels


def test_every_parameter_gradient_matches_finite_differences_of_the_loss():
    indptr, indices, x, p, labels = _case(1)
    slope = 0.2
    g = ot.gat2_backward(indptr, indices, x, p, labels, slope)
    rng = np.random.default_rng(0)
    for name in ("w1", "al1", "ar1", "b1", "w2", "al2", "ar2", "b2"):
        def loss_of(t, name=name):
            q = dict(p)
            q[name] = t
            return ot.gat2_forward(indptr, indices, x, q, labels, slope)["loss"]
        idx, fd = finite_difference(loss_of, p[name], h=1e-6, max_entries=8, rng=rng)
        np.testing.assert_allclose(g["g" + name].reshape(-1)[idx], fd, rtol=2e-5, atol=1e-9, err_msg=name)


def test_self_loops_only_reduce_to_a_two_layer_perceptron():
    # with a single self-loop per vertex the attention weight is 1 and a GAT layer is x -> x w
    n, fin, f1, c = 9, 4, 6, 4
    rng = np.random.default_rng(2)
    indptr, indices = tiny_graph(n, [(v, v) for v in range(n)])
    x = rng.standard_normal((n, fin))
    p = dict(w1=rng.standard_normal((fin, f1)), al1=rng.standard_normal((1, f1)), ar1=rng.standard_normal((1, f1)),
             b1=rng.standard_normal(f1), w2=rng.standard_normal((f1, c)), al2=rng.standard_normal((1, c)),
             ar2=rng.standard_normal((1, c)), b2=rng.standard_normal(c))
    labels = rng.integers(0, c, n)
    fwd = ot.gat2_forward(indptr, indices, x, p, labels, 0.2)
    pre = x @ p["w1"] + p["b1"]
    a1 = np.where(pre > 0, pre, np.expm1(pre))
    z = a1 @ p["w2"] + p["b2"]
    np.testing.assert_allclose(fwd["z"], z, rtol=1e-12, atol=1e-12)
    loss, gz = av.softmax_xent(z, labels)
    assert abs(fwd["loss"] - loss) < 1e-13
    g = ot.gat2_backward(indptr, indices, x, p, labels, 0.2, fwd)
    np.testing.assert_allclose(g["gw2"], a1.T @ gz, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["gb2"], gz.sum(axis=0), rtol=1e-10, atol=1e-12)
    ga1 = gz @ p["w2"].T
    gpre = ga1 * np.where(pre > 0, 1.0, np.exp(pre))
    np.testing.assert_allclose(g["gw1"], x.T @ gpre, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g["gb1"], gpre.sum(axis=0), rtol=1e-10, atol=1e-12)
    # the attention vectors cannot matter when every softmax has one term
    assert np.abs(g["gal1"]).max() < 1e-12 and np.abs(g["gar2"]).max() < 1e-12


def _params(kind, rng, fin, fout, K=2):
    s = 0.5
    if kind == "gat":
        return dict(w=rng.standard_normal((fin, fout)) * s, al=rng.standard_normal((1, fout)) * s,
                    ar=rng.standard_normal((1, fout)) * s)
    if kind == "edgeconv":
        return dict(theta=rng.standard_normal((fin, fout)) * s, phi=rng.standard_normal((fin, fout)) * s)
    if kind == "gmm":
        return dict(w_fc=rng.standard_normal((fin, K * fout)) * s, mu=rng.standard_normal((K, 2)) * 0.3,
                    inv_sigma=0.5 + rng.random((K, 2)))
    if kind == "monet":
        return dict(w_fc=rng.standard_normal((fin, K * fout)) * s, mu=rng.standard_normal((K, 3)) * 0.3,
                    inv_sigma=0.5 + rng.random((K, 3)), proj_w=rng.standard_normal((3, 2)),
                    proj_b=rng.standard_normal(3) * 0.2)
    return dict(w=rng.standard_normal((fin, fout)) * s)


import pytest


@pytest.mark.parametrize("kind", ["gat", "edgeconv", "gmm", "gcn", "monet"])
def test_generic_chain_matches_finite_differences_for_every_layer_type(kind):
    rng = np.random.default_rng(11)
    n, fin, hid, c = 12, 4, 5, 3
    indptr, indices = random_graph(rng, n, 40, self_loops=True, duplicates=False)
    x = rng.standard_normal((n, fin))
    consts = dict(slope=0.2, c=rng.uniform(0.3, 1.0, n), c_src=rng.uniform(0.3, 1.0, n),
                  c_dst=rng.uniform(0.3, 1.0, n))
    p1, p2 = _params(kind, rng, fin, hid), _params(kind, rng, hid, c)
    b1, b2 = rng.standard_normal(hid) * 0.1, rng.standard_normal(c) * 0.1
    labels = rng.integers(0, c, n)
    labels[::4] = -1
    g1, gb1, g2, gb2 = ot.two_layer_backward(kind, indptr, indices, x, p1, b1, p2, b2, consts, labels,
                                             act="leaky", act_slope=0.1)

    def loss(p1_=p1, b1_=b1, p2_=p2, b2_=b2):
        return ot.two_layer_forward(kind, indptr, indices, x, p1_, b1_, p2_, b2_, consts, labels,
                                    act="leaky", act_slope=0.1)["loss"]
    for name in p1:
        idx, fd = finite_difference(lambda t: loss(p1_={**p1, name: t}), p1[name], h=1e-6, max_entries=6, rng=rng)
        np.testing.assert_allclose(g1[name].reshape(-1)[idx], fd, rtol=5e-5, atol=1e-9, err_msg=f"layer 1 {name}")
        idx, fd = finite_difference(lambda t: loss(p2_={**p2, name: t}), p2[name], h=1e-6, max_entries=6, rng=rng)
        np.testing.assert_allclose(g2[name].reshape(-1)[idx], fd, rtol=5e-5, atol=1e-9, err_msg=f"layer 2 {name}")
    _, fd = finite_difference(lambda t: loss(b1_=t), b1)
    np.testing.assert_allclose(gb1, fd, rtol=5e-5, atol=1e-9)
    _, fd = finite_difference(lambda t: loss(b2_=t), b2)
    np.testing.assert_allclose(gb2, fd, rtol=5e-5, atol=1e-9)


def test_generic_gat_chain_equals_the_dedicated_one():
    indptr, indices, x, p, labels = _case(3, h1=1, f1=6)
    a = ot.gat2_backward(indptr, indices, x, p, labels, 0.2)
    g1, gb1, g2, gb2 = ot.two_layer_backward(
        "gat", indptr, indices, x, dict(w=p["w1"], al=p["al1"], ar=p["ar1"]), p["b1"],
        dict(w=p["w2"], al=p["al2"], ar=p["ar2"]), p["b2"], dict(slope=0.2), labels, act="elu")
    np.testing.assert_allclose(g1["w"], a["gw1"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g2["ar"], a["gar2"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(gb1, a["gb1"], rtol=1e-12, atol=1e-14)
