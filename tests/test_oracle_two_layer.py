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
