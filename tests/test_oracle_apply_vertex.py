"""Pins of the vertex operators and the loss: library routines, closed forms, finite differences."""
import numpy as np
import pytest
from scipy.special import log_softmax

from helpers import finite_difference
from oracle import apply_vertex as av


def test_activation_values_at_known_points():
    x = np.array([[-1.0, 0.0, 2.0]])
    np.testing.assert_allclose(av.bias_act_forward(x, None, "elu"), [[np.exp(-1.0) - 1.0, 0.0, 2.0]], rtol=1e-15)
    np.testing.assert_allclose(av.bias_act_forward(x, None, "relu"), [[0.0, 0.0, 2.0]])
    np.testing.assert_allclose(av.bias_act_forward(x, None, "leaky", 0.2), [[-0.2, 0.0, 2.0]])
    np.testing.assert_allclose(av.bias_act_forward(x, np.array([1.0, 1.0, 1.0]), "identity"), [[0.0, 1.0, 3.0]])
    # the bias is added before the activation
    np.testing.assert_allclose(av.bias_act_forward(x, np.array([2.0, -3.0, -5.0]), "relu"), [[1.0, 0.0, 0.0]])


@pytest.mark.parametrize("act", av.ACTS)
def test_backward_matches_finite_differences(act):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((7, 5))
    x[np.abs(x) < 0.05] = 0.3          # keep away from the kinks
    b = rng.standard_normal(5) * 0.1
    gout = rng.standard_normal((7, 5))
    gx, gb = av.bias_act_backward(x, b, act, gout, 0.2)
    _, fx = finite_difference(lambda t: float((gout * av.bias_act_forward(t, b, act, 0.2)).sum()), x)
    _, fb = finite_difference(lambda t: float((gout * av.bias_act_forward(x, t, act, 0.2)).sum()), b)
    np.testing.assert_allclose(gx.reshape(-1), fx, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(gb, fb, rtol=1e-6, atol=1e-8)


def test_kink_conventions():
    z = np.zeros((1, 1))
    one = np.ones((1, 1))
    assert av.bias_act_backward(z, None, "relu", one)[0][0, 0] == 0.0
    assert av.bias_act_backward(z, None, "leaky", one, 0.2)[0][0, 0] == 0.2
    assert av.bias_act_backward(z, None, "elu", one)[0][0, 0] == 1.0


def test_xent_uniform_logits_give_log_c():
    for c in (2, 4, 41):
        loss, g = av.softmax_xent(np.full((5, c), 3.7), np.arange(5) % c)
        assert abs(loss - np.log(c)) < 1e-14
        np.testing.assert_allclose(g.sum(axis=1), 0.0, atol=1e-16)


def test_xent_against_library_log_softmax_and_shift_invariance():
    rng = np.random.default_rng(4)
    z = rng.standard_normal((9, 6)) * 4
    labels = rng.integers(0, 6, 9)
    labels[[2, 5]] = -1
    lab = labels >= 0
    ref = -log_softmax(z[lab], axis=1)[np.arange(lab.sum()), labels[lab]].mean()
    loss, g = av.softmax_xent(z, labels)
    assert abs(loss - ref) < 1e-13
    assert (g[~lab] == 0).all()
    shifted, g2 = av.softmax_xent(z + rng.standard_normal((9, 1)) * 50, labels)
    assert abs(shifted - loss) < 1e-10
    np.testing.assert_allclose(g2, g, atol=1e-12)
    # huge logits must not overflow
    big, _ = av.softmax_xent(np.array([[1000.0, 0.0]]), np.array([0]))
    assert abs(big) < 1e-12


def test_xent_gradient_matches_finite_differences_and_no_labels():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((6, 4))
    labels = np.array([0, 3, -1, 2, 2, 1])
    _, g = av.softmax_xent(z, labels)
    _, fd = finite_difference(lambda t: av.softmax_xent(t, labels)[0], z)
    np.testing.assert_allclose(g.reshape(-1), fd, rtol=1e-6, atol=1e-9)
    loss, g0 = av.softmax_xent(z, np.full(6, -1))
    assert loss == 0.0 and (g0 == 0).all()
