"""Lightweight vertex operators around the graph layers, fp64.  Test infrastructure only.

The operator abstraction (Sec. 3, App. A.1) calls element-wise work on vertices a
lightweight ApplyVertex: here the bias plus activation between two layers, and the softmax
cross-entropy that closes a training step (the paper's end-to-end runs, Sec. 7.2, train
node classifiers).  Each function is the textbook definition written out.

Activations: "identity", "relu", "elu" (alpha = 1), "leaky" (slope given).  Derivatives at
the kink: ReLU'(0) = 0, LeakyReLU'(0) = slope (the convention of the GAT score), ELU is smooth.
"""
import numpy as np

ACTS = ("identity", "relu", "elu", "leaky")


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def bias_act_forward(x, bias, act, slope=0.0):
    """out = act(x + bias); bias may be None."""
    pre = _f64(x) + (0.0 if bias is None else _f64(bias)[None, :])
    if act == "identity":
        return pre
    if act == "relu":
        return np.where(pre > 0, pre, 0.0)
    if act == "elu":
        return np.where(pre > 0, pre, np.expm1(np.minimum(pre, 0.0)))
    if act == "leaky":
        return np.where(pre > 0, pre, slope * pre)
    raise ValueError(act)


def bias_act_backward(x, bias, act, gout, slope=0.0):
    """Gradients of <gout, act(x + bias)>: (gx, gbias)."""
    pre = _f64(x) + (0.0 if bias is None else _f64(bias)[None, :])
    gout = _f64(gout)
    if act == "identity":
        d = np.ones_like(pre)
    elif act == "relu":
        d = (pre > 0).astype(np.float64)
    elif act == "elu":
        d = np.where(pre > 0, 1.0, np.exp(np.minimum(pre, 0.0)))
    elif act == "leaky":
        d = np.where(pre > 0, 1.0, slope)
    else:
        raise ValueError(act)
    gx = gout * d
    return gx, gx.sum(axis=0)


def softmax_xent(logits, labels):
    """Mean cross-entropy over the labelled vertices (label >= 0) and its gradient.

    loss = (1/L) sum_v [ log sum_c exp(z[v,c]) - z[v, label[v]] ],  dz[v] = (softmax(z[v]) - onehot) / L,
    zero rows for unlabelled vertices; L = number of labelled vertices (loss 0 if none).
    """
    z = _f64(logits)
    labels = np.asarray(labels)
    lab = labels >= 0
    L = int(lab.sum())
    g = np.zeros_like(z)
    if L == 0:
        return 0.0, g
    zl = z[lab]
    mx = zl.max(axis=1, keepdims=True)
    ex = np.exp(zl - mx)
    se = ex.sum(axis=1, keepdims=True)
    lse = (mx + np.log(se))[:, 0]
    picked = zl[np.arange(L), labels[lab]]
    loss = float((lse - picked).sum() / L)
    p = ex / se
    p[np.arange(L), labels[lab]] -= 1.0
    g[lab] = p / L
    return loss, g
