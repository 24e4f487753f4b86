"""Two stacked GAT layers with bias and ELU between them and a softmax cross-entropy on top,
forward and backward, fp64.  Test infrastructure only.

This is the shape of the paper's end-to-end GAT runs (Sec. 7.2: two layers, node
classification).  Nothing new is computed here: the functions chain the single-layer
definitions (gat.py), the vertex operators and the loss (apply_vertex.py) by the chain rule.

    h1   = GAT_1(x)                 [n, H1*F1]
    a1   = ELU(h1 + b1)
    h2   = GAT_2(a1)                [n, C]      (one head)
    z    = h2 + b2
    loss = mean cross-entropy of z over the labelled vertices
"""
from . import apply_vertex as av
from . import gat as og


def gat2_forward(indptr, indices, x, p, labels, slope):
    """p: dict with w1, al1, ar1, b1, w2, al2, ar2, b2."""
    f1 = og.gat_forward(indptr, indices, x, p["w1"], p["al1"], p["ar1"], slope)
    a1 = av.bias_act_forward(f1["out"], p["b1"], "elu")
    f2 = og.gat_forward(indptr, indices, a1, p["w2"], p["al2"], p["ar2"], slope)
    z = av.bias_act_forward(f2["out"], p["b2"], "identity")
    loss, gz = av.softmax_xent(z, labels)
    return dict(f1=f1, a1=a1, f2=f2, z=z, loss=loss, gz=gz)


def gat2_backward(indptr, indices, x, p, labels, slope, fwd=None):
    """Gradients of the loss w.r.t. every parameter (same keys as p, prefixed with g)."""
    if fwd is None:
        fwd = gat2_forward(indptr, indices, x, p, labels, slope)
    gh2, gb2 = av.bias_act_backward(fwd["f2"]["out"], p["b2"], "identity", fwd["gz"])
    b2 = og.gat_backward(indptr, indices, fwd["a1"], p["w2"], p["al2"], p["ar2"], slope, gh2, fwd["f2"])
    gh1, gb1 = av.bias_act_backward(fwd["f1"]["out"], p["b1"], "elu", b2["gx"])
    b1 = og.gat_backward(indptr, indices, x, p["w1"], p["al1"], p["ar1"], slope, gh1, fwd["f1"])
    return dict(gw1=b1["gw"], gal1=b1["ga_l"], gar1=b1["ga_r"], gb1=gb1,
                gw2=b2["gw"], gal2=b2["ga_l"], gar2=b2["ga_r"], gb2=gb2,
                gh1=gh1, gh2=gh2, ga1=b2["gx"])
