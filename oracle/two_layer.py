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


# ---- the same chain for the other layer types --------------------------------------------
# A layer is described by (kind, parameter dict, constants dict):
#   "gat":      params w, al, ar;  consts slope
#   "edgeconv": params theta, phi
#   "gmm":      params w_fc, mu, inv_sigma;  consts c (per-vertex pseudo-coordinate)
#   "gcn":      params w;  consts c_src, c_dst
#   "monet":    params w_fc, mu, inv_sigma, proj_w, proj_b;  consts c   (pseudo-coordinates projected
#               from the pair (c[u], c[v]) to r = proj_w.shape[0] dimensions, each layer its own projection)
def layer_forward(kind, indptr, indices, x, p, k):
    if kind == "gat":
        return og.gat_forward(indptr, indices, x, p["w"], p["al"], p["ar"], k["slope"])
    if kind == "edgeconv":
        from . import edgeconv as oe
        return oe.edgeconv_forward(indptr, indices, x, p["theta"], p["phi"])
    if kind == "gmm":
        from . import gmm as om
        return om.gmm_forward(indptr, indices, x, p["w_fc"], k["c"], p["mu"], p["inv_sigma"])
    if kind == "gcn":
        from . import gcn as oc
        return oc.gcn_forward(indptr, indices, x, p["w"], k["c_src"], k["c_dst"])
    if kind == "monet":
        from . import gmm as om
        ps = om.pseudo_projection_forward(indptr, indices, k["c"], p["proj_w"], p["proj_b"])
        f = om.gmm_pseudo_forward(indptr, indices, x, p["w_fc"], ps, p["mu"], p["inv_sigma"])
        f["pseudo"] = ps
        return f
    raise ValueError(kind)


def layer_backward(kind, indptr, indices, x, p, k, gout, fwd):
    """Returns (gx, dict of parameter gradients keyed like p)."""
    if kind == "gat":
        b = og.gat_backward(indptr, indices, x, p["w"], p["al"], p["ar"], k["slope"], gout, fwd)
        return b["gx"], dict(w=b["gw"], al=b["ga_l"], ar=b["ga_r"])
    if kind == "edgeconv":
        from . import edgeconv as oe
        b = oe.edgeconv_backward(indptr, indices, x, p["theta"], p["phi"], gout, fwd)
        return b["gx"], dict(theta=b["gtheta"], phi=b["gphi"])
    if kind == "gmm":
        from . import gmm as om
        b = om.gmm_backward(indptr, indices, x, p["w_fc"], k["c"], p["mu"], p["inv_sigma"], gout, fwd)
        return b["gx"], dict(w_fc=b["gw_fc"], mu=b["gmu"], inv_sigma=b["ginv_sigma"])
    if kind == "gcn":
        from . import gcn as oc
        b = oc.gcn_backward(indptr, indices, x, p["w"], k["c_src"], k["c_dst"], gout, fwd)
        return b["gx"], dict(w=b["gw"])
    if kind == "monet":
        from . import gmm as om
        b = om.gmm_pseudo_backward(indptr, indices, x, p["w_fc"], fwd["pseudo"], p["mu"], p["inv_sigma"], gout, fwd)
        gP, gpb = om.pseudo_projection_backward(indptr, indices, k["c"], p["proj_w"], p["proj_b"], b["gpseudo"])
        return b["gx"], dict(w_fc=b["gw_fc"], mu=b["gmu"], inv_sigma=b["ginv_sigma"], proj_w=gP, proj_b=gpb)
    raise ValueError(kind)


def two_layer_forward(kind, indptr, indices, x, p1, b1, p2, b2, consts, labels, act="elu", act_slope=0.0):
    """layer -> act(. + b1) -> layer -> (. + b2) -> mean cross-entropy over labelled vertices."""
    f1 = layer_forward(kind, indptr, indices, x, p1, consts)
    a1 = av.bias_act_forward(f1["out"], b1, act, act_slope)
    f2 = layer_forward(kind, indptr, indices, a1, p2, consts)
    z = av.bias_act_forward(f2["out"], b2, "identity")
    loss, gz = av.softmax_xent(z, labels)
    return dict(f1=f1, a1=a1, f2=f2, z=z, loss=loss, gz=gz)


def two_layer_backward(kind, indptr, indices, x, p1, b1, p2, b2, consts, labels, act="elu", act_slope=0.0,
                       fwd=None):
    """Returns (g1, gb1, g2, gb2): parameter gradient dicts of the two layers and the bias gradients."""
    if fwd is None:
        fwd = two_layer_forward(kind, indptr, indices, x, p1, b1, p2, b2, consts, labels, act, act_slope)
    gh2, gb2 = av.bias_act_backward(fwd["f2"]["out"], b2, "identity", fwd["gz"])
    ga1, g2 = layer_backward(kind, indptr, indices, fwd["a1"], p2, consts, gh2, fwd["f2"])
    gh1, gb1 = av.bias_act_backward(fwd["f1"]["out"], b1, act, ga1, act_slope)
    _, g1 = layer_backward(kind, indptr, indices, x, p1, consts, gh1, fwd["f1"])
    return g1, gb1, g2, gb2
