"""Two-layer training steps chained from the C-ABI calls (the end-to-end setting of the paper's
Sec. 7.2: two layers, bias + activation between them, node classification).  This module owns
device buffers and orders the calls; every number is computed by the HIP kernels.

    h1 = Layer_1(x) -> a1 = act(h1 + b1) -> h2 = Layer_2(a1) -> z = h2 + b2 -> mean cross-entropy

A layer object holds its parameters (device tensors), the tensors its forward call saves and
its parameter gradients; `forward(x, ws)` returns the output tensor, `backward(x, gout, gx, ws)`
fills `grads` (and gx unless it is None).
"""
import torch

from . import binding as B


def _new(dev, *shape, dtype=torch.float32):
    return torch.empty(shape, dtype=dtype, device=dev)


class GatLayer:
    """params: w [fin, heads*f], al, ar [heads, f]."""

    def __init__(self, graph, fin, heads, f, slope, params):
        self.g, self.fin, self.h, self.f, self.slope, self.p = graph, fin, heads, f, slope, params
        n, hf, dev = graph.n, heads * f, params["w"].device
        self.fout = hf
        self.s = dict(z=_new(dev, n, hf), el=_new(dev, n, heads), er=_new(dev, n, heads), m=_new(dev, n, heads),
                      d=_new(dev, n, heads), out=_new(dev, n, hf), t=_new(dev, n, hf), sg=_new(dev, n, heads))
        self.grads = {k: torch.empty_like(v) for k, v in params.items()}

    def workspace_bytes(self):
        return B.gnn_gat_workspace_bytes(self.g, self.fin, self.h, self.f)

    def forward(self, x, ws):
        p, s = self.p, self.s
        B.gnn_gat_fwd(self.g, self.fin, self.h, self.f, self.slope, x, p["w"], p["al"], p["ar"], s["z"], s["el"],
                      s["er"], s["m"], s["d"], s["out"], s["t"], s["sg"], ws)
        return s["out"]

    def backward(self, x, gout, gx, ws):
        p, s, g = self.p, self.s, self.grads
        B.gnn_gat_bwd(self.g, self.fin, self.h, self.f, self.slope, x, p["w"], p["al"], p["ar"], s["z"], s["el"],
                      s["er"], s["m"], s["d"], s["out"], s["t"], s["sg"], gout, gx, g["w"], g["al"], g["ar"], ws)


class EdgeConvLayer:
    """params: theta, phi [fin, fout]."""

    def __init__(self, graph, fin, fout, params):
        self.g, self.fin, self.fout, self.p = graph, fin, fout, params
        n, dev = graph.n, params["theta"].device
        self.pq, self.out = _new(dev, n, 2 * fout), _new(dev, n, fout)
        self.argmax = _new(dev, n, fout, dtype=torch.int32)
        self.grads = {k: torch.empty_like(v) for k, v in params.items()}

    def workspace_bytes(self):
        return B.gnn_edgeconv_workspace_bytes(self.g, self.fin, self.fout)

    def forward(self, x, ws):
        B.gnn_edgeconv_fwd(self.g, self.fin, self.fout, x, self.p["theta"], self.p["phi"], self.pq, self.out,
                           self.argmax, ws)
        return self.out

    def backward(self, x, gout, gx, ws):
        B.gnn_edgeconv_bwd(self.g, self.fin, self.fout, x, self.p["theta"], self.p["phi"], self.argmax, gout,
                           gx, self.grads["theta"], self.grads["phi"], ws)


class GmmLayer:
    """params: w_fc [fin, k*fout], mu, inv_sigma [k, 2]; c [n]: per-vertex pseudo-coordinate (constant)."""

    def __init__(self, graph, fin, fout, k, params, c):
        self.g, self.fin, self.fout, self.k, self.p, self.c = graph, fin, fout, k, params, c
        n, dev = graph.n, c.device
        self.hk, self.out = _new(dev, n, k * fout), _new(dev, n, fout)
        self.grads = {k_: torch.empty_like(v) for k_, v in params.items()}

    def workspace_bytes(self):
        return B.gnn_gmm_workspace_bytes(self.g, self.fin, self.fout, self.k)

    def forward(self, x, ws):
        p = self.p
        B.gnn_gmm_fwd(self.g, self.fin, self.fout, self.k, x, p["w_fc"], self.c, p["mu"], p["inv_sigma"], self.hk,
                      self.out, ws)
        return self.out

    def backward(self, x, gout, gx, ws):
        p, g = self.p, self.grads
        B.gnn_gmm_bwd(self.g, self.fin, self.fout, self.k, x, p["w_fc"], self.c, p["mu"], p["inv_sigma"], self.hk,
                      gout, gx, g["w_fc"], g["mu"], g["inv_sigma"], ws)


class MonetLayer:
    """GMM layer with pseudo-coordinates projected from the pair (c[u], c[v]) to r dimensions.
    params: w_fc [fin, k*fout], mu, inv_sigma [k, r], proj_w [r, 2], proj_b [r]; c [n] constant."""

    def __init__(self, graph, fin, fout, k, r, params, c):
        self.g, self.fin, self.fout, self.k, self.r, self.p, self.c = graph, fin, fout, k, r, params, c
        n, e, dev = graph.n, max(graph.nnz, 1), c.device
        self.hk, self.out = _new(dev, n, k * fout), _new(dev, n, fout)
        # up to 64 projected floats per row the projection is fused into the layer's kernels and no
        # per-edge tensor exists; wider layers keep the coordinates, in both edge orders
        self.fused = k * fout <= 64
        if not self.fused:
            self.pseudo, self.gpseudo, self.pseudo_t = _new(dev, e, r), _new(dev, e, r), _new(dev, e, r)
        self.grads = {k_: torch.empty_like(v) for k_, v in params.items()}

    def workspace_bytes(self):
        return max(B.gnn_gmmp_workspace_bytes(self.g, self.fin, self.fout, self.k),
                   B.gnn_pseudo_proj_workspace_bytes(self.g))

    def forward(self, x, ws):
        p = self.p
        if self.fused:
            B.gnn_monet_fwd(self.g, self.fin, self.fout, self.k, self.r, x, p["w_fc"], self.c, p["proj_w"],
                            p["proj_b"], p["mu"], p["inv_sigma"], self.hk, self.out)
            return self.out
        B.gnn_pseudo_proj_fwd(self.g, self.r, self.c, p["proj_w"], p["proj_b"], self.pseudo, pseudo_t=self.pseudo_t)
        B.gnn_gmmp_fwd(self.g, self.fin, self.fout, self.k, self.r, x, p["w_fc"], self.pseudo, p["mu"],
                       p["inv_sigma"], self.hk, self.out)
        return self.out

    def backward(self, x, gout, gx, ws):
        p, g = self.p, self.grads
        if self.fused:
            B.gnn_monet_bwd(self.g, self.fin, self.fout, self.k, self.r, x, p["w_fc"], self.c, p["proj_w"],
                            p["proj_b"], p["mu"], p["inv_sigma"], self.hk, gout, gx, g["w_fc"], g["mu"],
                            g["inv_sigma"], g["proj_w"], g["proj_b"], ws)
            return
        B.gnn_gmmp_bwd(self.g, self.fin, self.fout, self.k, self.r, x, p["w_fc"], self.pseudo, p["mu"],
                       p["inv_sigma"], self.hk, gout, gx, g["w_fc"], g["mu"], g["inv_sigma"], self.gpseudo, ws,
                       pseudo_t=self.pseudo_t)
        B.gnn_pseudo_proj_bwd(self.g, self.r, self.c, self.pseudo, self.gpseudo, g["proj_w"], g["proj_b"], ws)


class GcnLayer:
    """params: w [fin, fout]; c_src, c_dst [n]: the two factors of the static edge weight."""

    def __init__(self, graph, fin, fout, params, c_src, c_dst):
        self.g, self.fin, self.fout, self.p, self.c_src, self.c_dst = graph, fin, fout, params, c_src, c_dst
        n, dev = graph.n, c_src.device
        self.zs, self.out = _new(dev, n, fout), _new(dev, n, fout)
        self.grads = {k: torch.empty_like(v) for k, v in params.items()}

    def workspace_bytes(self):
        return B.gnn_gcn_workspace_bytes(self.g, self.fin, self.fout)

    def forward(self, x, ws):
        B.gnn_gcn_fwd(self.g, self.fin, self.fout, x, self.p["w"], self.c_src, self.c_dst, self.zs, self.out)
        return self.out

    def backward(self, x, gout, gx, ws):
        B.gnn_gcn_bwd(self.g, self.fin, self.fout, x, self.p["w"], self.c_src, self.c_dst, gout, gx,
                      self.grads["w"], ws)


class TwoLayerStep:
    """layer1 -> act(. + b1) -> layer2 -> (. + b2) -> softmax cross-entropy; backward; optional SGD.
    labels: int32 [n], entries outside [0, classes) mark unlabelled vertices."""

    def __init__(self, layer1, layer2, b1, b2, labels, n_labelled, act="elu", act_slope=0.0):
        assert layer1.fout == layer2.fin
        self.l1, self.l2, self.b1, self.b2 = layer1, layer2, b1, b2
        self.labels, self.n_labelled, self.act, self.act_slope = labels, n_labelled, act, act_slope
        self.n, self.hid, self.c = layer1.g.n, layer1.fout, layer2.fout
        dev = labels.device
        self.a1, self.ga1 = _new(dev, self.n, self.hid), _new(dev, self.n, self.hid)
        self.logits, self.glogits, self.loss = _new(dev, self.n, self.c), _new(dev, self.n, self.c), _new(dev, 1)
        self.gb1, self.gb2 = torch.empty_like(b1), torch.empty_like(b2)
        ws_bytes = max(layer1.workspace_bytes(), layer2.workspace_bytes(),
                       B.gnn_bias_act_workspace_bytes(self.n, self.hid), B.gnn_bias_act_workspace_bytes(self.n, self.c),
                       B.gnn_softmax_xent_workspace_bytes(self.n), 16)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def forward(self, x):
        h1 = self.l1.forward(x, self.ws)
        B.gnn_bias_act_fwd(self.n, self.hid, self.act, self.act_slope, h1, self.b1, self.a1)
        h2 = self.l2.forward(self.a1, self.ws)
        B.gnn_bias_act_fwd(self.n, self.c, "identity", 0.0, h2, self.b2, self.logits)
        B.gnn_softmax_xent(self.n, self.c, self.n_labelled, self.logits, self.labels, self.loss, self.glogits,
                           self.ws)

    def backward(self, x):
        B.gnn_bias_act_bwd(self.n, self.c, "identity", 0.0, None, self.glogits, self.glogits, self.gb2, self.ws)
        self.l2.backward(self.a1, self.glogits, self.ga1, self.ws)
        B.gnn_bias_act_bwd(self.n, self.hid, self.act, self.act_slope, self.a1, self.ga1, self.ga1, self.gb1,
                           self.ws)
        self.l1.backward(x, self.ga1, None, self.ws)

    def parameters(self):
        """(parameter, gradient) pairs of everything the step trains."""
        pairs = [(self.b1, self.gb1), (self.b2, self.gb2)]
        for layer in (self.l1, self.l2):
            pairs += [(layer.p[k], layer.grads[k]) for k in layer.p]
        return pairs

    def sgd(self, lr):
        for param, grad in self.parameters():
            B.gnn_sgd_update(lr, grad, param)

    def step(self, x, lr=None):
        self.forward(x)
        self.backward(x)
        if lr is not None:
            self.sgd(lr)


class Gat2Step(TwoLayerStep):
    """Two GAT layers (the second with one head of `classes` columns), bias + ELU between them.
    params: w1 [fin,h1*f1], al1/ar1 [h1,f1], b1 [h1*f1], w2 [h1*f1,classes], al2/ar2 [1,classes], b2 [classes]."""

    def __init__(self, graph, fin, heads1, f1, classes, slope, params, labels, n_labelled, need_gx=False):
        del need_gx  # the input features carry no gradient
        l1 = GatLayer(graph, fin, heads1, f1, slope, dict(w=params["w1"], al=params["al1"], ar=params["ar1"]))
        l2 = GatLayer(graph, heads1 * f1, 1, classes, slope, dict(w=params["w2"], al=params["al2"], ar=params["ar2"]))
        super().__init__(l1, l2, params["b1"], params["b2"], labels, n_labelled, act="elu")
        self.grads = dict(w1=l1.grads["w"], al1=l1.grads["al"], ar1=l1.grads["ar"], b1=self.gb1,
                          w2=l2.grads["w"], al2=l2.grads["al"], ar2=l2.grads["ar"], b2=self.gb2)
