"""A two-layer GAT training step chained from the C-ABI calls (the end-to-end setting of the
paper's Sec. 7.2: two GAT layers, node classification).  This module owns device buffers
and orders the calls; every number is computed by the HIP kernels.

    h1 = GAT_1(x) -> a1 = ELU(h1 + b1) -> h2 = GAT_2(a1) -> z = h2 + b2 -> mean cross-entropy
"""
import torch

from . import binding as B


class Gat2Step:
    """params: dict of device tensors w1 [fin,h1*f1], al1/ar1 [h1,f1], b1 [h1*f1],
    w2 [h1*f1,classes], al2/ar2 [1,classes], b2 [classes]; labels int32 [n] (< 0: unlabelled)."""

    def __init__(self, graph, fin, heads1, f1, classes, slope, params, labels, n_labelled, need_gx=False):
        self.g, self.n = graph, graph.n
        self.fin, self.h1, self.f1, self.c, self.slope = fin, heads1, f1, classes, slope
        self.p, self.labels, self.n_labelled = params, labels, n_labelled
        n, hf, dev = self.n, heads1 * f1, labels.device
        new = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
        self.l1 = dict(z=new(n, hf), el=new(n, heads1), er=new(n, heads1), m=new(n, heads1), d=new(n, heads1),
                       out=new(n, hf), t=new(n, hf), sg=new(n, heads1))
        self.a1 = new(n, hf)
        self.l2 = dict(z=new(n, classes), el=new(n, 1), er=new(n, 1), m=new(n, 1), d=new(n, 1),
                       out=new(n, classes), t=new(n, classes), sg=new(n, 1))
        self.logits, self.glogits, self.loss = new(n, classes), new(n, classes), new(1)
        self.ga1 = new(n, hf)
        self.gx = new(n, fin) if need_gx else None
        self.grads = {k: torch.empty_like(v) for k, v in params.items()}
        ws_bytes = max(B.gnn_gat_workspace_bytes(graph, fin, heads1, f1),
                       B.gnn_gat_workspace_bytes(graph, hf, 1, classes),
                       B.gnn_bias_act_workspace_bytes(n, hf), B.gnn_bias_act_workspace_bytes(n, classes),
                       B.gnn_softmax_xent_workspace_bytes(n), 16)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def forward(self, x):
        p, l1, l2, n = self.p, self.l1, self.l2, self.n
        hf = self.h1 * self.f1
        B.gnn_gat_fwd(self.g, self.fin, self.h1, self.f1, self.slope, x, p["w1"], p["al1"], p["ar1"], l1["z"],
                      l1["el"], l1["er"], l1["m"], l1["d"], l1["out"], l1["t"], l1["sg"], self.ws)
        B.gnn_bias_act_fwd(n, hf, "elu", 0.0, l1["out"], p["b1"], self.a1)
        B.gnn_gat_fwd(self.g, hf, 1, self.c, self.slope, self.a1, p["w2"], p["al2"], p["ar2"], l2["z"],
                      l2["el"], l2["er"], l2["m"], l2["d"], l2["out"], l2["t"], l2["sg"], self.ws)
        B.gnn_bias_act_fwd(n, self.c, "identity", 0.0, l2["out"], p["b2"], self.logits)
        B.gnn_softmax_xent(n, self.c, self.n_labelled, self.logits, self.labels, self.loss, self.glogits, self.ws)

    def backward(self, x):
        p, g, l1, l2, n = self.p, self.grads, self.l1, self.l2, self.n
        hf = self.h1 * self.f1
        B.gnn_bias_act_bwd(n, self.c, "identity", 0.0, None, self.glogits, self.glogits, g["b2"], self.ws)
        B.gnn_gat_bwd(self.g, hf, 1, self.c, self.slope, self.a1, p["w2"], p["al2"], p["ar2"], l2["z"], l2["el"],
                      l2["er"], l2["m"], l2["d"], l2["out"], l2["t"], l2["sg"], self.glogits, self.ga1, g["w2"],
                      g["al2"], g["ar2"], self.ws)
        B.gnn_bias_act_bwd(n, hf, "elu", 0.0, self.a1, self.ga1, self.ga1, g["b1"], self.ws)
        B.gnn_gat_bwd(self.g, self.fin, self.h1, self.f1, self.slope, x, p["w1"], p["al1"], p["ar1"], l1["z"],
                      l1["el"], l1["er"], l1["m"], l1["d"], l1["out"], l1["t"], l1["sg"], self.ga1, self.gx,
                      g["w1"], g["al1"], g["ar1"], self.ws)

    def sgd(self, lr):
        for k, v in self.p.items():
            B.gnn_sgd_update(lr, self.grads[k], v)

    def step(self, x, lr=None):
        self.forward(x)
        self.backward(x)
        if lr is not None:
            self.sgd(lr)
