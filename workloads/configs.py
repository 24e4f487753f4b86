"""The named workloads: seeded graphs plus tensors shaped like the evaluation's.

Inputs only (random structure, random values); no layer arithmetic lives here.

  gat_c1   Cora-scale GAT forward, 64 -> 1 head x 16           (Sec. 7.2)
  gat_c2   Pubmed-scale GAT, 500 -> 8 heads x 8, fwd+bwd       (Sec. 7.2)
  ec_c3    EdgeConv, 32 clouds x 1024 points, k=20, 64 -> 64   (Sec. 7.2)
  gat_c4   Reddit-scale GAT, 602 -> 4 heads x 64, fwd+bwd      (Sec. 7.2/7.3)
  gmm_c5   MoNet, K=3 kernels, r=2 pseudo-coords, 64 -> 64     (Sec. 7.2)
  ec_k40   EdgeConv ablation setting: 64 clouds x 1024 points, k=40, 64 -> 64  (Sec. 7.3)
  gcn_c4   GCN with symmetric normalisation on the gat_c4 graph, 602 -> 256 (App. A.2)

Smaller "mid" variants keep a workload's feature widths (hence the same kernel
instantiation and launch shape) on a graph the CPU oracle finishes in seconds.
"""
from __future__ import annotations

import numpy as np

from . import graphs

SEED0 = 0x9E3779B97F4A7C15

__all__ = ["make", "NAMES", "glorot", "SEED0"]


def glorot(rng, fan_in, fan_out, shape):
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=shape).astype(np.float32)


def _normal(rng, shape):
    return rng.standard_normal(size=shape, dtype=np.float32)


def _gat(name, n, graph, fin, heads, f, seed, x_kind="normal"):
    indptr, indices = graph
    rng = graphs.rng_for(seed ^ 0xA5A5)
    if x_kind == "normal":
        x = _normal(rng, (n, fin))
    else:  # sparse binary bag-of-words features, 5 % ones
        x = (rng.random((n, fin), dtype=np.float32) < 0.05).astype(np.float32)
    return dict(
        name=name, kind="gat", n=n, nnz=int(indices.shape[0]), fin=fin, heads=heads, f=f,
        slope=0.2, indptr=indptr, indices=indices, x=x,
        w=glorot(rng, fin, heads * f, (fin, heads * f)),
        a_l=glorot(rng, f, 1, (heads, f)),
        a_r=glorot(rng, f, 1, (heads, f)),
        gout=_normal(rng, (n, heads * f)),
    )


def _gat2(name, n, graph, fin, heads1, f1, classes, seed, x_kind="normal", labelled=0.5):
    """Two-layer node classifier: fin -> heads1 x f1 (ELU) -> classes (one head), seeded labels on a
    fraction of the vertices (the others carry -1)."""
    indptr, indices = graph
    rng = graphs.rng_for(seed ^ 0xA5A5)
    if x_kind == "normal":
        x = _normal(rng, (n, fin))
    else:
        x = (rng.random((n, fin), dtype=np.float32) < 0.05).astype(np.float32)
    hf = heads1 * f1
    labels = rng.integers(0, classes, n).astype(np.int32)
    labels[rng.random(n) >= labelled] = -1
    return dict(
        name=name, kind="gat2", n=n, nnz=int(indices.shape[0]), fin=fin, heads1=heads1, f1=f1,
        classes=classes, slope=0.2, indptr=indptr, indices=indices, x=x, labels=labels,
        params=dict(
            w1=glorot(rng, fin, hf, (fin, hf)), al1=glorot(rng, f1, 1, (heads1, f1)),
            ar1=glorot(rng, f1, 1, (heads1, f1)), b1=(0.1 * _normal(rng, (hf,))).astype(np.float32),
            w2=glorot(rng, hf, classes, (hf, classes)), al2=glorot(rng, classes, 1, (1, classes)),
            ar2=glorot(rng, classes, 1, (1, classes)), b2=(0.1 * _normal(rng, (classes,))).astype(np.float32)),
    )


def _edgeconv(name, batch, points, k, fin, fout, seed):
    indptr, indices, coords = graphs.knn_point_clouds(batch, points, k, seed)
    n = batch * points
    rng = graphs.rng_for(seed ^ 0xA5A5)
    return dict(
        name=name, kind="edgeconv", n=n, nnz=int(indices.shape[0]), fin=fin, fout=fout,
        indptr=indptr, indices=indices, coords=coords,
        x=_normal(rng, (n, fin)),
        theta=glorot(rng, fin, fout, (fin, fout)),
        phi=glorot(rng, fin, fout, (fin, fout)),
        gout=_normal(rng, (n, fout)),
    )


def _gmm(name, n, graph, fin, fout, k, seed):
    indptr, indices = graph
    rng = graphs.rng_for(seed ^ 0xA5A5)
    deg = np.diff(indptr).astype(np.float64)
    c = (1.0 / np.sqrt(np.maximum(deg, 1.0))).astype(np.float32)
    return dict(
        name=name, kind="gmm", n=n, nnz=int(indices.shape[0]), fin=fin, fout=fout, k=k,
        indptr=indptr, indices=indices,
        x=_normal(rng, (n, fin)),
        w_fc=glorot(rng, fin, k * fout, (fin, k * fout)),
        c=c,
        mu=(0.1 * rng.standard_normal(size=(k, 2))).astype(np.float32),
        inv_sigma=np.ones((k, 2), dtype=np.float32),
        gout=_normal(rng, (n, fout)),
    )


def _gcn(name, n, graph, fin, fout, seed):
    indptr, indices = graph
    rng = graphs.rng_for(seed ^ 0xA5A5)
    indeg = np.diff(indptr).astype(np.float64)
    outdeg = np.bincount(indices, minlength=n).astype(np.float64)
    return dict(
        name=name, kind="gcn", n=n, nnz=int(indices.shape[0]), fin=fin, fout=fout,
        indptr=indptr, indices=indices,
        x=_normal(rng, (n, fin)),
        w=glorot(rng, fin, fout, (fin, fout)),
        # symmetric normalisation of a directed graph: 1/sqrt(out-degree of the source) and
        # 1/sqrt(in-degree of the destination)
        c_src=(1.0 / np.sqrt(np.maximum(outdeg, 1.0))).astype(np.float32),
        c_dst=(1.0 / np.sqrt(np.maximum(indeg, 1.0))).astype(np.float32),
        gout=_normal(rng, (n, fout)),
    )


def _make_gat_c1(seed):
    n = 2000
    return _gat("gat_c1", n, graphs.erdos_renyi(n, 10_000, seed), 64, 1, 16, seed)


def _make_gat_c2(seed):
    n = 20_000
    return _gat("gat_c2", n, graphs.chung_lu(n, 100_000, 2.1, seed), 500, 8, 8, seed,
                x_kind="binary")


def _make_ec_c3(seed):
    return _edgeconv("ec_c3", 32, 1024, 20, 64, 64, seed)


def _make_gat_c4(seed):
    n = 232_965
    return _gat("gat_c4", n, graphs.chung_lu(n, 114_000_000, 2.1, seed), 602, 4, 64, seed)


def _make_gmm_c5(seed):
    n = 100_000
    return _gmm("gmm_c5", n, graphs.chung_lu(n, 2_000_000, 2.1, seed), 64, 64, 3, seed)


def _make_ec_k40(seed):
    return _edgeconv("ec_k40", 64, 1024, 40, 64, 64, seed)


def _make_ec_l3(seed):
    # third and fourth layer widths of the four-layer EdgeConv model (Sec. 7.2: {64, 64, 128, 256})
    return _edgeconv("ec_l3", 64, 1024, 40, 64, 128, seed)


def _make_ec_l4(seed):
    return _edgeconv("ec_l4", 64, 1024, 40, 128, 256, seed)


def _make_ec_k40_mid(seed):
    return _edgeconv("ec_k40_mid", 3, 400, 40, 64, 128, seed)


def _make_gcn_c4(seed):
    n = 232_965
    # the same graph as gat_c4 (its id seeds the generator)
    return _gcn("gcn_c4", n, graphs.chung_lu(n, 114_000_000, 2.1, SEED0 ^ 4), 602, 256, seed)


def _make_gcnw_c4(seed):
    # gcn_c4 with a general static weight per edge (App. A.2 "GCN": e_uv), here uniform in (0, 2/indeg(v))
    c = _make_gcn_c4(seed)
    rng = graphs.rng_for(seed ^ 0x5A5A)
    indeg = np.diff(c["indptr"]).astype(np.float32)
    dst_deg = np.repeat(indeg, np.diff(c["indptr"]))
    c.update(name="gcnw_c4", ew=(rng.random(c["nnz"], dtype=np.float32) * 2.0 / np.maximum(dst_deg, 1.0)).astype(np.float32))
    return c


def _make_gcn_c5(seed):
    # GCN on the gmm_c5 graph (100 000 vertices, average degree 21): several rows per run of edges
    n = 100_000
    return _gcn("gcn_c5", n, graphs.chung_lu(n, 2_000_000, 2.1, SEED0 ^ 5), 64, 64, seed)


def _make_gat2_mid(seed):
    n = 3000
    return _gat2("gat2_mid", n, graphs.chung_lu(n, 60_000, 2.1, seed), 96, 2, 32, 8, seed)


def _make_gat2_c2(seed):
    # the end-to-end GAT setting of Sec. 7.2 (two layers, 128 hidden, one head) on the gat_c2 graph
    n = 20_000
    return _gat2("gat2_c2", n, graphs.chung_lu(n, 100_000, 2.1, SEED0 ^ 2), 500, 1, 128, 4, seed,
                 x_kind="binary", labelled=0.3)


def _make_gat2_c4(seed):
    # the same on the gat_c4 graph; 44 output columns stand in for Reddit's 41 classes (f % 4 == 0)
    n = 232_965
    return _gat2("gat2_c4", n, graphs.chung_lu(n, 114_000_000, 2.1, SEED0 ^ 4), 602, 1, 128, 44, seed,
                 labelled=0.66)


def _make_ec2_c3(seed):
    """Two EdgeConv layers on point clouds, graph built from the coordinates in every step
    (the end-to-end EdgeConv setting of Sec. 7.2, cut to two layers): 3 -> 64 -> 40 classes per point."""
    batch, points, k, hid, classes = 32, 1024, 20, 64, 40
    indptr, indices, coords = graphs.knn_point_clouds(batch, points, k, SEED0 ^ 3)
    n = batch * points
    rng = graphs.rng_for(seed ^ 0xA5A5)
    labels = rng.integers(0, classes, n).astype(np.int32)
    return dict(
        name="ec2_c3", kind="ec2", n=n, nnz=int(indices.shape[0]), fin=3, hid=hid, classes=classes,
        clouds=batch, points=points, k=k, indptr=indptr, indices=indices, coords=coords, x=coords, labels=labels,
        p1=dict(theta=glorot(rng, 3, hid, (3, hid)), phi=glorot(rng, 3, hid, (3, hid))),
        p2=dict(theta=glorot(rng, hid, classes, (hid, classes)), phi=glorot(rng, hid, classes, (hid, classes))),
        b1=(0.1 * _normal(rng, (hid,))).astype(np.float32), b2=(0.1 * _normal(rng, (classes,))).astype(np.float32),
    )


def _monet(name, n, graph, fin, fout, K, r, seed):
    """MoNet layer with r-dimensional pseudo-coordinates projected from (1/sqrt(deg_u), 1/sqrt(deg_v))
    (the paper's MoNet settings, Sec. 7.2 / 7.3)."""
    indptr, indices = graph
    rng = graphs.rng_for(seed ^ 0xA5A5)
    deg = np.maximum(np.diff(indptr), 1)
    return dict(
        name=name, kind="monet", n=n, nnz=int(indices.shape[0]), fin=fin, fout=fout, k=K, r=r,
        indptr=indptr, indices=indices, x=_normal(rng, (n, fin)),
        w_fc=glorot(rng, fin, K * fout, (fin, K * fout)), c=(1.0 / np.sqrt(deg)).astype(np.float32),
        proj_w=_normal(rng, (r, 2)), proj_b=(0.1 * _normal(rng, (r,))).astype(np.float32),
        mu=(0.3 * _normal(rng, (K, r))).astype(np.float32), inv_sigma=np.ones((K, r), dtype=np.float32),
        gout=_normal(rng, (n, fout)),
    )


def _make_monet_c4(seed):
    # the ablation setting of Sec. 7.3: k = 2, r = 1, 16 features, Reddit-scale graph
    n = 232_965
    return _monet("monet_c4", n, graphs.chung_lu(n, 114_000_000, 2.1, SEED0 ^ 4), 602, 16, 2, 1, seed)


def _make_monet_c5(seed):
    # k = 3, r = 3 (the Pubmed / Citeseer setting) on the gmm_c5 graph
    n = 100_000
    return _monet("monet_c5", n, graphs.chung_lu(n, 2_000_000, 2.1, SEED0 ^ 5), 64, 16, 3, 3, seed)


def _make_gcn_mid(seed):
    n = 6000
    return _gcn("gcn_mid", n, graphs.chung_lu(n, 300_000, 2.1, seed), 602, 256, seed)


# mid-size variants: same widths as the big workload, oracle-sized graphs
def _make_gat_c4_mid(seed):
    n = 6000
    return _gat("gat_c4_mid", n, graphs.chung_lu(n, 300_000, 2.1, seed), 602, 4, 64, seed)


def _make_ec_c3_mid(seed):
    return _edgeconv("ec_c3_mid", 3, 500, 20, 64, 64, seed)


def _make_gmm_c5_mid(seed):
    n = 8000
    return _gmm("gmm_c5_mid", n, graphs.chung_lu(n, 160_000, 2.1, seed), 64, 64, 3, seed)


_MAKERS = {
    "gat_c1": (1, _make_gat_c1),
    "gat_c2": (2, _make_gat_c2),
    "ec_c3": (3, _make_ec_c3),
    "gat_c4": (4, _make_gat_c4),
    "gmm_c5": (5, _make_gmm_c5),
    "gat_c4_mid": (104, _make_gat_c4_mid),
    "ec_c3_mid": (103, _make_ec_c3_mid),
    "gmm_c5_mid": (105, _make_gmm_c5_mid),
    "ec_k40": (7, _make_ec_k40),
    "ec_k40_mid": (107, _make_ec_k40_mid),
    "ec_l3": (11, _make_ec_l3),
    "ec_l4": (12, _make_ec_l4),
    "gcn_c4": (6, _make_gcn_c4),
    "gcnw_c4": (16, _make_gcnw_c4),
    "gcn_mid": (106, _make_gcn_mid),
    "gcn_c5": (8, _make_gcn_c5),
    "gat2_mid": (109, _make_gat2_mid),
    "gat2_c2": (9, _make_gat2_c2),
    "gat2_c4": (10, _make_gat2_c4),
    "ec2_c3": (13, _make_ec2_c3),
    "monet_c4": (14, _make_monet_c4),
    "monet_c5": (15, _make_monet_c5),
}
NAMES = tuple(_MAKERS)


def make(name: str, seed: int | None = None) -> dict:
    """Build the named workload.  Default seed = SEED0 xor the workload's id."""
    cid, fn = _MAKERS[name]
    s = (SEED0 ^ cid) if seed is None else int(seed)
    return fn(s)
