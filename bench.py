#!/usr/bin/env python3
"""Benchmark of the fused GNN layers, forward + backward, on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gat_c4]

Default workload: the Reddit-scale GAT layer (`gat_c4`), the largest GAT configuration,
on which the headline metric is quoted.  `ec_c3` (EdgeConv), `gmm_c5` (MoNet) and `gcn_c4`
(GCN on the same graph) run the same way.  One "step" is one pass of the whole hot path over the synthetic graph:
projection (MFMA), the fused edge kernels of the forward pass, the backward edge
kernels, parameter gradients and the backward products.  The graph plan (CSC
transpose, degree order, blocked edge lists) is built once per graph before the timed
region and its time is reported separately.  Inputs are resident in HBM when the timed
region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
FP32_VECTOR_TFLOPS = 157.3      # MI355X published fp32 vector peak


# ---- byte / flop models: every array a kernel touches counted once (unique), per-edge bytes with
# no cache reuse (gather), fp32 flops ------------------------------------------------------------
def gat_models(n, e, fin, H, F):
    HF = H * F
    V, S = 4 * n * HF, 4 * n * H        # one [n, HF] / one [n, H] fp32 matrix
    I = 4 * e + 8 * n                   # indices + indptr + degree order
    unique = {
        "gat_fwd_fused": I + V + 4 * S + 2 * V + S,    # z, el, er, m, d -> out, t, sg
        "gat_bwd_dst": I + 3 * V + 4 * S + S + 4 * S,  # z, out, gout, el, er, m, d -> der, table
        "gat_bwd_src": I + 3 * V + S + 4 * S + S + S,  # gout, z, dz, el, table, der -> del
    }
    gather = {
        "gat_fwd_fused": e * (4 + 4 * HF + 4 * H),
        "gat_bwd_dst": e * (4 + 4 * HF + 4 * H),
        "gat_bwd_src": e * (4 + 4 * HF + 16 * H),
    }
    flops = {
        "gat_fwd_fused": e * H * (4 * F + 14),
        "gat_bwd_dst": e * H * (2 * F + 14),
        "gat_bwd_src": e * H * (4 * F + 16),
    }
    return unique, gather, flops


def edgeconv_models(n, e, fin, F):
    V = 4 * n * F
    unique = {"edgeconv_fwd_fused": 4 * e + 8 * n + 2 * V + 2 * V,          # pq -> out, argmax
              "edgeconv_bwd_src": 8 * e + 8 * n + 2 * V + 2 * V}            # argmax, gout -> dpq
    gather = {"edgeconv_fwd_fused": e * (4 + 4 * F), "edgeconv_bwd_src": e * (8 + 8 * F)}
    flops = {"edgeconv_fwd_fused": e * F, "edgeconv_bwd_src": e * F}
    return unique, gather, flops


def gmm_models(n, e, fin, F, K):
    V = 4 * n * F
    I = 4 * e + 8 * n
    if fin % 4 == 0 and fin <= 256 and fin < K * F:
        # the library aggregates the input rows per kernel and projects afterwards: the edge kernels
        # of the forward pass and of the destination side of backward gather x (fin wide)
        X = 4 * n * fin
        unique = {"gmm_fwd_fused": I + X + 4 * n + K * X, "gmm_bwd_dst": I + X + 4 * n + K * X,
                  "gmm_bwd_src": I + V + 4 * n + K * V}
        gather = {"gmm_fwd_fused": e * (8 + 4 * fin), "gmm_bwd_dst": e * (8 + 4 * fin), "gmm_bwd_src": e * (8 + 4 * F)}
        flops = {"gmm_fwd_fused": e * K * (2 * fin + 12), "gmm_bwd_dst": e * K * (6 * fin + 14),
                 "gmm_bwd_src": e * K * (2 * F + 12)}
        return unique, gather, flops
    unique = {"gmm_fwd_fused": I + K * V + 4 * n + V,
              "gmm_bwd_dst": I + K * V + 4 * n + V,
              "gmm_bwd_src": I + V + 4 * n + K * V}
    gather = {"gmm_fwd_fused": e * (8 + 4 * K * F), "gmm_bwd_dst": e * (8 + 4 * K * F),
              "gmm_bwd_src": e * (8 + 4 * F)}
    flops = {"gmm_fwd_fused": e * K * (2 * F + 12), "gmm_bwd_dst": e * K * (6 * F + 14),
             "gmm_bwd_src": e * K * (2 * F + 12)}
    return unique, gather, flops


def gcn_models(n, e, fin, F):
    V = 4 * n * F
    I = 4 * e + 8 * n
    unique = {"gcn_fwd_fused": I + V + 4 * n + V, "gcn_bwd_src": I + V + 4 * n + V}
    gather = {"gcn_fwd_fused": e * (4 + 4 * F), "gcn_bwd_src": e * (4 + 4 * F)}
    flops = {"gcn_fwd_fused": e * F, "gcn_bwd_src": e * F}
    return unique, gather, flops


def read_traffic(workload):
    """HBM-side bytes per launch of the dominant kernel, measured with rocprofv3 --pmc
    (FETCH_SIZE, WRITE_SIZE, each calibrated on a device copy of known size) and kept in
    profiles/<workload>_hbm_traffic.txt."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    vals = {}
    try:
        for line in open(path):
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                vals[k.strip()] = v.strip()
    except OSError:
        return None
    return vals


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline_gat(c, budget_rows):
    """The numpy oracle (as it stands) timed on a bounded sample of the same workload:
    the dense products at all N vertices, and the per-edge part on the in-edges of
    `budget_rows` seeded destination rows, scaled to all E edges."""
    import numpy as np
    from oracle import gat as og
    from oracle.segments import restrict_rows
    n, e = c["n"], c["nnz"]
    rng = np.random.default_rng(12345)
    rows = np.sort(rng.choice(n, size=min(budget_rows, n), replace=False))
    ip, ix, _ = restrict_rows(c["indptr"], c["indices"], rows)
    e_s = int(ix.shape[0])
    t0 = time.perf_counter()
    fwd = og.gat_forward(ip, ix, c["x"], c["w"], c["a_l"], c["a_r"], c["slope"])
    bwd = og.gat_backward(ip, ix, c["x"], c["w"], c["a_l"], c["a_r"], c["slope"], c["gout"], fwd)
    t_sample = time.perf_counter() - t0
    # the three dense products inside that time do not shrink with the sample: time them alone
    X64, W64 = c["x"].astype(np.float64), c["w"].astype(np.float64)
    t1 = time.perf_counter()
    _ = X64 @ W64
    _ = X64.T @ bwd["dHt"]
    _ = bwd["dHt"] @ W64.T
    t_dense = time.perf_counter() - t1
    del fwd, bwd
    t_edges = max(t_sample - t_dense, 1e-9)
    t_full = t_dense + t_edges * (e / max(e_s, 1))
    return {
        "value": e / t_full, "unit": "edges/s", "cores": int(oracle_threads()), "kind": "oracle",
        "sample": (f"fp64 numpy oracle fwd+bwd on the in-edges of {len(rows)} seeded destination rows "
                   f"({e_s} of {e} edges) with all {n} vertices' dense products; measured {t_sample:.2f} s "
                   f"of which {t_dense:.2f} s dense; per-edge part scaled by E/E_sample"),
        "measured_s": t_sample,
    }


def cpu_baseline_gcn(c, budget_rows):
    """As cpu_baseline_gat: dense products at all vertices, per-edge part on sampled rows."""
    import numpy as np
    from oracle import gcn as og
    from oracle.segments import restrict_rows
    n, e = c["n"], c["nnz"]
    rng = np.random.default_rng(12345)
    rows = np.sort(rng.choice(n, size=min(budget_rows, n), replace=False))
    ip, ix, pos = restrict_rows(c["indptr"], c["indices"], rows)
    e_s = int(ix.shape[0])
    t0 = time.perf_counter()
    if "ew" in c:
        fwd = og.gcn_edge_forward(ip, ix, c["x"], c["w"], c["ew"][pos])
        bwd = og.gcn_edge_backward(ip, ix, c["x"], c["w"], c["ew"][pos], c["gout"], fwd)
    else:
        fwd = og.gcn_forward(ip, ix, c["x"], c["w"], c["c_src"], c["c_dst"])
        bwd = og.gcn_backward(ip, ix, c["x"], c["w"], c["c_src"], c["c_dst"], c["gout"], fwd)
    t_sample = time.perf_counter() - t0
    X64, W64 = c["x"].astype(np.float64), c["w"].astype(np.float64)
    t1 = time.perf_counter()
    _ = X64 @ W64
    _ = X64.T @ bwd["dZ"]
    _ = bwd["dZ"] @ W64.T
    t_dense = time.perf_counter() - t1
    del fwd, bwd
    t_full = t_dense + max(t_sample - t_dense, 1e-9) * (e / max(e_s, 1))
    return {
        "value": e / t_full, "unit": "edges/s", "cores": int(oracle_threads()), "kind": "oracle",
        "sample": (f"fp64 numpy oracle fwd+bwd on the in-edges of {len(rows)} seeded destination rows "
                   f"({e_s} of {e} edges) with all {n} vertices' dense products; measured {t_sample:.2f} s "
                   f"of which {t_dense:.2f} s dense; per-edge part scaled by E/E_sample"),
        "measured_s": t_sample,
    }


def cpu_baseline_gat2(c, sample_vertices=8192):
    """Two-layer step: the oracle runs whole on the subgraph induced by a seeded vertex sample."""
    import numpy as np
    from oracle import two_layer as ot
    n = c["n"]
    rng = np.random.default_rng(12345)
    keep = np.sort(rng.choice(n, size=min(sample_vertices, n), replace=False))
    new_id = np.full(n, -1, dtype=np.int64)
    new_id[keep] = np.arange(len(keep))
    dst = np.repeat(np.arange(n), np.diff(c["indptr"]))
    src = c["indices"].astype(np.int64)
    ok = (new_id[dst] >= 0) & (new_id[src] >= 0)
    d2, s2 = new_id[dst[ok]], new_id[src[ok]]          # still sorted by destination
    ip = np.zeros(len(keep) + 1, dtype=np.int32)
    np.add.at(ip, d2 + 1, 1)
    ip = np.cumsum(ip).astype(np.int32)
    ix = s2.astype(np.int32)
    t0 = time.perf_counter()
    fwd = ot.gat2_forward(ip, ix, c["x"][keep], c["params"], c["labels"][keep], c["slope"])
    ot.gat2_backward(ip, ix, c["x"][keep], c["params"], c["labels"][keep], c["slope"], fwd)
    dt = time.perf_counter() - t0
    return {"value": len(ix) / dt, "unit": "edges/s", "cores": int(oracle_threads()), "kind": "oracle",
            "sample": (f"fp64 numpy oracle, whole two-layer forward + backward on the subgraph induced by "
                       f"{len(keep)} seeded vertices ({len(ix)} edges), {dt:.2f} s"),
            "measured_s": dt}


def cpu_baseline_ec2(c, sample_clouds=2):
    """Two-layer EdgeConv step incl. the neighbour search: the oracle on the first clouds of the batch."""
    from oracle import knn as ok
    from oracle import two_layer as ot
    m = min(sample_clouds, c["clouds"]) * c["points"]
    t0 = time.perf_counter()
    ip, ix = ok.knn_graph(c["coords"][:m], m // c["points"], c["points"], c["k"])
    fwd = ot.two_layer_forward("edgeconv", ip, ix, c["x"][:m], c["p1"], c["b1"], c["p2"], c["b2"], {},
                               c["labels"][:m], "leaky", 0.2)
    ot.two_layer_backward("edgeconv", ip, ix, c["x"][:m], c["p1"], c["b1"], c["p2"], c["b2"], {}, c["labels"][:m],
                          "leaky", 0.2, fwd)
    dt = time.perf_counter() - t0
    return {"value": len(ix) / dt, "unit": "edges/s", "cores": int(oracle_threads()), "kind": "oracle",
            "sample": (f"numpy oracle, neighbour search (float32 distances) + fp64 two-layer forward + backward on "
                       f"the first {m // c['points']} clouds ({len(ix)} edges), {dt:.2f} s"),
            "measured_s": dt}


def cpu_baseline_monet(c, budget_rows):
    """The oracle on the in-edges of sampled destination rows (projection, layer forward and backward)."""
    import numpy as np
    from oracle import gmm as om
    from oracle.segments import restrict_rows
    n, e = c["n"], c["nnz"]
    rng = np.random.default_rng(12345)
    rows = np.sort(rng.choice(n, size=min(budget_rows, n), replace=False))
    ip, ix, _ = restrict_rows(c["indptr"], c["indices"], rows)
    t0 = time.perf_counter()
    ps = om.pseudo_projection_forward(ip, ix, c["c"], c["proj_w"], c["proj_b"])
    fwd = om.gmm_pseudo_forward(ip, ix, c["x"], c["w_fc"], ps, c["mu"], c["inv_sigma"])
    bwd = om.gmm_pseudo_backward(ip, ix, c["x"], c["w_fc"], ps, c["mu"], c["inv_sigma"], c["gout"], fwd)
    om.pseudo_projection_backward(ip, ix, c["c"], c["proj_w"], c["proj_b"], bwd["gpseudo"])
    dt = time.perf_counter() - t0
    e_s = int(ix.shape[0])
    return {"value": e_s / dt, "unit": "edges/s", "cores": int(oracle_threads()), "kind": "oracle",
            "sample": (f"fp64 numpy oracle (projection + layer, fwd+bwd) on the in-edges of {len(rows)} seeded "
                       f"destination rows ({e_s} of {e} edges) with all {n} vertices' dense products, {dt:.2f} s; "
                       f"edges of the sample per second"),
            "measured_s": dt}


def cpu_baseline_full(c):
    """EdgeConv / GMM workloads are small enough for the oracle to run whole."""
    e = c["nnz"]
    t0 = time.perf_counter()
    if c["kind"] == "edgeconv":
        from oracle import edgeconv as oe
        fwd = oe.edgeconv_forward(c["indptr"], c["indices"], c["x"], c["theta"], c["phi"])
        oe.edgeconv_backward(c["indptr"], c["indices"], c["x"], c["theta"], c["phi"], c["gout"], fwd)
    else:
        from oracle import gmm as om
        args = (c["indptr"], c["indices"], c["x"], c["w_fc"], c["c"], c["mu"], c["inv_sigma"])
        fwd = om.gmm_forward(*args)
        om.gmm_backward(*args, c["gout"], fwd)
    dt = time.perf_counter() - t0
    return {"value": e / dt, "unit": "edges/s", "cores": int(oracle_threads()), "kind": "oracle",
            "sample": f"fp64 numpy oracle fwd+bwd on the whole workload ({e} edges), {dt:.2f} s",
            "measured_s": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gat_c4")
    ap.add_argument("--cpu-rows", type=int, default=2048, help="destination rows of the CPU baseline sample (GAT)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hip-graph", action="store_true",
                    help="record one step into a HIP graph and time its replays (launch-bound small workloads)")
    ap.add_argument("--gcn-mapping", "--mapping", dest="gcn_mapping", choices=("vertex", "edge", "tuned"),
                    default="vertex",
                    help="GCN and GMM workloads: thread mapping of the aggregation; 'tuned' times both on the "
                         "graph first (gnn_gcn_tune / gnn_gmm_tune) and uses the faster one")
    ap.add_argument("--arm", choices=("vertex_stash", "recompute", "edge_stash"), default="vertex_stash",
                    help="GAT workloads, the recomputation study: vertex_stash (default: forward stashes the "
                         "vertex-sized sums t, sg), recompute (nothing but m, d is kept; one more edge pass in "
                         "backward), edge_stash (per-edge softmax values stored after forward and read back)")
    ap.add_argument("--gather-fp16", action="store_true",
                    help="GAT workloads on the column-blocked path: gather neighbour rows from an fp16 copy "
                         "(sums in fp32); outside the 1e-4 contract, reported as a variant only")
    ap.add_argument("--single-launch", action="store_true",
                    help="use the single-launch kernels also where the column-blocked ones apply")
    ap.add_argument("--block-cols", type=int, default=None,
                    help="gathered vertices per column block of the blocked edge lists (library default 12288)")
    ap.add_argument("--monet-two-call", action="store_true",
                    help="MoNet workloads: projection and layer as separate calls with [E, r] coordinate arrays "
                         "between them (gnn_pseudo_proj_* + gnn_gmmp_*) instead of gnn_monet_*")
    ap.add_argument("--no-pseudo-t", action="store_true",
                    help="MoNet workloads: the backward pass reads the pseudo-coordinates through the plan's "
                         "position -> edge table instead of a second copy in the transposed list's order")
    ap.add_argument("--no-merge-blocks", action="store_true",
                    help="one launch per column block instead of merged launches over sparse blocks")
    ap.add_argument("--resident-sums", type=int, default=None, choices=(0, 1),
                    help="1: the column-blocked kernels run all blocks in one persistent launch with the "
                         "running sums kept on the chip; 0: one launch per block group")
    ap.add_argument("--compare-unfused", action="store_true",
                    help="also time the one-operator-per-kernel comparator (GAT with heads*f = 256: forward and "
                         "backward graph operators; EdgeConv and GMM: forward)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2110_09524_amd as pk
    from workloads import make

    t0 = time.perf_counter()
    c = make(args.workload)
    t_gen = time.perf_counter() - t0
    kind, n, e, fin = c["kind"], c["n"], c["nnz"], c["fin"]
    print(f"[bench] {args.workload}: kind={kind} N={n} E={e} (generated in {t_gen:.1f} s)",
          file=sys.stderr, flush=True)

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    new = lambda *shape, dtype=torch.float32: torch.empty(shape, dtype=dtype, device=dev)
    indptr, indices = to(c["indptr"]), to(c["indices"])

    # a plain copy of known size, so a counter run of this script can be calibrated
    cal_src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    if args.single_launch:
        pk.gnn_config_set("force_simple_kernels", 1)
    if args.gather_fp16:
        pk.gnn_config_set("gather_precision", 1)
    if args.block_cols is not None:
        pk.gnn_config_set("block_cols", args.block_cols)
    if args.no_merge_blocks:
        pk.gnn_config_set("merge_blocks", 0)
    if args.resident_sums is not None:
        pk.gnn_config_set("resident_sums", args.resident_sums)
    for kv in filter(None, os.environ.get("GNN_CONFIG", "").split(",")):  # experiments: key=value,key=value
        pk.gnn_config_set(kv.split("=")[0], int(kv.split("=")[1]))
    t0 = time.perf_counter()
    g = pk.Graph(indptr, indices)
    torch.cuda.synchronize()
    t_plan = time.perf_counter() - t0

    x = to(c["x"])
    gout = to(c["gout"]) if "gout" in c else None
    gemm_total_flops = None
    if kind == "ec2":
        from paper_2110_09524_amd import steps as S
        clouds, points, k_nn, hid, C2 = c["clouds"], c["points"], c["k"], c["hid"], c["classes"]
        coords = x
        knn_ptr, knn_idx = new(n + 1, dtype=torch.int32), new(e, dtype=torch.int32)
        P1, P2 = {k: to(v) for k, v in c["p1"].items()}, {k: to(v) for k, v in c["p2"].items()}
        l1, l2 = S.EdgeConvLayer(g, fin, hid, P1), S.EdgeConvLayer(g, hid, C2, P2)
        model = S.TwoLayerStep(l1, l2, to(c["b1"]), to(c["b2"]), to(c["labels"]), n, act="leaky", act_slope=0.2)
        ws_bytes = model.ws.numel()
        held = {"g": g}

        def step():
            # the graph is rebuilt from the coordinates in every step: neighbour search, then the plan
            pk.gnn_knn_graph(clouds, points, fin, k_nn, coords, knn_ptr, knn_idx)
            g_new = pk.Graph(knn_ptr, knn_idx)
            l1.g = l2.g = g_new
            model.step(x, 1e-3)
            if held["g"] is not g:
                held["g"].close()
            held["g"] = g_new
        u1, g1, f1_ = edgeconv_models(n, e, fin, hid)
        u2, g2, f2_ = edgeconv_models(n, e, hid, C2)
        unique = {k: u1[k] + u2[k] for k in u1}
        gather = {k: g1[k] + g2[k] for k in g1}
        flops = {k: f1_[k] + f2_[k] for k in f1_}
        metric = "two-layer EdgeConv training step incl. kNN graph construction (fwd + bwd + SGD) edges/sec"
        cfg = {"layers": 2, "in_feat": fin, "hidden": hid, "classes": C2, "activation": "bias + LeakyReLU(0.2)",
               "graph": f"{clouds} clouds x {points} points, kNN k={k_nn} incl. self, rebuilt on the GPU every step",
               "loss": "softmax cross-entropy per point", "optimizer": "SGD"}
        gemm_flops = (2.0 * n * fin * 2 * hid + 2.0 * n * hid * 2 * C2) / 2
        gemm_total_flops = 3 * (2.0 * n * fin * 2 * hid + 2.0 * n * hid * 2 * C2)
    elif kind == "gat2":
        from paper_2110_09524_amd.steps import Gat2Step
        H, F, C2 = c["heads1"], c["f1"], c["classes"]
        HF = H * F
        params = {k: to(v) for k, v in c["params"].items()}
        model = Gat2Step(g, fin, H, F, C2, c["slope"], params, to(c["labels"]), int((c["labels"] >= 0).sum()))
        ws_bytes = model.ws.numel()
        lr = 1e-3

        def step():
            model.step(x, lr)
        u1, g1, f1_ = gat_models(n, e, fin, H, F)
        u2, g2, f2_ = gat_models(n, e, HF, 1, C2)
        unique = {k: u1[k] + u2[k] for k in u1}
        gather = {k: g1[k] + g2[k] for k in g1}
        flops = {k: f1_[k] + f2_[k] for k in f1_}
        metric = "two-layer GAT training step (fwd + bwd + SGD) edges/sec"
        cfg = {"layers": 2, "in_feat": fin, "hidden": f"{H}x{F}", "classes": C2, "activation": "bias + ELU",
               "loss": "softmax cross-entropy on seeded labels", "optimizer": "SGD",
               "graph": "Chung-Lu power law (gamma 2.1) + self-loops, seeded"}
        # products named gemm_f32_mfma: layer-1 projection, layer-2 projection, layer-2 input gradient
        gemm_flops = (2.0 * n * fin * HF + 2 * 2.0 * n * HF * C2) / 3
        gemm_total_flops = 2 * 2.0 * n * fin * HF + 3 * 2.0 * n * HF * C2
    elif kind == "gat":
        H, F = c["heads"], c["f"]
        HF = H * F
        w, a_l, a_r = to(c["w"]), to(c["a_l"]), to(c["a_r"])
        z, out, t = new(n, HF), new(n, HF), new(n, HF)      # t, sg: stashed dst-side sums
        el, er, m, d, sg = (new(n, H) for _ in range(5))
        gx, gw, ga_l, ga_r = new(n, fin), new(fin, HF), new(H, F), new(H, F)
        ws_bytes = pk.gnn_gat_workspace_bytes(g, fin, H, F)
        ws = new(max(ws_bytes, 16), dtype=torch.uint8)

        if args.arm == "recompute":
            t, sg = None, None
        alpha_t = new(e, H) if args.arm == "edge_stash" else None

        def step():
            pk.gnn_gat_fwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg, ws)
            if alpha_t is None:
                pk.gnn_gat_bwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg, gout,
                               gx, gw, ga_l, ga_r, ws)
            else:
                pk.gnn_gat_stash_alpha(g, H, F, c["slope"], el, er, m, d, alpha_t)
                pk.gnn_gat_bwd_stashed(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg,
                                       alpha_t, gout, gx, gw, ga_l, ga_r, ws)
        unique, gather, flops = gat_models(n, e, fin, H, F)
        metric = "fused GAT layer fwd+bwd edges/sec"
        saved = 4 * (3 * n * HF + 4 * n * H) + (4 * (n * HF + n * H) if t is not None else 0) \
            + (4 * e * H if alpha_t is not None else 0)
        cfg = {"in_feat": fin, "heads": H, "hidden_per_head": F, "arm": args.arm,
               "single_launch_kernels": bool(args.single_launch), "saved_for_backward_bytes": saved,
               "gather_storage": "fp16 copy (variant outside the 1e-4 contract)" if args.gather_fp16 else "fp32",
               "graph": "Chung-Lu power law (gamma 2.1) + self-loops, seeded"}
        gemm_flops = 2.0 * n * fin * HF
    elif kind == "edgeconv":
        F = c["fout"]
        theta, phi = to(c["theta"]), to(c["phi"])
        pq, out, argmax = new(n, 2 * F), new(n, F), new(n, F, dtype=torch.int32)
        gx, gtheta, gphi = new(n, fin), new(fin, F), new(fin, F)
        ws_bytes = pk.gnn_edgeconv_workspace_bytes(g, fin, F)
        ws = new(max(ws_bytes, 16), dtype=torch.uint8)

        def step():
            pk.gnn_edgeconv_fwd(g, fin, F, x, theta, phi, pq, out, argmax, ws)
            pk.gnn_edgeconv_bwd(g, fin, F, x, theta, phi, argmax, gout, gx, gtheta, gphi, ws)
        unique, gather, flops = edgeconv_models(n, e, fin, F)
        metric = "fused EdgeConv layer fwd+bwd edges/sec"
        k_nn, points = e // n, 1024
        cfg = {"in_feat": fin, "out_feat": F,
               "graph": f"{n // points} clouds x {points} points, kNN k={k_nn} incl. self, seeded"}
        # building the same kind of graph on the GPU from the coordinates (not part of `value`:
        # the layer is timed on a resident graph, as for the other workloads)
        coords = to(c["coords"])
        knn_ptr = new(n + 1, dtype=torch.int32)
        knn_idx = new(e, dtype=torch.int32)
        for rep in range(4):
            if rep == 1:
                torch.cuda.synchronize()
                t_k0 = time.perf_counter()
            pk.gnn_knn_graph(n // points, points, coords.shape[1], k_nn, coords, knn_ptr, knn_idx)
        torch.cuda.synchronize()
        cfg["knn_graph_build_ms"] = 1e3 * (time.perf_counter() - t_k0) / 3
        del coords, knn_ptr, knn_idx
        gemm_flops = 2.0 * n * fin * 2 * F
    elif kind == "gmm":
        F, K = c["fout"], c["k"]
        w_fc, cc, mu, inv_sigma = to(c["w_fc"]), to(c["c"]), to(c["mu"]), to(c["inv_sigma"])
        hk, out = new(n, K * F), new(n, F)
        gx, gw_fc, gmu, gis = new(n, fin), new(fin, K * F), new(K, 2), new(K, 2)
        ws_bytes = pk.gnn_gmm_workspace_bytes(g, fin, F, K)
        ws = new(max(ws_bytes, 16), dtype=torch.uint8)

        def step():
            pk.gnn_gmm_fwd(g, fin, F, K, x, w_fc, cc, mu, inv_sigma, hk, out, ws)
            pk.gnn_gmm_bwd(g, fin, F, K, x, w_fc, cc, mu, inv_sigma, hk, gout, gx, gw_fc, gmu, gis, ws)
        unique, gather, flops = gmm_models(n, e, fin, F, K)
        pk.gnn_config_set("gmm_mapping", {"vertex": 0, "edge": 1, "tuned": 2}[args.gcn_mapping])
        gmm_tune_ms = None
        if args.gcn_mapping == "tuned":
            pk.gnn_gmm_fwd(g, fin, F, K, x, w_fc, cc, mu, inv_sigma, hk, out)
            t = pk.gnn_gmm_tune(g, F, K, hk, cc, mu, inv_sigma, out)
            gmm_tune_ms = {"fwd_vertex": round(t[0], 4), "fwd_edge": round(t[1], 4)}
        metric = "fused MoNet/GMM layer fwd+bwd edges/sec"
        cfg = {"in_feat": fin, "out_feat": F, "kernels": K,
               "graph": "Chung-Lu power law (gamma 2.1) + self-loops, seeded", "mapping": args.gcn_mapping}
        if gmm_tune_ms:
            cfg["tune_ms"] = gmm_tune_ms
        gemm_flops = 2.0 * n * fin * K * F
    elif kind == "monet":
        F, K, R = c["fout"], c["k"], c["r"]
        w_fc, cc, mu, inv_sigma = to(c["w_fc"]), to(c["c"]), to(c["mu"]), to(c["inv_sigma"])
        proj_w, proj_b = to(c["proj_w"]), to(c["proj_b"])
        fused = not args.monet_two_call and K * F <= 64   # projection evaluated inside the layer's kernels
        hk, out = new(n, K * F), new(n, F)
        gx, gw_fc, gmu, gis = new(n, fin), new(fin, K * F), new(K, R), new(K, R)
        gproj_w, gproj_b = new(R, 2), new(R)
        ws_bytes = max(pk.gnn_gmmp_workspace_bytes(g, fin, F, K), pk.gnn_pseudo_proj_workspace_bytes(g))
        ws = new(max(ws_bytes, 16), dtype=torch.uint8)
        V, I = 4 * n * F, 4 * e + 8 * n
        if fused:
            def step():
                pk.gnn_monet_fwd(g, fin, F, K, R, x, w_fc, cc, proj_w, proj_b, mu, inv_sigma, hk, out)
                pk.gnn_monet_bwd(g, fin, F, K, R, x, w_fc, cc, proj_w, proj_b, mu, inv_sigma, hk, gout, gx, gw_fc,
                                 gmu, gis, gproj_w, gproj_b, ws)
            # no per-edge array: the index list, the vertex scalar c (4 n bytes) and the rows
            unique = {"monet_fwd_fused": I + 4 * n + K * V + V, "monet_bwd_dst": I + 4 * n + K * V + V,
                      "monet_bwd_src": I + 4 * n + V + K * V}
            gather = {"monet_fwd_fused": e * (4 + 4 + 4 * K * F), "monet_bwd_dst": e * (4 + 4 + 4 * K * F),
                      "monet_bwd_src": e * (4 + 4 + 4 * F)}
            flops = {"monet_fwd_fused": e * (K * (2 * F + 4 * R + 8) + 12 * R),
                     "monet_bwd_dst": e * (K * (2 * F + 10 * R + 10) + 20 * R),
                     "monet_bwd_src": e * (K * (2 * F + 4 * R + 8) + 12 * R)}
        else:
            pseudo, gpseudo = new(e, R), new(e, R)
            pseudo_t = None if args.no_pseudo_t else new(e, R)   # the coordinates in the transposed list's order

            def step():
                pk.gnn_pseudo_proj_fwd(g, R, cc, proj_w, proj_b, pseudo, pseudo_t=pseudo_t)
                pk.gnn_gmmp_fwd(g, fin, F, K, R, x, w_fc, pseudo, mu, inv_sigma, hk, out)
                pk.gnn_gmmp_bwd(g, fin, F, K, R, x, w_fc, pseudo, mu, inv_sigma, hk, gout, gx, gw_fc, gmu, gis,
                                gpseudo, ws, pseudo_t=pseudo_t)
                pk.gnn_pseudo_proj_bwd(g, R, cc, pseudo, gpseudo, gproj_w, gproj_b, ws)
            unique = {"gmmp_fwd_fused": I + 4 * e * R + K * V + V, "gmmp_bwd_dst": I + 8 * e * R + K * V + V,
                      "gmmp_bwd_src": (1 if pseudo_t is not None else 2) * I + 4 * e * R + V + K * V}
            gather = {"gmmp_fwd_fused": e * (4 + 4 * R + 4 * K * F), "gmmp_bwd_dst": e * (4 + 8 * R + 4 * K * F),
                      "gmmp_bwd_src": e * ((4 if pseudo_t is not None else 8) + 4 * R + 4 * F)}
            flops = {"gmmp_fwd_fused": e * K * (2 * F + 4 * R + 8), "gmmp_bwd_dst": e * K * (2 * F + 10 * R + 10),
                     "gmmp_bwd_src": e * K * (2 * F + 4 * R + 8)}
        metric = "MoNet/GMM layer with projected pseudo-coordinates fwd+bwd edges/sec"
        cfg = {"in_feat": fin, "out_feat": F, "kernels": K, "pseudo_dim": R,
               "pseudo": "tanh(proj_w (1/sqrt(deg_u), 1/sqrt(deg_v)) + proj_b), " +
                         ("evaluated inside the layer's kernels, no per-edge array" if fused else "[E, r] fp32 arrays"),
               "graph": "Chung-Lu power law (gamma 2.1) + self-loops, seeded"}
        gemm_flops = 2.0 * n * fin * K * F
    elif kind == "gcn":
        F = c["fout"]
        w, c_src, c_dst = to(c["w"]), to(c["c_src"]), to(c["c_dst"])
        zs, out = new(n, F), new(n, F)
        gx, gw = new(n, fin), new(fin, F)
        ws_bytes = pk.gnn_gcn_workspace_bytes(g, fin, F)
        ws = new(max(ws_bytes, 16), dtype=torch.uint8)

        ew = pk.EdgeWeights(g, to(c["ew"])) if "ew" in c else None   # general static weight per edge

        def step():
            if ew is not None:
                pk.gnn_gcn_edge_fwd(g, ew, fin, F, x, w, zs, out)
                pk.gnn_gcn_edge_bwd(g, ew, fin, F, x, w, gout, gx, gw, ws)
            else:
                pk.gnn_gcn_fwd(g, fin, F, x, w, c_src, c_dst, zs, out)
                pk.gnn_gcn_bwd(g, fin, F, x, w, c_src, c_dst, gout, gx, gw, ws)
        unique, gather, flops = gcn_models(n, e, fin, F)
        if ew is not None:    # one more 4-byte stream per edge and pass
            unique = {k: v + 4 * e for k, v in unique.items()}
            gather = {k: v + 4 * e for k, v in gather.items()}
        metric = "fused GCN layer fwd+bwd edges/sec"
        cfg = {"in_feat": fin, "out_feat": F,
               "edge_weight": "general static scalar per edge" if ew is not None else "1/sqrt(outdeg(u) indeg(v))",
               "graph": "Chung-Lu power law (gamma 2.1) + self-loops, seeded", "mapping": args.gcn_mapping}
        pk.gnn_config_set("gcn_mapping", {"vertex": 0, "edge": 1, "tuned": 2}[args.gcn_mapping])
        if args.gcn_mapping == "tuned":
            t = pk.gnn_gcn_tune(g, F, ws)
            cfg["tune_ms"] = {"in_vertex": round(t[0], 4), "in_edge": round(t[1], 4),
                              "out_vertex": round(t[2], 4), "out_edge": round(t[3], 4)}
        gemm_flops = 2.0 * n * fin * F
    else:
        raise SystemExit(f"unknown workload kind {kind}")

    run = step
    if args.hip_graph:
        # the entry points only enqueue kernels on the given stream, so a step can be recorded
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph, stream=side):
            step()
        run = hip_graph.replay
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_per_step = 1e3 * t_total / args.steps
    edges_per_s = e * args.steps / t_total

    # per-kernel durations: HIP events recorded by the library on the launch stream
    pk.gnn_prof_reset()
    pk.gnn_prof_enable(True)
    prof_steps = max(3, min(args.steps, 10))
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    rep = pk.gnn_prof_report()
    pk.gnn_prof_enable(False)
    kern = {k: {"avg_launch_ms": ms / cnt, "launches_per_step": cnt / prof_steps,
                "ms_per_step": ms / prof_steps} for k, (ms, cnt) in rep.items()}
    edge_kernels = [k for k in unique if k in kern]
    dom = max(edge_kernels, key=lambda k: kern[k]["ms_per_step"])
    # a large graph is walked in several column-block launches of the same kernel: the
    # algorithmic bytes of the operation are split evenly over them
    lps = kern[dom]["launches_per_step"]
    achieved = unique[dom] / lps / (kern[dom]["avg_launch_ms"] * 1e-3) / 1e9
    for k in edge_kernels:
        t_k = kern[k]["ms_per_step"] * 1e-3
        kern[k].update(unique_GBps=unique[k] / t_k / 1e9, gather_model_GBps=gather[k] / t_k / 1e9,
                       fp32_TFLOPs=flops[k] / t_k / 1e12)
    if "gemm_f32_mfma" in kern:
        # the projection and the input-gradient product take this name; same flop count each
        kern["gemm_f32_mfma"]["fp32_mfma_TFLOPs"] = gemm_flops / (kern["gemm_f32_mfma"]["avg_launch_ms"] * 1e-3) / 1e12

    if "gemm_f32_mfma_attn" in kern:   # the projection with the attention halves in its epilogue
        kern["gemm_f32_mfma_attn"]["fp32_mfma_TFLOPs"] = (
            2.0 * n * fin * HF / (kern["gemm_f32_mfma_attn"]["avg_launch_ms"] * 1e-3) / 1e12)

    # HBM-side counter readings are kept in a file; they are only reported when they were taken on
    # the very kernel instantiation this run launched (the library names it)
    tv = read_traffic(args.workload)
    traffic, traffic_kernel = None, None
    if tv and dom in [k.strip() for k in tv.get("kernel", "").split(",")]:   # one kernel may serve several passes
        if kind == "gat":
            mode = {"gat_bwd_src": 2, "gat_bwd_dst": 1, "gat_fwd_fused": 3 if t is not None else 0}.get(dom)
            traffic_kernel = pk.gnn_gat_blocked_kernel_name(g, H, F, mode) if mode is not None else None
            if traffic_kernel and traffic_kernel == tv.get("rocprof_kernel"):
                traffic = float(tv["hbm_bytes_per_launch"])
            else:
                print(f"[bench] profiles/{args.workload}_hbm_traffic.txt was measured on "
                      f"'{tv.get('rocprof_kernel')}', this run launches '{traffic_kernel}': traffic not reported",
                      file=sys.stderr, flush=True)
        elif kind == "gcn":
            traffic_kernel = pk.gnn_gcn_blocked_kernel_name(g, F, ew is not None)
            if traffic_kernel and traffic_kernel == tv.get("rocprof_kernel"):
                traffic = float(tv["hbm_bytes_per_launch"])
            else:
                print(f"[bench] profiles/{args.workload}_hbm_traffic.txt was measured on "
                      f"'{tv.get('rocprof_kernel')}', this run launches '{traffic_kernel}': traffic not reported",
                      file=sys.stderr, flush=True)
        else:
            traffic = float(tv["hbm_bytes_per_launch"])
    roofline = {
        "kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_kernel": traffic_kernel,
        "algorithmic_bytes_per_launch": unique[dom] / lps, "avg_launch_ms": kern[dom]["avg_launch_ms"],
        "launches_per_step": lps,
        "bytes_model": "minimal unique bytes: every array the kernel touches counted once",
        "gather_model_GBps": kern[dom]["gather_model_GBps"],
        "fp32_alu_frac": kern[dom]["fp32_TFLOPs"] / FP32_VECTOR_TFLOPS,
        # the larger of the two floors of this kernel (unique bytes at HBM speed, flops at the
        # fp32 vector peak) over its measured time
        "frac_combined": max(unique[dom] / (HBM_PEAK_GBPS * 1e9), flops[dom] / (FP32_VECTOR_TFLOPS * 1e12))
                         / (kern[dom]["ms_per_step"] * 1e-3),
    }
    # whole-layer floor: edge kernels at max(unique bytes / HBM, flops / fp32 vector peak), the
    # three dense products at the fp32 MFMA peak
    floor_s = sum(max(unique[k] / (HBM_PEAK_GBPS * 1e9), flops[k] / (FP32_VECTOR_TFLOPS * 1e12)) for k in edge_kernels)
    floor_s += (3 * gemm_flops if gemm_total_flops is None else gemm_total_flops) / (FP32_VECTOR_TFLOPS * 1e12)
    layer_floor = {"floor_ms": floor_s * 1e3, "frac": floor_s * 1e3 / ms_per_step,
                   "edge_kernels_ms_per_step": sum(kern[k]["ms_per_step"] for k in edge_kernels),
                   "edge_kernels_edges_per_s": e / (1e-3 * sum(kern[k]["ms_per_step"] for k in edge_kernels))}
    cfg.update(workload=args.workload, vertices=n, edges=e, hip_graph=bool(args.hip_graph),
               plan_ms_once_per_graph=1e3 * t_plan,
               workspace_bytes=ws_bytes)
    result = {
        "metric": metric, "value": edges_per_s, "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "config": cfg, "roofline": roofline, "layer_floor": layer_floor, "kernels": kern,
    }
    if args.compare_unfused and kind == "gat":
        from unfused_baseline.compare import compare_gat
        dz_fused = ws.view(torch.float32)[: n * HF].view(n, HF)     # first workspace region holds dz
        result["unfused_comparison"] = compare_gat(
            c, g, indptr, indices, z, el, er, gout, a_l, a_r, out, dz_fused,
            {k: v["ms_per_step"] for k, v in kern.items()})
    if args.compare_unfused and kind == "edgeconv":
        from unfused_baseline.compare import compare_edgeconv
        result["unfused_comparison"] = compare_edgeconv(
            c, indptr, indices, x, theta, phi,
            lambda: pk.gnn_edgeconv_fwd(g, fin, F, x, theta, phi, pq, out, argmax, ws), out)
    if args.compare_unfused and kind == "gmm":
        from unfused_baseline.compare import compare_gmm
        pk.gnn_linear_fwd(x, w_fc, hk)      # the comparator's input (the fused layer may skip hk)
        cmp = compare_gmm(c, indptr, indices, cc, mu, inv_sigma, hk,
                          lambda: pk.gnn_gmm_fwd(g, fin, F, K, x, w_fc, cc, mu, inv_sigma, hk, out, ws), out)
        cmp["fused_graph_fwd_ms"] = kern["gmm_fwd_fused"]["ms_per_step"]
        cmp["time_ratio_unfused_over_fused"] = cmp["unfused_graph_fwd_ms"] / cmp["fused_graph_fwd_ms"]
        result["unfused_comparison"] = cmp
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample ...", file=sys.stderr, flush=True)
        if kind == "gat":
            result["cpu_baseline"] = cpu_baseline_gat(c, args.cpu_rows)
        elif kind == "gat2":
            result["cpu_baseline"] = cpu_baseline_gat2(c)
        elif kind == "ec2":
            result["cpu_baseline"] = cpu_baseline_ec2(c)
        elif kind == "monet":
            result["cpu_baseline"] = cpu_baseline_monet(c, args.cpu_rows)
        elif kind == "gcn":
            result["cpu_baseline"] = cpu_baseline_gcn(c, args.cpu_rows)
        else:
            result["cpu_baseline"] = cpu_baseline_full(c)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
