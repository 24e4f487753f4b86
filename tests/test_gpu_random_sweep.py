"""Seeded random sweep over all four layers: graph sizes from 1 to 1800 vertices, empty graphs, hub
vertices that hear from / speak to most of the graph, rows without in-edges, duplicate edges, odd
and maximal widths, forced column blocking in one persistent launch or with merged and unmerged launches, both thread
mappings, every backward arm — each case against the fp64 oracle element by element."""
import numpy as np
import pytest

from helpers import tiny_graph

pytestmark = pytest.mark.gpu

GAT_SHAPES = [(1, 4), (1, 16), (2, 12), (3, 8), (4, 64), (4, 32), (8, 8), (8, 16), (1, 256), (2, 256), (8, 128),
              (5, 4), (16, 4), (1, 512), (1, 32), (2, 32), (1, 64), (1, 128), (2, 64), (4, 16)]


def random_graph_with_extremes(rng, n, m, hub, empties):
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    if hub:
        for h in rng.choice(n, size=int(rng.integers(1, 4)), replace=False):
            fans = rng.choice(n, size=min(n, int(rng.integers(n // 2, n + 1))), replace=False)
            src, dst = np.concatenate([src, fans]), np.concatenate([dst, np.full(len(fans), h)])
            out_sz = int(rng.integers(n // 4, n))
            src = np.concatenate([src, np.full(out_sz, h)])
            dst = np.concatenate([dst, rng.integers(0, n, size=out_sz)])
    if empties:
        dead = rng.choice(n, size=max(1, n // 20), replace=False)
        keep = ~np.isin(dst, dead)
        src, dst = src[keep], dst[keep]
    return tiny_graph(n, list(zip(src.tolist(), dst.tolist())))


def one_trial(rng, pk):
    import gpu_harness
    import test_gpu_edgeconv as TE
    import test_gpu_gat as TG
    import test_gpu_gcn as TC
    import test_gpu_gmm as TM
    n = int(rng.choice([1, 7, 60, 257, 900, 1800]))
    m = int(rng.integers(0, 30 * n + 1)) if n > 1 else int(rng.integers(0, 3))
    indptr, indices = random_graph_with_extremes(rng, n, m, hub=n >= 60 and rng.random() < 0.6,
                                                 empties=n >= 60 and rng.random() < 0.5)
    bc = int(rng.choice([24576, 16, 64, 128, 300, 512])) if n >= 60 else 24576
    mg = int(rng.integers(0, 2))
    kind = str(rng.choice(["gat", "gat", "gmm", "ec", "gcn", "gcnw"]))
    rs = int((int(indices.sum()) + len(indices) + n) % 2)   # persistent launch or launches per block (a function
    pk.gnn_config_set("block_cols", bc)                      # of the graph, so the random stream stays as it was)
    pk.gnn_config_set("merge_blocks", mg)
    pk.gnn_config_set("resident_sums", rs)
    gpu_harness.ROW_SCALED_IN_SWEEP.update({"gx", "out"} if kind == "gmm" else {"gx"})
    if kind == "gat":
        H, F = GAT_SHAPES[int(rng.integers(0, len(GAT_SHAPES)))]
        fin = int(rng.choice([2, 5, 24, 70]))
        stash, astash = bool(rng.random() < 0.7), bool(rng.random() < 0.25)
        desc = f"gat n={n} nnz={len(indices)} fin={fin} H={H} F={F} bc={bc} merge={mg} resident={rs} stash={stash} alpha_stash={astash}"
        c = TG.synth(rng, indptr, indices, fin, H, F)
        fwd, bwd = TG.oracle_all(c)
        try:
            amb_vh, _ = gpu_harness.gat_kink_masks(c["indptr"], fwd)
        except AssertionError:
            return desc + " (skipped: too many raw scores on the LeakyReLU kink)", False
        res = gpu_harness.run_gat(c, stash=stash, alpha_stash=astash)
        res.pop("alpha_t", None)
        if amb_vh.any():   # either slope is legitimate there, so sums over all edges are not comparable
            for k in ("gw", "ga_l", "ga_r"):
                res[k] = bwd[k]
        TG.compare(c, res, fwd, bwd)
    elif kind == "gmm":
        fin, fout, K = int(rng.choice([3, 16, 40])), int(rng.choice([4, 16, 64, 100, 256])), int(rng.integers(1, 9))
        mp = int(rng.integers(0, 2))
        desc = f"gmm n={n} nnz={len(indices)} fin={fin} fout={fout} K={K} mapping={mp}"
        pk.gnn_config_set("gmm_mapping", mp)
        TM.check(TM.synth(rng, indptr, indices, fin, fout, K))
    elif kind == "ec":
        fin, fout = int(rng.choice([3, 16, 40])), int(rng.choice([4, 16, 64, 128, 260, 1024]))
        desc = f"ec n={n} nnz={len(indices)} fin={fin} fout={fout}"
        TE.check(TE.synth(rng, indptr, indices, fin, fout))
    else:
        fin, fout = int(rng.choice([3, 16, 40])), int(rng.choice([4, 32, 64, 128, 256, 512, 1024, 36]))
        mp = int(rng.integers(0, 2))
        desc = f"{kind} n={n} nnz={len(indices)} fin={fin} fout={fout} bc={bc} merge={mg} resident={rs} mapping={mp}"
        c = TC.synth(rng, indptr, indices, fin, fout)
        if kind == "gcn":
            pk.gnn_config_set("gcn_mapping", mp)
            TC.check(c)
        else:
            c["ew"] = rng.standard_normal(len(indices)).astype(np.float32)
            TC.check_edge(c)
    return desc, True


@pytest.mark.parametrize("seed", range(6))
def test_random_cases_match_the_oracle(seed):
    import paper_2110_09524_amd as pk
    import gpu_harness
    failures, ran = [], 0
    try:
        for trial in range(100):
            rng = np.random.default_rng(1_000_003 * seed + trial)
            desc = "?"
            try:
                desc, counted = one_trial(rng, pk)
                ran += counted
            except AssertionError as ex:
                failures.append(f"seed {seed} trial {trial}: {str(ex)[:300]}")
            finally:
                gpu_harness.ROW_SCALED_IN_SWEEP.clear()
                pk.gnn_config_set("block_cols", 12288)
                pk.gnn_config_set("merge_blocks", 1)
                pk.gnn_config_set("resident_sums", 1)
                pk.gnn_config_set("gmm_mapping", 2)
                pk.gnn_config_set("gcn_mapping", 2)
    finally:
        gpu_harness.ROW_SCALED_IN_SWEEP.clear()
    print(f"sweep seed {seed}: {ran} cases compared", flush=True)
    assert not failures, "\n".join(failures)
    assert ran >= 80
