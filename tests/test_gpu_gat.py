"""GAT layer: HIP path (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest

from oracle import gat as og
from helpers import random_graph, tiny_graph
from workloads import make

pytestmark = pytest.mark.gpu


def oracle_all(c, backward=True):
    fwd = og.gat_forward(c["indptr"], c["indices"], c["x"], c["w"], c["a_l"], c["a_r"], c["slope"])
    bwd = None
    if backward:
        bwd = og.gat_backward(c["indptr"], c["indices"], c["x"], c["w"], c["a_l"], c["a_r"],
                              c["slope"], c["gout"], fwd)
    return fwd, bwd


def compare(c, res, fwd, bwd):
    from gpu_harness import assert_close, gat_kink_masks
    n, H, F = c["n"], c["heads"], c["f"]
    amb_vh, amb_vertex = gat_kink_masks(c["indptr"], fwd)
    keep_vh = ~amb_vh
    keep_hf = np.repeat(keep_vh, F, axis=1)
    Ht = fwd["Ht"].reshape(n, H * F)
    assert_close("z", res["z"], Ht)
    assert_close("el", res["el"], np.einsum("nhf,hf->nh", fwd["Ht"], c["a_l"].astype(np.float64)))
    assert_close("er", res["er"], np.einsum("nhf,hf->nh", fwd["Ht"], c["a_r"].astype(np.float64)))
    assert_close("m", res["m"], fwd["mx"])
    assert_close("d", res["d"], fwd["den"])
    assert_close("out", res["out"], fwd["out"])
    if "t" in res:
        # stashed destination-side sums: t = sum alpha_e g_e Ht[u], sg = sum alpha_e g_e,
        # g_e = LeakyReLU'(M0_e), written out from the oracle's materialised tensors
        from oracle.segments import segment_sum
        ag = fwd["M2"] * np.where(fwd["M0"] > 0, 1.0, c["slope"])
        sg_ref = segment_sum(c["indptr"], ag)
        t_ref = segment_sum(c["indptr"], ag[:, :, None] * fwd["Ht"][fwd["src"]]).reshape(n, H * F)
        assert_close("sg", np.where(keep_vh, res["sg"], sg_ref), sg_ref)
        assert_close("t", np.where(keep_hf, res["t"], t_ref), t_ref)
    if bwd is not None:
        assert_close("gx", np.where(amb_vertex[:, None], bwd["gx"], res["gx"]), bwd["gx"])
        assert_close("gw", res["gw"], bwd["gw"], reduce_scale=True)
        assert_close("ga_l", res["ga_l"], bwd["ga_l"], reduce_scale=True)
        assert_close("ga_r", res["ga_r"], bwd["ga_r"], reduce_scale=True)


def synth(rng, indptr, indices, fin, H, F, slope=0.2):
    n = len(indptr) - 1
    return dict(n=n, nnz=len(indices), fin=fin, heads=H, f=F, slope=slope, indptr=indptr,
                indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                # Glorot-scaled like the workloads: scores stay O(1)
                w=(rng.standard_normal((fin, H * F)) * np.sqrt(2.0 / (fin + H * F))).astype(np.float32),
                a_l=(rng.standard_normal((H, F)) * np.sqrt(2.0 / (F + 1))).astype(np.float32),
                a_r=(rng.standard_normal((H, F)) * np.sqrt(2.0 / (F + 1))).astype(np.float32),
                gout=rng.standard_normal((n, H * F)).astype(np.float32))


def test_c1_forward():
    from gpu_harness import run_gat
    print("gat: gat_c1 forward", flush=True)
    c = make("gat_c1")
    fwd, _ = oracle_all(c, backward=False)
    compare(c, run_gat(c, backward=False), fwd, None)


@pytest.mark.parametrize("name", ["gat_c1", "gat_c2", "gat_c4_mid"])
def test_workload_forward_backward(name):
    from gpu_harness import run_gat
    print("gat:", name, "fwd+bwd", flush=True)
    c = make(name)
    fwd, bwd = oracle_all(c)
    compare(c, run_gat(c), fwd, bwd)
    # without the stash the backward call recomputes the destination-side sums
    compare(c, run_gat(c, stash=False), fwd, bwd)


@pytest.mark.parametrize("fin,H,F", [(7, 1, 4), (33, 3, 8), (5, 2, 12), (19, 5, 4), (64, 2, 64),
                                     (40, 8, 64), (24, 3, 256), (130, 1, 16)])
def test_shapes_heads_and_widths(fin, H, F):
    from gpu_harness import run_gat
    print(f"gat: shape fin={fin} H={H} F={F}", flush=True)
    rng = np.random.default_rng(fin * 1000 + H * 10 + F)
    indptr, indices = random_graph(rng, 257, 3000, self_loops=True, duplicates=True)
    c = synth(rng, indptr, indices, fin, H, F)
    fwd, bwd = oracle_all(c)
    compare(c, run_gat(c), fwd, bwd)


def test_empty_rows_isolated_vertices_and_hub():
    from gpu_harness import run_gat
    print("gat: empty rows + hub", flush=True)
    rng = np.random.default_rng(5)
    n = 700
    # vertex 0 is a hub receiving from everyone (several chunks and a ragged tail),
    # vertices 1..9 have no in-edges, vertex 10 sends to nobody, the rest is sparse
    edges = [(u, 0) for u in range(n) if u != 10]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(11, n) for _ in range(int(v) % 4)]
    edges = [(u if u != 10 else 11, v) for (u, v) in edges]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, 20, 4, 16)
    fwd, bwd = oracle_all(c)
    res = run_gat(c)
    compare(c, res, fwd, bwd)
    assert (res["out"][1:10] == 0).all() and (res["m"][1:10] == 0).all() and (res["d"][1:10] == 1).all()


def test_single_vertex_self_loop_and_skipped_input_gradient():
    from gpu_harness import run_gat
    print("gat: single vertex", flush=True)
    rng = np.random.default_rng(6)
    c = synth(rng, np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32), 3, 2, 4)
    fwd, bwd = oracle_all(c)
    res = run_gat(c, want_gx=False)
    res["gx"] = bwd["gx"]
    compare(c, res, fwd, bwd)


def test_graph_without_edges():
    from gpu_harness import run_gat
    print("gat: no edges", flush=True)
    rng = np.random.default_rng(61)
    n = 37
    c = synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 5, 2, 8)
    fwd, bwd = oracle_all(c)
    res = run_gat(c)
    compare(c, res, fwd, bwd)
    assert (res["out"] == 0).all() and (res["m"] == 0).all() and (res["d"] == 1).all()
    for k in ("gx", "gw", "ga_l", "ga_r"):
        assert (res[k] == 0).all(), k


def test_results_are_bit_reproducible():
    from gpu_harness import run_gat
    print("gat: reproducibility", flush=True)
    c = make("gat_c2")
    a, b = run_gat(c), run_gat(c)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_bad_arguments_raise():
    import paper_2110_09524_amd as pk
    import torch
    from gpu_harness import dev, empty, workspace
    print("gat: error paths", flush=True)
    c = make("gat_c1")
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    n = c["n"]
    x, w = dev(c["x"]), dev(c["w"])
    bufs = [empty((n, 16)) for _ in range(2)] + [empty((n, 1)) for _ in range(4)]
    z, out, el, er, m, d = bufs
    a6 = empty((1, 6))
    with pytest.raises(pk.GnnError) as e:        # f = 6 is not a multiple of 4
        pk.gnn_gat_fwd(g, 64, 1, 6, 0.2, x, w, a6, a6, z, el, er, m, d, out)
    assert e.value.status == 4
    a = dev(c["a_l"])
    with pytest.raises(pk.GnnError) as e:        # t without sg
        pk.gnn_gat_fwd(g, 64, 1, 16, 0.2, x, w, a, a, z, el, er, m, d, out, empty((n, 16)), None)
    assert e.value.status == 1
    pk.gnn_gat_fwd(g, 64, 1, 16, 0.2, x, w, a, a, z, el, er, m, d, out)
    need = pk.gnn_gat_workspace_bytes(g, 64, 1, 16)
    assert need > 0
    with pytest.raises(pk.GnnError) as e:        # workspace too small
        pk.gnn_gat_bwd(g, 64, 1, 16, 0.2, x, w, a, a, z, el, er, m, d, out, None, None,
                       dev(c["gout"]), None, empty((64, 16)), empty((1, 16)), empty((1, 16)),
                       workspace(need - 256))
    assert e.value.status == 3
    torch.cuda.synchronize()


@pytest.mark.parametrize("block_cols,H,F", [(256, 4, 64), (1024, 4, 64), (500, 1, 256), (300, 8, 16),
                                            (200, 2, 256), (128, 8, 128),
                                            # 512-byte rows: four slices of 128 bytes; narrower rows
                                            # take the single-launch kernels on such graphs, too
                                            (256, 1, 128), (300, 4, 32), (256, 2, 64), (500, 1, 64),
                                            # one head of at most 64 columns: a single slice of the
                                            # persistent kernels (merge = 2), rows shorter than the slice
                                            (300, 1, 44), (256, 1, 4), (200, 1, 60)])
@pytest.mark.parametrize("merge", [0, 1, 2])
def test_column_blocked_path(block_cols, H, F, merge):
    """The multi-launch, column-blocked kernels (used when the gathered matrix exceeds
    the L2 caches) on a graph small enough for the oracle, with small blocks forced: one launch
    per block (0), launches that walk several sparse blocks per row (1), and all blocks in one
    persistent launch that keeps the running sums in LDS (2; rows cut into 256-byte slices, the
    other shapes fall back to the launches)."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    print(f"gat: blocked path block_cols={block_cols} H={H} F={F} merge={merge}", flush=True)
    if (H, F) == (4, 64):
        c = make("gat_c4_mid")
    else:
        rng = np.random.default_rng(block_cols + H + F)
        indptr, indices = random_graph(rng, 1500, 30000, self_loops=False, duplicates=True)
        c = synth(rng, indptr, indices, 24, H, F)
    fwd, bwd = oracle_all(c)
    pk.gnn_config_set("block_cols", block_cols)
    pk.gnn_config_set("merge_blocks", int(merge == 1))
    pk.gnn_config_set("resident_sums", int(merge == 2))
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        nb = g.blocked(0)[0]
        assert nb == -(-c["n"] // block_cols)
        launches = len(g.launch_groups(0, 2)) - 1
        print(f"  {nb} blocks in {launches} launches", flush=True)
        assert launches == nb if merge != 1 else 1 <= launches <= nb
        res = run_gat(c, graph=g)
        res_recompute = run_gat(c, graph=g, stash=False)   # blocked recompute of the dst side
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("merge_blocks", 1)
        pk.gnn_config_set("resident_sums", 1)
    compare(c, res, fwd, bwd)
    compare(c, res_recompute, fwd, bwd)
    # same inputs through the single-launch kernels: both paths must agree with the oracle
    pk.gnn_config_set("force_simple_kernels", 1)
    try:
        res2 = run_gat(c, graph=g)
    finally:
        pk.gnn_config_set("force_simple_kernels", 0)
    compare(c, res2, fwd, bwd)
    assert np.array_equal(res["m"], res2["m"])      # the row maximum is exact on both paths


@pytest.mark.parametrize("H,F,block_cols", [(4, 64, 256), (1, 256, 500), (2, 256, 200), (1, 128, 256), (2, 64, 300)])
def test_resident_sums_repeat_the_launch_per_block_results_bit_for_bit(H, F, block_cols):
    """The persistent kernel adds a row's chunks in the order of the launch-per-block kernels, whoever
    draws the row and however the workgroups pace each other (also with the bounded wait cut to zero
    polls): every output equals the unmerged launches' bit for bit."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    print(f"gat: resident sums H={H} F={F} block_cols={block_cols}", flush=True)
    rng = np.random.default_rng(7 * block_cols + H + F)
    n = 1800
    indptr, indices = random_graph(rng, n, 40000, self_loops=False, duplicates=True)
    c = synth(rng, indptr, indices, 16, H, F)
    pk.gnn_config_set("block_cols", block_cols)
    pk.gnn_config_set("merge_blocks", 0)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        runs = {}
        for key, resident, spin in (("launches", 0, 4096), ("resident", 1, 4096), ("unpaced", 1, 0)):
            pk.gnn_config_set("resident_sums", resident)
            pk.gnn_config_set("resident_spin", spin)
            runs[key] = (run_gat(c, graph=g), run_gat(c, graph=g, stash=False))
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("merge_blocks", 1)
        pk.gnn_config_set("resident_sums", 1)
        pk.gnn_config_set("resident_spin", 4096)
    g.close()
    for key in ("resident", "unpaced"):
        for a, b in zip(runs["launches"], runs[key]):
            for name in a:
                if isinstance(a[name], np.ndarray):
                    assert np.array_equal(a[name], b[name]), f"{key}: {name} differs from the launch-per-block result"


@pytest.mark.parametrize("H,F", [(4, 64), (8, 32), (1, 512), (2, 128), (1, 256)])
def test_blocked_path_with_the_score_table_in_lds(H, F):
    """A column block whose rows are long (>= 128 edges per row on average) is walked by the
    persistent variant that keeps the block's el table in LDS and draws rows from a counter;
    sparser blocks of the same graph take the plain variant.  Both against the oracle, and
    the two variants bit for bit against each other (they add the same terms in the same order)."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    print(f"gat: blocked path, LDS score table H={H} F={F}", flush=True)
    rng = np.random.default_rng(1000 + H * F)
    n, block_cols = 700, 512
    edges = []
    for v in range(n):
        if v == 5:
            continue                                   # a row without in-edges
        k0 = n if v == 0 else 150 + int(rng.integers(0, 60))   # vertex 0: every source, the rest: a long row
        srcs = np.arange(n) if v == 0 else np.concatenate(
            [rng.choice(block_cols, size=k0, replace=False),
             block_cols + rng.choice(n - block_cols, size=20, replace=False)])
        edges += [(int(u), v) for u in srcs]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, 16, H, F)
    in_block0 = int((indices < block_cols).sum())
    assert in_block0 >= 128 * n and len(indices) - in_block0 < 128 * n   # one block of each kind
    fwd, bwd = oracle_all(c)
    pk.gnn_config_set("block_cols", block_cols)
    pk.gnn_config_set("resident_sums", 0)       # the launch-per-block kernels are the ones with the table
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        assert g.blocked(0)[0] == 2
        pk.gnn_prof_reset()
        pk.gnn_prof_enable(True)
        res = run_gat(c, graph=g)
        pk.gnn_prof_enable(False)
        assert "gat_blk_queue_reset" in pk.gnn_prof_report()       # the persistent variant was set up
        res_nostash = run_gat(c, graph=g, stash=False)
        pk.gnn_config_set("lds_scalar_table", 0)
        try:
            ref = run_gat(c, graph=g)
        finally:
            pk.gnn_config_set("lds_scalar_table", 1)
        g.close()
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("resident_sums", 1)
    compare(c, res, fwd, bwd)
    compare(c, res_nostash, fwd, bwd)
    for k in res:
        assert np.array_equal(res[k], ref[k]), f"{k}: LDS-table and plain variants differ"


@pytest.mark.parametrize("blocked", [False, True, "launch per block"])
def test_large_score_range_is_stable(blocked):
    """Scores spanning hundreds of units: without the max subtraction exp() would overflow,
    with it most weights underflow to exactly 0 and the rest must still match (Sec. 7.2, the
    numerically stable softmax of App. A.1).  Forward values are held to the usual bar.  A raw
    score of magnitude |s| carries |s| 2^-24 of fp32 rounding, which exp() turns into the same
    relative error of every weight; at |s| ~ 150 that is ~1e-5 per edge, ten times the usual
    1e-6, so the gradients (sums of differences of such weights) get ten times the usual bar."""
    import paper_2110_09524_amd as pk
    from gpu_harness import ATOL, RTOL, assert_close, dev, gat_kink_masks, run_gat
    print(f"gat: large score range, blocked={blocked}", flush=True)
    rng = np.random.default_rng(77)
    indptr, indices = random_graph(rng, 600, 9000, self_loops=True, duplicates=False)
    c = synth(rng, indptr, indices, 12, 4, 32)
    c["a_l"] = (c["a_l"] * 60).astype(np.float32)
    c["a_r"] = (c["a_r"] * 60).astype(np.float32)
    fwd, bwd = oracle_all(c)
    spread = float(np.abs(fwd["M1"]).max())
    assert spread > 100.0                                       # the case is what it claims to be
    pk.gnn_config_set("block_cols", 128 if blocked else 12288)
    pk.gnn_config_set("resident_sums", int(blocked != "launch per block"))
    try:
        res = run_gat(c)
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("resident_sums", 1)
    grads = {k: res.pop(k) for k in ("gx", "gw", "ga_l", "ga_r")}
    compare(c, res, fwd, None)
    assert np.isfinite(res["out"]).all() and (res["d"] >= 1.0 - 1e-6).all()
    _, amb_vertex = gat_kink_masks(c["indptr"], fwd)
    assert_close("gx", np.where(amb_vertex[:, None], bwd["gx"], grads["gx"]), bwd["gx"], rtol=10 * RTOL,
                 atol=10 * ATOL, row_scale=True)
    for k in ("gw", "ga_l", "ga_r"):
        assert_close(k, grads[k], bwd[k], rtol=10 * RTOL, atol=10 * ATOL, reduce_scale=True)


@pytest.mark.parametrize("fin,H,F", [(8, 64, 16), (8, 1, 1024), (1024, 2, 8), (4, 64, 4)])
def test_largest_supported_shapes(fin, H, F):
    """heads*f = 1024 (the widest row the kernels take), 64 heads, a wide input."""
    from gpu_harness import run_gat
    print(f"gat: largest shapes fin={fin} H={H} F={F}", flush=True)
    rng = np.random.default_rng(fin + 7 * H + 13 * F)
    indptr, indices = random_graph(rng, 200, 1500, self_loops=True, duplicates=True)
    c = synth(rng, indptr, indices, fin, H, F)
    fwd, bwd = oracle_all(c)
    compare(c, run_gat(c), fwd, bwd)


def test_many_vertices_few_edges_on_the_blocked_path():
    """More vertices than one column block holds, almost all (row, block) segments empty,
    rows without any edge in the first block, whole rows without edges."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    print("gat: 70000 vertices, sparse", flush=True)
    rng = np.random.default_rng(4242)
    n = 70_000
    src = rng.integers(0, n, size=150_000)
    dst = rng.integers(0, n // 2, size=150_000)            # the upper half has no in-edges
    order = np.lexsort((src, dst))
    src, dst = src[order], dst[order]
    indptr = np.zeros(n + 1, dtype=np.int32)
    np.add.at(indptr, dst + 1, 1)
    indptr = np.cumsum(indptr).astype(np.int32)
    indices = src.astype(np.int32)
    c = synth(rng, indptr, indices, 6, 4, 32)
    fwd, bwd = oracle_all(c)
    g = pk.Graph(dev(indptr), dev(indices))
    assert g.blocked(0)[0] == -(-n // 12288)
    res = run_gat(c, graph=g)
    compare(c, res, fwd, bwd)
    assert (res["out"][n // 2:] == 0).all()
    compare(c, run_gat(c, graph=g, stash=False), fwd, bwd)
    g.close()


@pytest.mark.parametrize("stash", [True, False])
@pytest.mark.parametrize("name", ["gat_c2", "gat_c4_mid"])
def test_fusion_with_stashing_arm(name, stash):
    """The per-edge softmax values stored after the forward pass (CSC order, signed by the raw
    score) equal the oracle's materialised M2, and the backward pass that reads them back gives
    the oracle's gradients."""
    from gpu_harness import assert_close, run_gat
    print(f"gat: fusion with stashing {name} vertex-stash={stash}", flush=True)
    c = make(name)
    fwd, bwd = oracle_all(c)
    res = run_gat(c, stash=stash, alpha_stash=True)
    # CSC order: edges by (source, CSR position)
    order = np.lexsort((np.arange(c["nnz"]), c["indices"]))
    ref = (fwd["M2"] * np.where(fwd["M0"] > 0, 1.0, -1.0))[order]
    got = res.pop("alpha_t")[:c["nnz"]]
    near_kink = np.abs(fwd["M0"][order]) < 1e-5
    assert_close("alpha_t", np.where(near_kink, ref, got), ref)
    compare(c, res, fwd, bwd)


def test_fusion_with_stashing_arm_on_a_column_blocked_graph_and_bad_arguments():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, run_gat
    rng = np.random.default_rng(321)
    indptr, indices = random_graph(rng, 1500, 30000, self_loops=False, duplicates=True)
    c = synth(rng, indptr, indices, 24, 4, 64)
    fwd, bwd = oracle_all(c)
    from gpu_harness import assert_close
    n, nnz, H = c["n"], c["nnz"], c["heads"]
    pk.gnn_config_set("block_cols", 256)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        assert pk.gnn_gat_stash_layout(g, 4, 64) == 1    # the stash is laid out for the column-blocked kernel
        res = run_gat(c, graph=g, alpha_stash=True)      # forward and stashed backward both column-blocked
    finally:
        pk.gnn_config_set("block_cols", 12288)
    # layout 1: [h][q], q = position in the source side's blocked list = the CSC entries (source,
    # CSR position) stable-sorted by (block of the destination, source)
    csc = np.lexsort((np.arange(nnz), c["indices"]))
    dst = np.repeat(np.arange(n), np.diff(c["indptr"]))
    key = (dst[csc] // 256).astype(np.int64) * n + c["indices"][csc]
    order = csc[np.argsort(key, kind="stable")]
    ref = (fwd["M2"] * np.where(fwd["M0"] > 0, 1.0, -1.0))[order].T
    got = res.pop("alpha_t").reshape(-1)[:H * nnz].reshape(H, nnz)
    near_kink = np.abs(fwd["M0"][order]).T < 1e-5
    assert_close("alpha_b", np.where(near_kink, ref, got), ref)
    compare(c, res, fwd, bwd)
    a = empty((4, 4))
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_gat_bwd_stashed(g, 24, 4, 64, 0.2, a, a, a, a, a, a, a, a, a, a, None, None, None, a, None, a, a, a,
                               None)
    assert e.value.status == 1
    g.close()


def test_sparse_graph_spanning_blocks_takes_the_single_launch_kernels():
    """Default rule: column blocking is used from 16 edges per (row, block) on average."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    rng = np.random.default_rng(77)
    n = 1500
    indptr, indices = random_graph(rng, n, 30000, self_loops=False, duplicates=True)   # 20 edges per row
    c = synth(rng, indptr, indices, 16, 4, 64)

    def kernels_used(min_edges, block_cols):
        pk.gnn_config_set("blocked_min_edges", min_edges)
        pk.gnn_config_set("block_cols", block_cols)
        try:
            g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
            pk.gnn_prof_reset()
            pk.gnn_prof_enable(True)
            run_gat(c, graph=g)
            names = set(pk.gnn_prof_report())
            pk.gnn_prof_enable(False)
            g.close()
        finally:
            pk.gnn_config_set("block_cols", 12288)
            pk.gnn_config_set("blocked_min_edges", 0)
        return names
    assert "gat_head_major" not in kernels_used(16, 256)      # 6 blocks: 3.3 edges per (row, block)
    assert "gat_head_major" not in kernels_used(16, 1024)     # 2 blocks: 10 per (row, block)
    assert "gat_head_major" in kernels_used(8, 1024)          # the same graph with the bar at 8


@pytest.mark.parametrize("resident", [1, 0])
@pytest.mark.parametrize("H,F", [(4, 64), (2, 64), (2, 128), (1, 512), (8, 64), (1, 128)])
def test_fp16_gather_storage(H, F, resident):
    """gather_precision = 1: the column-blocked kernels (the persistent launch, or a launch per block with
    resident = 0) gather from an fp16 copy of z / gout and sum in fp32.  Every gathered element carries a relative rounding error of up to 2^-11; in the backward
    pass these errors enter dot products over f columns, so the worst entry of a gradient may be off by
    several 1e-3 of the tensor's rms.  The results are compared with the oracle at 1.5e-2 of the rms
    (worst entry) and 2e-3 (rms of the error), not at the 1e-4 contract; the fp32 path on the same
    inputs must be at least as close."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    print(f"gat: fp16 gather storage H={H} F={F} resident={resident}", flush=True)
    rng = np.random.default_rng(4000 + H * F)
    indptr, indices = random_graph(rng, 1200, 30000, self_loops=True, duplicates=True)
    c = synth(rng, indptr, indices, 20, H, F)
    fwd, bwd = oracle_all(c)
    pk.gnn_config_set("block_cols", 256)
    pk.gnn_config_set("resident_sums", resident)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        ref32 = run_gat(c, graph=g)
        pk.gnn_config_set("gather_precision", 1)
        try:
            res16 = run_gat(c, graph=g)
        finally:
            pk.gnn_config_set("gather_precision", 0)
        g.close()
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("resident_sums", 1)
    compare(c, ref32, fwd, bwd)                       # the default path keeps the contract

    def rel(a, b):
        b = np.asarray(b, dtype=np.float64).reshape(np.shape(a))
        scale = max(np.sqrt(np.mean(b * b)), 1e-30)
        return float(np.abs(a - b).max() / scale), float(np.sqrt(np.mean((a - b) ** 2)) / scale)
    for key, ref in (("out", fwd["out"]), ("gx", bwd["gx"]), ("gw", bwd["gw"]), ("ga_l", bwd["ga_l"]),
                     ("ga_r", bwd["ga_r"])):
        (w16, r16), (w32, _) = rel(res16[key], ref), rel(ref32[key], ref)
        print(f"  {key}: fp16 worst {w16:.1e} rms {r16:.1e}; fp32 worst {w32:.1e}", flush=True)
        assert w16 < 1.5e-2 and r16 < 2e-3, f"{key}: fp16 gather error worst {w16:.2e} rms {r16:.2e}"
        assert w32 <= w16 + 1e-7 or w16 < 1e-6, f"{key}: fp32 {w32:.2e} vs fp16 {w16:.2e}"
    assert np.array_equal(res16["m"], ref32["m"]) and np.array_equal(res16["el"], ref32["el"])   # scores are fp32
    # the copy was used, by the forward pass and by the source-side backward
    assert not np.array_equal(res16["out"], ref32["out"])
    assert not np.array_equal(res16["gx"], ref32["gx"])


def test_fp16_gather_storage_leaves_uncovered_shapes_in_fp32():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    rng = np.random.default_rng(4100)
    indptr, indices = random_graph(rng, 900, 20000, self_loops=True, duplicates=True)
    c = synth(rng, indptr, indices, 12, 4, 32)          # 64-column slices would span two heads
    pk.gnn_config_set("block_cols", 256)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        a = run_gat(c, graph=g)
        pk.gnn_config_set("gather_precision", 1)
        try:
            b = run_gat(c, graph=g)
        finally:
            pk.gnn_config_set("gather_precision", 0)
        g.close()
    finally:
        pk.gnn_config_set("block_cols", 12288)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    with pytest.raises(pk.GnnError):
        pk.gnn_config_set("gather_precision", 2)


@pytest.mark.parametrize("resident", [1, 0])
@pytest.mark.parametrize("H,F", [(4, 64), (1, 128)])
def test_column_blocked_path_with_64_bit_row_offsets(H, F, resident):
    """Gathered matrices of 4 GB and more are addressed with 64-bit offsets; the configuration key
    "wide_offsets" takes that path on a graph small enough for the oracle."""
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, run_gat
    print(f"gat: blocked path, 64-bit row offsets H={H} F={F}", flush=True)
    rng = np.random.default_rng(77 + H)
    indptr, indices = random_graph(rng, 1500, 30000, self_loops=False, duplicates=True)
    c = synth(rng, indptr, indices, 24, H, F)
    fwd, bwd = oracle_all(c)
    pk.gnn_config_set("block_cols", 300)
    pk.gnn_config_set("wide_offsets", 1)
    pk.gnn_config_set("resident_sums", resident)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
        res = run_gat(c, graph=g)
        g.close()
    finally:
        pk.gnn_config_set("block_cols", 12288)
        pk.gnn_config_set("wide_offsets", 0)
        pk.gnn_config_set("resident_sums", 1)
    compare(c, res, fwd, bwd)

