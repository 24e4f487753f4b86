"""gnn_gat_bwd_noalloc (scratch in a device array built into the library) against gnn_gat_bwd
(caller's workspace): two calls in a row through the C ABI, the second on a smaller input, and
the size limit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _both(c, stash):
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    n, fin, H, F = c["n"], c["fin"], c["heads"], c["f"]
    HF = H * F
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    need = pk.gnn_gat_workspace_bytes(g, fin, H, F)
    assert need <= pk.NOALLOC_SCRATCH_BYTES
    x, w, a_l, a_r, gout = (dev(c[k]) for k in ("x", "w", "a_l", "a_r", "gout"))
    z, out = empty((n, HF)), empty((n, HF))
    el, er, m, d = (empty((n, H)) for _ in range(4))
    t = empty((n, HF)) if stash else None
    sg = empty((n, H)) if stash else None
    ws = workspace(need)
    pk.gnn_gat_fwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg, ws)
    res = []
    for noalloc in (False, True):
        gx, gw, ga_l, ga_r = empty((n, fin)), empty((fin, HF)), empty((H, F)), empty((H, F))
        args = (g, fin, H, F, c["slope"], x, w, a_l, a_r, z, el, er, m, d, out, t, sg, gout, gx, gw, ga_l, ga_r)
        if noalloc:
            pk.gnn_gat_bwd_noalloc(*args)
        else:
            ws.fill_(0xFF)
            pk.gnn_gat_bwd(*args, ws)
        torch.cuda.synchronize()
        res.append({k: v.cpu().numpy() for k, v in dict(gx=gx, gw=gw, ga_l=ga_l, ga_r=ga_r).items()})
    g.close()
    return res


def test_noalloc_backward_matches_the_workspace_backward_twice_in_a_row():
    from gpu_harness import assert_close
    from workloads import make
    big, small = make("gat_c2"), make("gat_c1")
    assert small["n"] < big["n"]
    for c, stash in ((big, True), (small, False)):      # the second call: smaller input, other path
        print(f"noalloc: n = {c['n']}, stash = {stash}", flush=True)
        ref, got = _both(c, stash)
        for k in ("gx", "gw", "ga_l", "ga_r"):
            assert_close(k, got[k], ref[k], reduce_scale=k != "gx")
            assert np.array_equal(got[k], ref[k]), f"{k}: same kernels, same order: expected identical bits"


def test_noalloc_backward_on_the_column_blocked_kernels():
    import paper_2110_09524_amd as pk
    from workloads import make
    c = make("gat_c4_mid")
    pk.gnn_config_set("block_cols", 1024)
    try:
        ref, got = _both(c, True)
    finally:
        pk.gnn_config_set("block_cols", 12288)
    for k in ("gx", "gw", "ga_l", "ga_r"):
        assert np.array_equal(got[k], ref[k]), k


def test_noalloc_backward_rejects_what_its_array_cannot_hold():
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty
    n = 300_000                                          # dz alone would be 307 MB
    indptr = torch.arange(n + 1, dtype=torch.int32, device="cuda")
    indices = torch.arange(n, dtype=torch.int32, device="cuda")
    g = pk.Graph(indptr, indices)
    assert pk.gnn_gat_workspace_bytes(g, 8, 4, 64) > pk.NOALLOC_SCRATCH_BYTES
    a = empty((4, 64))
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_gat_bwd_noalloc(g, 8, 4, 64, 0.2, a, a, a, a, a, a, a, a, a, a, None, None, a, None, a, a, a)
    assert e.value.status == 3 and "scratch" in str(e.value)
    g.close()
