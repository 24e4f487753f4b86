"""The forward and backward entry points only enqueue kernels on the caller's stream
(no allocation, no synchronisation, no memset), so a caller may record them into a HIP
graph.  A captured GAT step is replayed several times, with the program's own eager work
and synchronisations in between and with new input values each time; every replay must
reproduce the eager result of the same inputs bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,block_cols", [("gat_c2", None), ("gat_c4_mid", None), ("gat_c4_mid", 1024)])
def test_captured_gat_step_replays_exactly(name, block_cols):
    """block_cols = 1024 puts the 6000-vertex graph on the column-blocked path: the persistent
    kernels (and the small kernel that zeroes their step counters) are what the graph records."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    from workloads import make
    print(f"graph capture: {name} block_cols={block_cols}", flush=True)
    c = make(name)
    n, fin, H, F = c["n"], c["fin"], c["heads"], c["f"]
    HF = H * F
    if block_cols:
        pk.gnn_config_set("block_cols", block_cols)
    try:
        g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    finally:
        pk.gnn_config_set("block_cols", 12288)
    assert not block_cols or g.blocked(0)[0] > 1
    x, w, a_l, a_r, gout = (dev(c[k]) for k in ("x", "w", "a_l", "a_r", "gout"))
    bufs = lambda: dict(z=empty((n, HF)), out=empty((n, HF)), t=empty((n, HF)), el=empty((n, H)),
                        er=empty((n, H)), m=empty((n, H)), d=empty((n, H)), sg=empty((n, H)),
                        gx=empty((n, fin)), gw=empty((fin, HF)), ga_l=empty((H, F)), ga_r=empty((H, F)))
    ws = workspace(pk.gnn_gat_workspace_bytes(g, fin, H, F))

    def step(b):
        pk.gnn_gat_fwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, b["z"], b["el"], b["er"], b["m"], b["d"],
                       b["out"], b["t"], b["sg"], ws)
        pk.gnn_gat_bwd(g, fin, H, F, c["slope"], x, w, a_l, a_r, b["z"], b["el"], b["er"], b["m"], b["d"],
                       b["out"], b["t"], b["sg"], gout, b["gx"], b["gw"], b["ga_l"], b["ga_r"], ws)

    captured = bufs()
    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(captured)                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(captured)

    rng = np.random.default_rng(17)
    for replay in range(3):
        # new values in the same input buffers, by the program's own eager work
        x.copy_(dev(rng.standard_normal(c["x"].shape).astype(np.float32)))
        gout.mul_(-0.5)
        torch.cuda.synchronize()
        eager = bufs()
        step(eager)
        torch.cuda.synchronize()
        for t in captured.values():     # poison: the replay must rewrite every output
            t.fill_(float("nan"))
        ws.fill_(0xFF)
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(eager[k], captured[k]), f"replay {replay}: {k} differs from the eager result"
    g.close()


def test_captured_monet_step_replays_exactly():
    """The same for the MoNet layer with the projection fused in (a two-stage fixed-order reduction of the
    parameter gradients sits inside the captured backward call)."""
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev, empty, workspace
    from workloads import make
    print("graph capture: monet_c5", flush=True)
    c = make("monet_c5")
    n, fin, F, K, R = c["n"], c["fin"], c["fout"], c["k"], c["r"]
    g = pk.Graph(dev(c["indptr"]), dev(c["indices"]))
    x, w_fc, cc, P, pb, mu, isg, gout = (dev(c[k]) for k in ("x", "w_fc", "c", "proj_w", "proj_b", "mu", "inv_sigma",
                                                              "gout"))
    bufs = lambda: dict(hk=empty((n, K * F)), out=empty((n, F)), gx=empty((n, fin)), gw_fc=empty((fin, K * F)),
                        gmu=empty((K, R)), gis=empty((K, R)), gP=empty((R, 2)), gpb=empty((R,)))
    ws = workspace(pk.gnn_monet_workspace_bytes(g, fin, F, K))

    def step(b):
        pk.gnn_monet_fwd(g, fin, F, K, R, x, w_fc, cc, P, pb, mu, isg, b["hk"], b["out"])
        pk.gnn_monet_bwd(g, fin, F, K, R, x, w_fc, cc, P, pb, mu, isg, b["hk"], gout, b["gx"], b["gw_fc"], b["gmu"],
                         b["gis"], b["gP"], b["gpb"], ws)

    captured = bufs()
    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(captured)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(captured)
    rng = np.random.default_rng(23)
    for replay in range(3):
        x.copy_(dev(rng.standard_normal(c["x"].shape).astype(np.float32)))
        P.mul_(-0.7)
        torch.cuda.synchronize()
        eager = bufs()
        step(eager)
        torch.cuda.synchronize()
        for t in captured.values():
            t.fill_(float("nan"))
        ws.fill_(0xFF)
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            assert torch.equal(eager[k], captured[k]), f"replay {replay}: {k} differs from the eager result"
    g.close()
