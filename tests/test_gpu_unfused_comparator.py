"""The bench-only one-operator-per-kernel comparator computes the same layer: its
outputs are checked against the oracle so that the ratios bench.py reports compare
like with like."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_comparator_matches_the_oracle():
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import assert_close, dev
    from oracle import gat as og
    from unfused_baseline.compare import UnfusedGat
    from workloads import make
    print("unfused comparator: gat_c4_mid", flush=True)
    c = make("gat_c4_mid")
    n, H, F = c["n"], c["heads"], c["f"]
    fwd = og.gat_forward(c["indptr"], c["indices"], c["x"], c["w"], c["a_l"], c["a_r"], c["slope"])
    bwd = og.gat_backward(c["indptr"], c["indices"], c["x"], c["w"], c["a_l"], c["a_r"], c["slope"],
                          c["gout"], fwd)
    indptr, indices = dev(c["indptr"]), dev(c["indices"])
    g = pk.Graph(indptr, indices)
    Ht = fwd["Ht"]
    z = dev(Ht.reshape(n, H * F).astype(np.float32))
    el = dev(np.einsum("nhf,hf->nh", Ht, c["a_l"].astype(np.float64)).astype(np.float32))
    er = dev(np.einsum("nhf,hf->nh", Ht, c["a_r"].astype(np.float64)).astype(np.float32))
    u = UnfusedGat(c, g, indptr, indices)
    u.fwd(z, el, er)
    u.bwd(z, dev(c["gout"]), dev(c["a_l"]), dev(c["a_r"]))
    torch.cuda.synchronize()
    assert_close("out", u.out.view(n, -1).cpu().numpy(), fwd["out"])
    assert_close("alpha", u.M2.view(-1, H).cpu().numpy(), fwd["M2"])
    assert_close("dz", u.dz.view(n, -1).cpu().numpy(), bwd["dHt"])


def test_edgeconv_comparator_matches_the_oracle():
    import torch
    from gpu_harness import assert_close, dev
    from oracle import edgeconv as oe
    from unfused_baseline.compare import UnfusedEdgeConv
    from workloads import make
    print("unfused comparator: ec_c3_mid", flush=True)
    c = make("ec_c3_mid")
    fwd = oe.edgeconv_forward(c["indptr"], c["indices"], c["x"], c["theta"], c["phi"])
    u = UnfusedEdgeConv(c, dev(c["indptr"]), dev(c["indices"]))
    u.fwd(dev(c["x"]), dev(c["theta"]), dev(c["phi"]))
    torch.cuda.synchronize()
    assert_close("out", u.out.cpu().numpy(), fwd["out"])
    # the winner the comparator stored reaches the maximum (near-ties may pick another edge)
    am = u.argmax.cpu().numpy().astype(np.int64)
    E2 = u.E2.cpu().numpy()
    cols = np.broadcast_to(np.arange(c["fout"]), am.shape)
    assert_close("value at argmax", E2[am, cols], fwd["out"])


def test_gmm_comparator_matches_the_oracle():
    import torch
    from gpu_harness import assert_close, dev
    from oracle import gmm as om
    from unfused_baseline.compare import UnfusedGmm
    from workloads import make
    print("unfused comparator: gmm_c5_mid", flush=True)
    c = make("gmm_c5_mid")
    fwd = om.gmm_forward(c["indptr"], c["indices"], c["x"], c["w_fc"], c["c"], c["mu"], c["inv_sigma"])
    hk = (c["x"].astype(np.float64) @ c["w_fc"].astype(np.float64)).astype(np.float32)
    u = UnfusedGmm(c, dev(c["indptr"]), dev(c["indices"]))
    u.fwd(dev(c["c"]), dev(c["mu"]), dev(c["inv_sigma"]), dev(hk))
    torch.cuda.synchronize()
    assert_close("out", u.out.cpu().numpy(), fwd["out"])
