"""k-nearest-neighbour graph construction: HIP path against the oracle, bit for bit."""
import numpy as np
import pytest

from oracle import knn as ok

pytestmark = pytest.mark.gpu


def build(coords, clouds, points, k):
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    n, dim = clouds * points, coords.shape[1]
    indptr = torch.empty(n + 1, dtype=torch.int32, device="cuda:0")
    indices = torch.empty(n * k, dtype=torch.int32, device="cuda:0")
    pk.gnn_knn_graph(clouds, points, dim, k, dev(coords), indptr, indices)
    torch.cuda.synchronize()
    return indptr.cpu().numpy(), indices.cpu().numpy()


@pytest.mark.parametrize("clouds,points,dim,k", [(1, 1, 3, 1), (3, 50, 3, 7), (2, 64, 3, 64), (5, 333, 3, 20),
                                                 (4, 1024, 3, 20), (2, 1024, 3, 40), (2, 200, 8, 9),
                                                 (1, 2048, 3, 33), (3, 130, 1, 5), (2, 200, 3, 150), (1, 65, 2, 65),
                                                 (70, 100, 3, 10)])
def test_matches_the_oracle_exactly(clouds, points, dim, k):
    print(f"knn: clouds={clouds} points={points} dim={dim} k={k}", flush=True)
    rng = np.random.default_rng(clouds * 1000 + points + k)
    coords = rng.random((clouds * points, dim), dtype=np.float32)
    ip, ix = build(coords, clouds, points, k)
    rp, rx = ok.knn_graph(coords, clouds, points, k)
    assert (ip == rp).all()
    assert (ix == rx).all()


def test_ties_go_to_the_lower_index():
    # points on an integer grid: many exactly equal distances
    rng = np.random.default_rng(5)
    coords = rng.integers(0, 4, size=(2 * 300, 3)).astype(np.float32)
    ip, ix = build(coords, 2, 300, 12)
    rp, rx = ok.knn_graph(coords, 2, 300, 12)
    assert (ix == rx).all()
    same = np.zeros((64, 2), dtype=np.float32)      # all points equal: neighbours 0..k-1
    _, ix = build(same, 1, 64, 5)
    assert (ix.reshape(64, 5) == np.arange(5)).all()


def test_the_graph_feeds_the_edgeconv_layer():
    """The constructed CSR is accepted by gnn_graph_create and gives the layer's oracle result."""
    import paper_2110_09524_amd as pk
    from gpu_harness import run_edgeconv
    from oracle import edgeconv as oe
    from workloads import make
    c = dict(make("ec_c3_mid"))
    clouds, points = 3, 500
    ip, ix = build(c["coords"], clouds, points, 20)
    rp, rx = ok.knn_graph(c["coords"], clouds, points, 20)
    assert (ix == rx).all()
    c["indptr"], c["indices"] = ip, ix
    res = run_edgeconv(c, backward=False)
    ref = oe.edgeconv_forward(ip, ix, c["x"], c["theta"], c["phi"])
    np.testing.assert_allclose(res["out"], ref["out"], rtol=1e-4, atol=1e-5)


def test_bad_arguments_raise():
    import torch
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    coords = dev(np.zeros((10, 3), dtype=np.float32))
    ip = torch.empty(11, dtype=torch.int32, device="cuda:0")
    ix = torch.empty(10 * 11, dtype=torch.int32, device="cuda:0")
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_knn_graph(1, 10, 3, 11, coords, ip, ix)        # k above the cloud size
    assert e.value.status == 4
    with pytest.raises(pk.GnnError) as e:
        pk.gnn_knn_graph(1, 10, 3, 0, coords, ip, ix)
    assert e.value.status == 1
