"""MoNet / GMMConv layer: HIP path against the fp64 oracle."""
import numpy as np
import pytest

from oracle import gmm as om
from helpers import random_graph, tiny_graph
from workloads import make

pytestmark = pytest.mark.gpu


def check(c):
    from gpu_harness import assert_close, run_gmm
    args = (c["indptr"], c["indices"], c["x"], c["w_fc"], c["c"], c["mu"], c["inv_sigma"])
    fwd = om.gmm_forward(*args)
    bwd = om.gmm_backward(*args, c["gout"], fwd)
    res = run_gmm(c)
    n = c["n"]
    assert_close("hk", res["hk"], fwd["Hk"].reshape(n, -1))
    assert_close("out", res["out"], fwd["out"])
    assert_close("gx", res["gx"], bwd["gx"], row_scale=True)
    assert_close("gw_fc", res["gw_fc"], bwd["gw_fc"], reduce_scale=True)
    assert_close("gmu", res["gmu"], bwd["gmu"], reduce_scale=True)
    assert_close("ginv_sigma", res["ginv_sigma"], bwd["ginv_sigma"], reduce_scale=True)


def synth(rng, indptr, indices, fin, fout, K):
    n = len(indptr) - 1
    deg = np.diff(indptr)
    return dict(n=n, fin=fin, fout=fout, k=K, indptr=indptr, indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                w_fc=(rng.standard_normal((fin, K * fout)) * 0.3).astype(np.float32),
                c=(1.0 / np.sqrt(np.maximum(deg, 1))).astype(np.float32),
                mu=(rng.standard_normal((K, 2)) * 0.3).astype(np.float32),
                inv_sigma=(0.5 + rng.random((K, 2))).astype(np.float32),
                gout=rng.standard_normal((n, fout)).astype(np.float32))


@pytest.mark.parametrize("name", ["gmm_c5_mid", "gmm_c5"])
def test_workloads(name):
    print("gmm:", name, flush=True)
    check(make(name))


@pytest.mark.parametrize("fin,fout,K", [(6, 4, 8), (3, 16, 5), (5, 16, 1), (9, 16, 4), (64, 64, 3), (12, 32, 8), (7, 256, 5),
                                        (20, 24, 2)])
def test_shapes(fin, fout, K):
    print(f"gmm: shape {fin}->{fout} K={K}", flush=True)
    rng = np.random.default_rng(fin + fout + K)
    indptr, indices = random_graph(rng, 263, 2600, self_loops=True, duplicates=True)
    check(synth(rng, indptr, indices, fin, fout, K))


def test_graph_without_edges():
    print("gmm: no edges", flush=True)
    rng = np.random.default_rng(62)
    n = 41
    check(synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 16, 3))


def test_empty_rows_and_hub():
    print("gmm: empty rows + hub", flush=True)
    rng = np.random.default_rng(3)
    n = 500
    edges = [(u, 0) for u in range(n)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(10, n) for _ in range(2)]
    indptr, indices = tiny_graph(n, edges)
    check(synth(rng, indptr, indices, 10, 32, 3))
