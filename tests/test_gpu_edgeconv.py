"""EdgeConv layer: HIP path against the fp64 oracle."""
import numpy as np
import pytest

from oracle import edgeconv as oe
from helpers import random_graph, tiny_graph
from workloads import make

pytestmark = pytest.mark.gpu

TIE_TOL = 1e-4     # messages closer than this to the row maximum may swap winners in fp32


def check(c):
    """Arg-max is unique only away from near-ties.  Entries (v, j) whose runner-up lies
    within TIE_TOL of the maximum are 'ambiguous': there the GPU may pick any edge
    whose oracle message is within TIE_TOL of the maximum, and the upstream gradient
    is zeroed for both sides so the choice cannot leak into the gradient comparison."""
    from gpu_harness import assert_close, run_edgeconv
    ip, ix = c["indptr"], c["indices"]
    fwd = oe.edgeconv_forward(ip, ix, c["x"], c["theta"], c["phi"])
    amb = oe.near_tie_mask(ip, fwd, TIE_TOL)
    gout = np.where(amb, 0.0, c["gout"]).astype(np.float32)
    bwd = oe.edgeconv_backward(ip, ix, c["x"], c["theta"], c["phi"], gout, fwd)
    res = run_edgeconv(c, gout=gout)
    n, fout = c["n"], c["fout"]
    P = c["x"].astype(np.float64) @ c["theta"].astype(np.float64)
    Q = c["x"].astype(np.float64) @ (c["phi"].astype(np.float64) - c["theta"].astype(np.float64))
    assert_close("pq", res["pq"], np.concatenate([P, Q], axis=1))
    assert_close("out", res["out"], fwd["out"])
    arg = res["argmax"].astype(np.int64)
    clear = ~amb
    assert np.array_equal(arg[clear], fwd["argmax"][clear]), "arg-max differs away from ties"
    # ambiguous entries: the pick must be an in-edge of the row and near-maximal
    vs, js = np.nonzero(amb)
    for v, j in zip(vs, js):
        e = arg[v, j]
        assert ip[v] <= e < ip[v + 1]
        assert fwd["E_TP"][e, j] >= fwd["out"][v, j] - TIE_TOL
    assert_close("gx", res["gx"], bwd["gx"])
    assert_close("gtheta", res["gtheta"], bwd["gtheta"], reduce_scale=True)
    assert_close("gphi", res["gphi"], bwd["gphi"], reduce_scale=True)
    return int(amb.sum())


def synth(rng, indptr, indices, fin, fout):
    n = len(indptr) - 1
    return dict(n=n, fin=fin, fout=fout, indptr=indptr, indices=indices,
                x=rng.standard_normal((n, fin)).astype(np.float32),
                theta=(rng.standard_normal((fin, fout)) * 0.4).astype(np.float32),
                phi=(rng.standard_normal((fin, fout)) * 0.4).astype(np.float32),
                gout=rng.standard_normal((n, fout)).astype(np.float32))


def test_c3_mid():
    print("edgeconv: ec_c3_mid", flush=True)
    check(make("ec_c3_mid"))


def test_k40_mid():
    print("edgeconv: ec_k40_mid", flush=True)
    check(make("ec_k40_mid"))


def test_c3_full():
    print("edgeconv: ec_c3", flush=True)
    check(make("ec_c3"))


@pytest.mark.parametrize("fin,fout", [(3, 4), (9, 20), (64, 64), (17, 128), (8, 512)])
def test_shapes(fin, fout):
    print(f"edgeconv: shape {fin}->{fout}", flush=True)
    rng = np.random.default_rng(fin + fout)
    indptr, indices = random_graph(rng, 301, 2500, self_loops=True, duplicates=False)
    check(synth(rng, indptr, indices, fin, fout))


def test_graph_without_edges():
    from gpu_harness import run_edgeconv
    print("edgeconv: no edges", flush=True)
    rng = np.random.default_rng(63)
    n = 29
    c = synth(rng, np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32), 6, 8)
    res = run_edgeconv(c, backward=False)
    assert (res["argmax"] == -1).all() and (res["out"] == 0).all()
    check(c)


def test_duplicate_edges_empty_rows_and_hub():
    from gpu_harness import run_edgeconv
    print("edgeconv: duplicates + empty rows + hub", flush=True)
    rng = np.random.default_rng(9)
    n = 400
    edges = [(u, 0) for u in range(n)] + [(3, 5), (3, 5), (7, 5), (7, 5)]
    edges += [(int(rng.integers(0, n)), int(v)) for v in range(20, n) for _ in range(3)]
    indptr, indices = tiny_graph(n, edges)
    c = synth(rng, indptr, indices, 6, 8)
    # exact ties between duplicate edges: the earliest CSR position must win on both sides
    fwd = oe.edgeconv_forward(indptr, indices, c["x"], c["theta"], c["phi"])
    res = run_edgeconv(c, backward=False)
    row5 = slice(indptr[5], indptr[6])
    assert list(indices[row5]) == [3, 3, 7, 7]
    assert set(res["argmax"][5].tolist()) <= {int(indptr[5]), int(indptr[5]) + 2}
    assert (res["argmax"][1] == -1).all() and (res["out"][1] == 0).all()
    check(c)
