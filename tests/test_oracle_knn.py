"""Pins of the k-nearest-neighbour oracle: cases with a known answer, brute force, the fp64 generator."""
import numpy as np

from oracle import knn as ok
from workloads import graphs


def test_points_on_a_line_have_known_neighbours_and_ties_go_to_the_lower_index():
    P = 9
    coords = np.arange(P, dtype=np.float32)[:, None]
    indptr, indices = ok.knn_graph(coords, 1, P, 3)
    nb = indices.reshape(P, 3)
    assert (indptr == np.arange(P + 1) * 3).all()
    assert nb[0].tolist() == [0, 1, 2] and nb[P - 1].tolist() == [P - 3, P - 2, P - 1]
    for i in range(1, P - 1):
        assert nb[i].tolist() == [i - 1, i, i + 1]
    # k = 2: the point itself, then i-1 and i+1 tie and the lower index wins
    nb2 = ok.knn_graph(coords, 1, P, 2)[1].reshape(P, 2)
    assert nb2[0].tolist() == [0, 1]
    for i in range(1, P):
        assert nb2[i].tolist() == [i - 1, i]


def test_duplicate_points_tie_to_the_lower_index():
    coords = np.zeros((5, 3), dtype=np.float32)
    nb = ok.knn_graph(coords, 1, 5, 2)[1].reshape(5, 2)
    assert (nb == np.array([0, 1])).all()


def test_against_brute_force_in_python_loops():
    rng = np.random.default_rng(7)
    clouds, P, D, k = 2, 23, 3, 5
    coords = rng.random((clouds * P, D), dtype=np.float32)
    _, indices = ok.knn_graph(coords, clouds, P, k)
    for b in range(clouds):
        for i in range(P):
            cand = []
            for j in range(P):
                acc = np.float32(0)
                for d in range(D):
                    diff = np.float32(coords[b * P + i, d] - coords[b * P + j, d])
                    acc = np.float32(acc + np.float32(diff * diff))
                cand.append((float(acc), j))
            want = sorted(j + b * P for _, j in sorted(cand)[:k])
            assert indices[(b * P + i) * k:(b * P + i + 1) * k].tolist() == want


def test_clouds_do_not_mix_and_every_point_is_its_own_neighbour():
    rng = np.random.default_rng(8)
    clouds, P, k = 3, 40, 6
    coords = rng.random((clouds * P, 3), dtype=np.float32)
    indptr, indices = ok.knn_graph(coords, clouds, P, k)
    nb = indices.reshape(clouds * P, k)
    own = np.arange(clouds * P)
    assert ((nb // P) == (own // P)[:, None]).all()
    assert (nb == own[:, None]).any(axis=1).all()
    assert (np.diff(nb, axis=1) > 0).all()


def test_agrees_with_the_float64_generator_except_at_rounding_ties():
    indptr, indices, coords = graphs.knn_point_clouds(2, 300, 8, 1234)
    ip, ix = ok.knn_graph(coords, 2, 300, 8)
    assert (ip == indptr).all()
    same = (ix.reshape(-1, 8) == indices.reshape(-1, 8)).all(axis=1)
    assert same.mean() > 0.995
    # where they differ the k-th distances agree to float32 rounding
    c64 = coords.astype(np.float64)
    for v in np.flatnonzero(~same):
        da = np.sort(((c64[ix.reshape(-1, 8)[v]] - c64[v]) ** 2).sum(axis=1))
        db = np.sort(((c64[indices.reshape(-1, 8)[v]] - c64[v]) ** 2).sum(axis=1))
        np.testing.assert_allclose(da, db, rtol=1e-5, atol=1e-7)
