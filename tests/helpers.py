"""Small helpers shared by the CPU tests: tiny graph builders and finite differences."""
import numpy as np


def tiny_graph(n, edges):
    """edges: list of (src, dst), duplicates allowed -> CSR by destination, stable order."""
    edges = sorted(edges, key=lambda e: (e[1], e[0]))
    indptr = np.zeros(n + 1, dtype=np.int32)
    for _, d in edges:
        indptr[d + 1] += 1
    indptr = np.cumsum(indptr).astype(np.int32)
    indices = np.array([s for s, _ in edges], dtype=np.int32).reshape(-1)
    return indptr, indices


def random_graph(rng, n, m, self_loops=True, duplicates=False):
    src = rng.integers(0, n, size=m)
    dst = rng.integers(0, n, size=m)
    edges = list(zip(src.tolist(), dst.tolist()))
    if not duplicates:
        edges = list(dict.fromkeys(edges))
    if self_loops:
        edges += [(v, v) for v in range(n) if (v, v) not in set(edges)]
    return tiny_graph(n, edges)


def finite_difference(fun, theta, h=1e-6, max_entries=None, rng=None):
    """Central differences of the scalar fun at theta (fp64), entry by entry."""
    theta = np.array(theta, dtype=np.float64)
    flat = theta.reshape(-1)
    idx = np.arange(flat.size)
    if max_entries is not None and flat.size > max_entries:
        idx = rng.choice(flat.size, size=max_entries, replace=False)
    g = np.zeros(idx.size)
    for j, i in enumerate(idx):
        old = flat[i]
        flat[i] = old + h
        fp = fun(theta)
        flat[i] = old - h
        fm = fun(theta)
        flat[i] = old
        g[j] = (fp - fm) / (2 * h)
    return idx, g
