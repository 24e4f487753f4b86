"""Sec. 6 / Sec. 7.3: what the layer calls make the caller keep or lend is O(|V|), never O(|E|).
The saved tensors are vertex-shaped by their declarations; the workspace sizes the library asks
for must not grow when only the number of edges grows."""
import numpy as np
import pytest

from helpers import random_graph

pytestmark = pytest.mark.gpu


def test_workspace_does_not_depend_on_the_number_of_edges():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    print("memory claim: workspace vs edge count", flush=True)
    rng = np.random.default_rng(123)
    n = 3000
    sizes = []
    for m in (6000, 24000, 72000):
        indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=True)
        g = pk.Graph(dev(indptr), dev(indices))
        sizes.append((pk.gnn_gat_workspace_bytes(g, 64, 4, 64), pk.gnn_edgeconv_workspace_bytes(g, 64, 64),
                      pk.gnn_gmm_workspace_bytes(g, 64, 64, 3)))
        g.close()
    assert sizes[0] == sizes[1] == sizes[2], sizes
    # and they are a small multiple of the vertex tensors: GAT keeps dz [n, HF] plus O(n H) scalars,
    # parameter partials and the split-K slabs of gw
    gat, ec, gmm = sizes[0]
    vertex = 4 * n * 256
    assert gat < 4 * vertex and ec < 4 * vertex and gmm < 4 * vertex


def test_blocked_path_workspace_is_still_vertex_sized():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    rng = np.random.default_rng(124)
    n = 3000
    pk.gnn_config_set("block_cols", 512)
    try:
        sizes = []
        for m in (20000, 60000):
            indptr, indices = random_graph(rng, n, m, self_loops=True, duplicates=True)
            g = pk.Graph(dev(indptr), dev(indices))
            assert g.blocked(0)[0] == 6
            sizes.append(pk.gnn_gat_workspace_bytes(g, 64, 4, 64))
            g.close()
    finally:
        pk.gnn_config_set("block_cols", 12288)
    assert sizes[0] == sizes[1]
    assert sizes[0] < 6 * 4 * n * 256
