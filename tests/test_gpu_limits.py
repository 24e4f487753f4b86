"""Documented size limits of the C ABI: every call below is rejected by a host-side check before
anything is launched (status GNN_ERR_UNSUPPORTED = 4), so the buffers are tiny stand-ins."""
import ctypes as C

import numpy as np
import pytest

from helpers import random_graph

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def small():
    import paper_2110_09524_amd as pk
    from gpu_harness import dev
    rng = np.random.default_rng(5)
    indptr, indices = random_graph(rng, 40, 200)
    g = pk.Graph(dev(indptr), dev(indices))
    yield g
    g.close()


def _unsupported(fn, *args):
    import paper_2110_09524_amd as pk
    with pytest.raises(pk.GnnError) as e:
        fn(*args)
    assert e.value.status == 4, str(e.value)


def test_edge_count_beyond_32_bits_is_rejected_before_any_access():
    import paper_2110_09524_amd as pk
    from paper_2110_09524_amd import binding
    from gpu_harness import dev
    print("limits: nnz = 2^31", flush=True)
    ptr = dev(np.zeros(4, dtype=np.int32))
    handle = C.c_void_p()
    status = binding.lib().gnn_graph_create(3, 2 ** 31, C.c_void_p(ptr.data_ptr()), C.c_void_p(ptr.data_ptr()),
                                            None, C.byref(handle))
    assert status == 4 and not handle.value
    assert b"32-bit" in binding.lib().gnn_last_error()


def test_layer_shapes_outside_the_kernels_range(small):
    import paper_2110_09524_amd as pk
    from gpu_harness import empty
    print("limits: layer shapes", flush=True)
    g, b = small, empty((4, 4))
    i32 = empty((4, 4)).int()
    # GAT: heads * f <= 1024, heads <= 64, f a multiple of 4
    for heads, f in ((2, 1024), (128, 4), (1, 6)):
        _unsupported(pk.gnn_gat_fwd, g, 8, heads, f, 0.2, b, b, b, b, b, b, b, b, b, b)
        _unsupported(pk.gnn_gat_bwd, g, 8, heads, f, 0.2, b, b, b, b, b, b, b, b, b, b, None, None, b, b, b, b, b, None)
    # EdgeConv and GCN: fout a multiple of 4, at most 1024
    for fout in (1028, 10):
        _unsupported(pk.gnn_edgeconv_fwd, g, 8, fout, b, b, b, b, b, i32)
        _unsupported(pk.gnn_gcn_fwd, g, 8, fout, b, b, b, b, b, b)
    # GMM: fout at most 256, at most 8 kernels; general form: at most 4 kernels and 4 dimensions
    _unsupported(pk.gnn_gmm_fwd, g, 8, 260, 2, b, b, b, b, b, b, b)
    _unsupported(pk.gnn_gmm_fwd, g, 8, 16, 9, b, b, b, b, b, b, b)
    _unsupported(pk.gnn_gmmp_fwd, g, 8, 16, 5, 1, b, b, b, b, b, b, b)
    _unsupported(pk.gnn_gmmp_fwd, g, 8, 16, 2, 5, b, b, b, b, b, b, b)
    _unsupported(pk.gnn_pseudo_proj_fwd, g, 5, b, b, b, b)


def test_vertex_operator_and_knn_limits():
    import paper_2110_09524_amd as pk
    from gpu_harness import empty
    print("limits: vertex operators, kNN", flush=True)
    b = empty((4, 4))
    i32 = empty((4, 4)).int()
    _unsupported(pk.gnn_bias_act_fwd, 4, 1028, "relu", 0.0, b, b, b)      # f at most 1024
    _unsupported(pk.gnn_softmax_xent, 4, 5000, 4, b, i32, b, b, None)      # at most 4096 classes
    _unsupported(pk.gnn_knn_graph, 1, 8, 3, 9, b, i32, i32)                # k beyond the cloud size
    _unsupported(pk.gnn_knn_graph, 1, 1 << 20, 3, 4, b, i32, i32)          # cloud too large for one workgroup's scan
