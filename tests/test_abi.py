"""The C-ABI library loads and exports every function the header declares
(no compute calls here: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gnn_fused.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gnn_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_layer_calls():
    names = declared_functions()
    for required in ["gnn_graph_create", "gnn_graph_destroy", "gnn_gat_fwd", "gnn_gat_bwd",
                     "gnn_edgeconv_fwd", "gnn_edgeconv_bwd", "gnn_gmm_fwd", "gnn_gmm_bwd",
                     "gnn_last_error"]:
        assert required in names


def test_library_exports_every_declared_symbol():
    import paper_2110_09524_amd as pk
    if not os.path.exists(pk.LIB_PATH):
        pytest.fail(f"{pk.LIB_PATH} is not built; run __graft_entry__.build() first")
    lib = ctypes.CDLL(pk.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in gnn_fused.h but not exported"
    assert set(pk.EXPORTS) == set(declared_functions())


def test_missing_library_fails_loudly(tmp_path):
    import paper_2110_09524_amd as pk
    with pytest.raises(ImportError):
        pk.load_library(str(tmp_path / "nope.so"))


def test_last_error_is_empty_string_initially():
    import paper_2110_09524_amd as pk
    lib = pk.load_library()
    assert isinstance(lib.gnn_last_error(), bytes)
