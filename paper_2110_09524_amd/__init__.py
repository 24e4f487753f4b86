"""Reorganized, fused GNN layers for MI355X: thin Python binding over the C ABI
declared in include/gnn_fused.h.  All arithmetic runs in the HIP kernels of
csrc/; importing this package without the built library raises ImportError."""
from .binding import (  # noqa: F401
    EXPORTS, GNN_NUM_BUCKETS, LIB_PATH, GnnError, Graph, lib, load_library,
    gnn_config_set, gnn_linear_fwd, gnn_release_cached_memory,
    gnn_gat_workspace_bytes, gnn_gat_fwd, gnn_gat_bwd, gnn_gat_bwd_noalloc, NOALLOC_SCRATCH_BYTES, gnn_gat_blocked_kernel_name, gnn_gat_stash_alpha, gnn_gat_stash_layout, gnn_gat_bwd_stashed,
    gnn_edgeconv_workspace_bytes, gnn_edgeconv_fwd, gnn_edgeconv_bwd,
    gnn_gmm_workspace_bytes, gnn_gmm_fwd, gnn_gmm_bwd, gnn_gmm_tune, gnn_gmm_tune_bwd,
    gnn_gmmp_workspace_bytes, gnn_gmmp_fwd, gnn_gmmp_bwd,
    gnn_pseudo_proj_workspace_bytes, gnn_pseudo_proj_fwd, gnn_pseudo_proj_bwd,
    gnn_monet_workspace_bytes, gnn_monet_fwd, gnn_monet_bwd,
    gnn_gcn_workspace_bytes, gnn_gcn_fwd, gnn_gcn_bwd, gnn_gcn_tune, gnn_gcn_blocked_kernel_name,
    EdgeWeights, gnn_gcn_edge_fwd, gnn_gcn_edge_bwd,
    gnn_bias_act_fwd, gnn_bias_act_workspace_bytes, gnn_bias_act_bwd,
    gnn_softmax_xent_workspace_bytes, gnn_softmax_xent, gnn_sgd_update, gnn_knn_graph,
    gnn_prof_enable, gnn_prof_reset, gnn_prof_report,
)
