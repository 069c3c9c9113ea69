"""MI355X-native GCN layer path: Python binding over the C-ABI library ``libgcn.so``.

The binding only marshals arguments (torch tensors -> device pointers, current stream);
every step of the path runs in the library's HIP kernels.  Importing this package fails
loudly if the library has not been built (``python -m paper_2212_05009_amd.build`` or
``__graft_entry__.build()``); there is no CPU fallback.
"""
from .binding import (  # noqa: F401
    BF16, F32, EPI_NONE, EPI_RELU, EPI_MASK, ACT_NONE, ACT_RELU, BUILD_CSC, PART_LOCAL, PART_HALO,
    Csr, GcnError, gcn_csr_build, gcn_csr_induced, gcn_spmm, gcn_spmm_noalloc, gcn_spmm_t, gcn_spmm_part, gcn_dense_fwd, gcn_halo_gather, gcn_layer_fwd,
    gcn_layer_bwd, gcn_layer_fwd_ld, gcn_layer_bwd_ld, gcn_layer_bwd_pull, gcn_softmax_xent, gcn_sgd_update, gcn_partition_stats, gcn_profile_enable, gcn_profile_filter, gcn_debug_max_grid_x, gcn_debug_set_tuning, gcn_feature_ld, feature_buffer, gcn_profile_records, library_path,
)
