"""MI355X-native sparse fully-connected training step of Mixed Sparsity Training.

The product is the C-ABI library ``libmst_hip.so`` (HIP kernels for gfx950, declared in
``include/mst.h``); this package is a thin ctypes binding with the same entry-point
names.  PyTorch is used by callers for device memory and streams only.
"""
from .binding import (  # noqa: F401
    MstError,
    ScheduleCfg,
    UpdateStats,
    Layer,
    lib,
    lib_path,
    mst_schedule_density,
    mst_update_counts,
    mst_workspace_bytes,
    mst_layer_device_bytes,
    mst_sparse_fc_fwd,
    mst_sparse_fc_bwd_input,
    mst_sparse_fc_bwd_weight,
    mst_sparse_fc_bwd_weight_static,
    mst_static_scratch_bytes,
    mst_sparse_fc_bwd,
    mst_bwd_force_shape,
    mst_mask_update,
    mst_mask_update_from_scores,
    mst_sparse_fc_bwd_weight_update,
    mst_dense_grad,
    mst_spmm_force_shape,
    mst_erdos_renyi_density,
    mst_flops_fc_forward,
    mst_flops_transformer,
    mst_strided_attention_mask,
    mst_strided_attention_count,
    MST_F32,
    MST_BF16,
    MST_PATH_AUTO,
    MST_PATH_SPARSE,
    MST_PATH_DENSE,
)
