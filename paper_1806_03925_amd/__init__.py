"""MI355X-native Gear Training sparse-part step (libgear.so) and its thin Python binding."""
from .binding import (  # noqa: F401
    GEAR_BF16, GEAR_ERR_CAPACITY, GEAR_ERR_HIP, GEAR_ERR_INVALID, GEAR_ERR_RANGE, GEAR_F32, GEAR_OK,
    AdamMoments, DenseStandIn, DeviceBatch, GearError, GearProfile, GearState, gear_config, gear_fill_normal, gear_gemm, gear_group_ids, gear_init_tables,
    gear_expired_ids, gear_mlp_param_count, gear_mlp_param_offset, gear_refresh_dfv, gear_refresh_dfv_n, gear_stamp_dfv, gear_stamp_dfv_n, gear_step, gear_step_adam, gear_step_static,
    gear_workspace_bytes, gear_debug_fail_launch, gear_debug_helper_idle,
    gear_workspace_region, lib, make_config,
)


def config_for(wl, max_batch=None, max_nnz=None):
    """gear_config for a workload description (any object with the fields of gear_inputs.GearWorkload)."""
    mb = wl.batch if max_batch is None else max_batch
    return make_config(wl.n_users, wl.n_urls, wl.n_images, wl.emb_dim, wl.dfv_dim, wl.layers,
                       wl.emb_dtype, wl.dfv_dtype, wl.mlp_dtype, max_batch=mb,
                       max_nnz=mb * wl.max_images if max_nnz is None else max_nnz,
                       seed=wl.seed, emb_init_std=wl.emb_std)
