"""MI355X-native Dynamic Sparse Window Attention (DSVT, arXiv 2301.06051).

The package is a thin binding over libdsvt.so (hand-written HIP for gfx950); see binding.py.
"""
from .binding import (  # noqa: F401
    DsvtError, LayerWeights, PoolWeights, SetMaps, SetMapsXY, Vfe, dsvt_vfe, dsvt_vfe_workspace_size, dsvt_set_attention_workspace_size, dsvt_attn_pool, dsvt_attn_pool_static, dsvt_attn_pool_workspace_size, dsvt_bev_scatter, dsvt_block,
    dsvt_block_workspace_size, dsvt_partition, dsvt_partition_bound, dsvt_partition_xy, dsvt_partition_xy_multi, dsvt_set_attention, lib, part_cfg,
    prof_collect, prof_enable)
