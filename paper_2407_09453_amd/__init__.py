"""Block-sparse convolution / fully-connected inference for AMD MI355X.

A thin binding over libbsp.so (C ABI in include/bsp.h): argument marshalling
only.  There is no CPU or PyTorch fallback: importing the device entry points
without the built library raises.
"""
from .binding import (  # noqa: F401
    BSP_BF16,
    BSP_F32,
    BSP_I8,
    BSP_IMPORTANCE_L1,
    BSP_IMPORTANCE_L2,
    BSP_IMPORTANCE_VAR,
    BSP_I32,
    BspError,
    BspLayer,
    BspLayerI8,
    BspMatrix,
    bsp_bcsr,
    bsp_bcsr_index,
    bsp_block_importance,
    bsp_conv2d,
    bsp_conv2d_fused,
    bsp_conv2d_general,
    bsp_conv2d_i8,
    bsp_fc,
    bsp_fc_fused,
    bsp_fc_i8,
    bsp_mask_step,
    bsp_pack,
    bsp_pack_count,
    bsp_plan_build,
    bsp_plan_size,
    bsp_quantize,
    bsp_select_mask,
    bsp_spgemm_nt,
    bsp_strerror,
    bsp_unpack,
    bsp_validate,
    bsp_version,
    bsp_weights,
    lib_path,
    load_library,
)
