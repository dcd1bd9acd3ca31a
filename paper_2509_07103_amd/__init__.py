"""MI355X-native lmKAN layer: Python names mirror the C ABI of include/lmkan.h."""
from .binding import (LMKAN_BF16, LMKAN_F16, LMKAN_F32, LMKAN_FLAG_ACCUMULATE_GRAD_COEF, LMKAN_FLAG_WORKSPACE_HAS_RECORDS,
                      LMKAN_LAYOUT_PACKED, LMKAN_LAYOUT_PAPER, LMKAN_MAX_GRID, LMKAN_PACK_TILE, LMKAN_STATIC_SCRATCH_BYTES,
                      Conv2d, LayerDesc, LmkanError, lib, lmkan_backward, lmkan_conv2d_backward,
                      lmkan_conv2d_forward, lmkan_conv2d_rows, lmkan_forward, lmkan_forward_static, lmkan_grid,
                      lmkan_fold, lmkan_hessian_reg,
                      lmkan_locate, lmkan_microbench, MICROBENCH, lmkan_pack, lmkan_time_next_kernel, lmkan_packed_bytes, lmkan_status_string,
                      lmkan_version, lmkan_workspace_bytes)

__all__ = [n for n in dir() if n.startswith(("lmkan_", "LMKAN_", "Layer", "Lmkan", "Conv2d", "lib", "MICROBENCH"))]
