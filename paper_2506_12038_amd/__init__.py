"""MI355X-native hot path of LCD's smoothed table-lookup linear layer (HIP, gfx950).

The product lives in ``liblcd.so`` (C ABI declared in ``include/lcd.h``); this package only
marshals torch tensors into it.  Nothing here computes on the CPU.
"""
from .binding import (  # noqa: F401
    LcdError, LIB_PATH, EXPORTS, load_library,
    lcd_version, lcd_layout_revision, lcd_packed_bytes, lcd_lut_bytes, lcd_workspace_bytes,
    lcd_pack_indices, lcd_unpack_indices, lcd_pack_indices_host, lcd_unpack_indices_host,
    lcd_build_lut, lcd_lut_gemv, lcd_lut_gemm, lcd_lut_gemv_q8, lcd_lut_gemm_q8, lcd_lut_gemv_noalloc, lcd_lut_gemv_grouped, lcd_workspace_bytes_grouped, GemvGroup, lcd_lut_gemm_grouped, GemmGroup,
    lcd_assign_indices, lcd_cluster_counts, lcd_merge_closest,
)
