"""Structured-binary (STBLLM) GEMV/GEMM for AMD MI355X: Python binding of libstb."""
from .binding import (  # noqa: F401
    LIB_PATH, EXPORTS, STB_BLOCK, STB_MAX_BATCH, STB_PLANE_ALIGN,
    STB_OK, STB_EINVAL, STB_ENULL, STB_EALIGN, STB_ENONFINITE, STB_EHIP, STB_EUNSUPPORTED, STB_ETOOBIG, STB_GEMV_STATIC_SCRATCH_BYTES,
    STB_KIND_ROWMAJOR, STB_KIND_TILED, StbError, stb_cfg_t, stb_layout_t, PLANE_FIELDS, PackedMatrix, make_cfg, aligned_bytes,
    stb_layout_sizes, stb_layout_bind, stb_tiled_sizes, stb_tile, stb_untile, stb_tile_device, stb_pack, stb_pack_obc, stb_hessian_factor, stb_pack_obc_hybrid, stb_pack_obc_hybrid_workspace_bytes, stb_pack_device, stb_pack_device_workspace_bytes, stb_unpack, stb_salient_columns, stb_salient_columns_hc, stb_layer_l2_norm, stb_layer_nm_assignment, stb_code24_export, stb_code24_import, stb_code24_index, stb_dequant, stb_gemv, stb_gemv_static, stb_gemv_workspace_bytes, stb_gemv_batched, stb_gemv_batched_workspace_bytes,
    stb_gemm, stb_gemm_workspace_bytes, new_device_scratch, stb_probe_read, stb_probe_mfma, stb_set_kernel_override, GEMV_THIN, GEMM_DENSE, GEMM_DENSE32, GEMM_SPARSE16, GEMM_SHARED,
)
