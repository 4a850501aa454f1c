"""MI355X (gfx950) library for the GPU hot path of LSP-Offload: compress S = P^T G Q and
decompress-and-apply W <- W - P S Q^T with (d,r)-sparse ELL projectors (Alg. 1 / Alg. 3, Def. 1),
and the estimation bias of Def. 2 built from the two.

This package is a thin binding: it marshals torch device pointers into the C ABI declared in
``include/lsp.h``.  Every step of the path runs in the HIP kernels of ``liblsp_hip.so``; there is
no CPU fallback, and importing the binding fails loudly if the library has not been built.
"""
from .binding import (  # noqa: F401
    LspError, DTYPE_CODE, lib, lib_path,
    lsp_compress, lsp_compress_workspace_bytes, lsp_workspace_bytes,
    lsp_plan_bytes, lsp_plan_build, lsp_plan_build_host, lsp_plan_build_async, lsp_plan_build_workspace_bytes,
    lsp_compress_planned, lsp_compress_planned_workspace_bytes, lsp_compress_planned_static, lsp_static_scratch_bytes,
    lsp_decompress_apply, lsp_compress_planned_grouped, lsp_decompress_apply_grouped, lsp_compress_dense, lsp_compress_dense_workspace_bytes,
    lsp_estimation_bias, lsp_estimation_bias_workspace_bytes,
    lsp_reproject_state, lsp_reproject_state_workspace_bytes, lsp_projector_reorder_host, lsp_projector_reorder,
    lsp_compress_item, lsp_apply_item, compress_items, apply_items, lsp_validate_projector, lsp_strerror, lsp_version,
    torch_dtype_code, lsp_plan_refresh_values, lsp_bias_gradient, lsp_bias_gradient_workspace_bytes, lsp_hbm_probe_read, lsp_hbm_probe_rmw, lsp_hbm_probe_workspace_bytes,
)
