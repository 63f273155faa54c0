"""XQuant / XQuant-CL decode hot path for MI355X (gfx950): thin Python binding over
the C-ABI library libxquant.so (see include/xquant.h).  PyTorch is used only for
device memory and streams; every step of the path runs in the library's kernels."""
from .binding import (  # noqa: F401
    XQCache, XQAttn, XQError, alloc_cache, lib_path, load_library,
    xq_version, xq_status_string, xq_codes_row_bytes, xq_meta_row_elems,
    xq_quantize_append, xq_cl_delta_quantize, xq_cl_accumulate,
    xq_prepared_weights_bytes, xq_prepare_weights,
    xq_remat_attn_workspace_bytes, xq_remat_attn_decode, xq_remat_attn_decode_static, XQ_STATIC_SCRATCH_BYTES,
    xq_latent_project, xq_prepare_weights_latent, xq_remat_attn_decode_latent,
    xq_prepared_weights_latent_bytes, xq_remat_attn_latent_workspace_bytes,
    xq_cl_latent_delta_project, xq_cl_latent_delta_project_bulk, xq_prepared_upproject_bytes, xq_prepare_upproject,
    xq_cl_accumulate_latent_workspace_bytes, xq_cl_accumulate_latent,
    xq_remat_attn_prefill_workspace_bytes, xq_remat_attn_prefill,
    alloc_cache_per_channel, xq_quantize_blocks_per_channel,
    xq_remat_attn_per_channel_workspace_bytes, xq_remat_attn_decode_per_channel,
    xq_per_channel_terms_bytes, alloc_per_channel_terms,
    xq_prepared_weights_pairs_bytes, xq_prepare_weights_pairs,
    xq_remat_attn_latent_per_channel_workspace_bytes, xq_remat_attn_decode_latent_per_channel,
    xq_prepare_projection, xq_latent_project_bulk,
)
