"""MI355X-native shard-local latent-attention decode for TPLA (arXiv 2508.15881).

The compute lives in libtpla.so (HIP, gfx950) behind the C ABI declared in
include/tpla.h; `binding` marshals torch tensors into it.  Importing the
package does not load the library; the first call does, and fails loudly if
the library has not been built (python -m paper_2508_15881_amd.build).
"""
from .binding import (  # noqa: F401
    TPLA_BF16, TPLA_F32, TPLA_U_DENSE, TPLA_U_HADAMARD, TPLA_U_IDENTITY,
    TplaError, TplaShape, lib_path, load_library,
    tpla_absorb_query, tpla_combine_shards, tpla_decode_shard, tpla_last_error,
    tpla_transform_latent, tpla_transform_latent_paged, tpla_version,
    tpla_workspace_bytes, tpla_write_mla_cache, tpla_profile_enable, tpla_profile_collect, tpla_decode_shards, tpla_workspace_bytes_all, tpla_append_token_sliced, tpla_output_projection, tpla_output_projection_workspace_bytes,
    tpla_latent_moments, tpla_latent_moments_workspace_bytes, tpla_pca_basis, tpla_prefill_attention, tpla_prefill_workspace_bytes, tpla_stream_read,
    tpla_decode_shards_combine, tpla_validate_block_table, tpla_decode_shards_combine_static,
    tpla_combine_shards_to, tpla_decode_shards_combine_to, tpla_output_projection_to,
    tpla_attention_block_workspace_bytes, tpla_decode_shards_project,
)
