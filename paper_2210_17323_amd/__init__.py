"""MI355X-native GPTQ layer solver: thin Python binding over the C-ABI library libgptq_mi355.so.

All arithmetic runs in the hand-written HIP kernels under csrc/; PyTorch only provides device
memory and streams.  There is no CPU fallback: loading fails loudly if the library is missing.
"""
from .binding import (  # noqa: F401
    GptqError, lib, load_library, version, exported_symbols, gptq_release_thread_resources,
    gptq_hessian_accumulate, gptq_hessian_accumulate_workspace_bytes, gptq_hessian_accumulate_launches, gptq_hessian_symmetrize,
    gptq_hessian_accumulate_token_major, gptq_hessian_accumulate_token_major_workspace_bytes,
    gptq_damp_cholesky_inverse, gptq_damp_cholesky_inverse_workspace_bytes, gptq_check_info,
    gptq_damp_cholesky_inverse_noalloc, gptq_noalloc_max_n,
    gptq_damp_cholesky, gptq_damp_cholesky_workspace_bytes, gptq_quantize_layer_from_factor, gptq_quantize_layer_from_factor_supports,
    gptq_quantize_layer, gptq_quantize_layer_workspace_bytes, gptq_trailing_update,
    gptq_trailing_update_split, gptq_trailing_update_split_workspace_bytes,
    gptq_symmetric_update_split, gptq_symmetric_update_split_workspace_bytes, gptq_set_split_min_tiles,
    gptq_pack, gptq_unpack, packed_words_per_row, gptq_dequantize_packed, gptq_matvec_packed,
    GPTQ_GRID_MINMAX, GPTQ_GRID_TERNARY,
)
