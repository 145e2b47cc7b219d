"""V:N:M sparse linear layers for AMD MI355X: thin Python binding over the libvnm C ABI.

The three calls of the hot path -- vnm_prune_compress, vnm_spmm, vnm_decompress -- run entirely in
the HIP kernels of libvnm.so; this package only marshals arguments.  There is no CPU fallback: if
the library is missing, importing the binding raises.
"""

from .binding import (  # noqa: F401
    VnmError, VnmSizes, Compressed, lib_path, load_library, vnm_query_sizes, vnm_prune_compress,
    vnm_pack, vnm_spmm, vnm_spmm_bind, vnm_spmm_noalloc, NOALLOC_SCRATCH_BYTES, vnm_spmm_workspace_bytes, vnm_stage_x, vnm_spmm_staged,
    vnm_spmm_scratch_bytes, vnm_spmm_kernel_choice, KERNEL_GENERIC, KERNEL_FEW_TOKENS, KERNEL_RESIDENT,
    KERNEL_STAGED, vnm_decompress, vnm_ria_scores, vnm_prune_compress_scored,
    vnm_mask_diversity_log, vnm_select_vm, vnm_spmm_fused, vnm_fold_permutations, vnm_permutation_search,
    vnm_permutation_gain, vnm_retained_score, vnm_lora_merge, vnm_refresh_mask, PATH_AUTO, PATH_GENERIC, PATH_SMFMAC,
)
