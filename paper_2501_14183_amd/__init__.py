"""VarDrop training hot path for AMD MI355X: k-DFH hashing, stratified sampling, gather and
multi-head attention over the kept variate tokens (and their embedding), as HIP kernels behind a C ABI
(include/vardrop.h).  This package is the thin Python binding of that ABI."""
from .binding import (  # noqa: F401
    BF16, F32, Context, VarDropError, library_path, load_library,
    vardrop_attn_bwd, vardrop_attn_fwd, vardrop_embed_bwd, vardrop_embed_fwd, vardrop_gather, vardrop_gather_attn_fwd,
    vardrop_hash, vardrop_kernel_name,
    vardrop_profile_read, vardrop_profile_select, vardrop_profile_stride, vardrop_sample, vardrop_sample_nearest, vardrop_scatter,
    vardrop_attn_bwd_dev, vardrop_gather_attn_fwd_dev, vardrop_gather_dev, vardrop_sample_dev, vardrop_scatter_dev,
    vardrop_sample_nearest_noalloc, vardrop_attn_fwd_dev, vardrop_embed_fwd_dev, vardrop_embed_bwd_dev, vardrop_profile_read_all, K_ALL, vardrop_signal_after,
)
