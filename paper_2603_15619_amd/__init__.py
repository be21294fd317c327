"""MoDA attention (Mixture-of-Depths Attention) for AMD MI355X: thin Python
binding over the libmoda C ABI.  All arithmetic runs in the HIP kernels."""
from .binding import (MODAError, MODAShape, lib, moda_attn_bwd, moda_attn_bwd_workspace_bytes,
                      moda_attn_decode, moda_attn_fwd, moda_calibrate_mfma, moda_depth_append, status_string)

__all__ = ["MODAError", "MODAShape", "lib", "moda_attn_fwd", "moda_attn_bwd",
           "moda_attn_bwd_workspace_bytes", "moda_attn_decode", "moda_calibrate_mfma", "moda_depth_append",
           "status_string"]
