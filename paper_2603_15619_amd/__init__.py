"""MoDA attention (Mixture-of-Depths Attention) for AMD MI355X: thin Python
binding over the libmoda C ABI.  All arithmetic runs in the HIP kernels."""
