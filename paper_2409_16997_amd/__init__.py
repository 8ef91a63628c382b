"""INT-FlashAttention forward for AMD MI355X: thin Python binding over the C ABI of libintfa.so.

Every step of the path runs in the hand-written HIP kernels of csrc/; this package only marshals
arguments (torch is used for device memory and streams).  There is no CPU fallback: if the library
has not been built, loading it raises.
"""
from .binding import (  # noqa: F401
    IFA_F32, IFA_F16, IFA_BF16, IntfaError, lib, lib_path, quantize_tokenwise, quantize_headwise, quantize_blockwise, quantize_qk, quantize_qkv,
    int_flash_attn_fwd, int_flash_attn_fwd_splitk, splitk_workspace_bytes, block_cols, int_flash_attn_fwd_half, block_cols_half, debug_fwd, status_str,
)
