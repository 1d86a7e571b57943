"""MI355X-native judge-augmented verification of speculation windows (AutoJudge, Section 3.3).

The product is the C-ABI library ``libaj.so`` (hand-written HIP for gfx950, declared in
``include/aj.h``); this package is its thin ctypes binding.  There is no CPU fallback: without
the built library every call raises.
"""
from .binding import (  # noqa: F401
    AJ_BF16, AJ_F32, AJ_FLAG_DEBUG, AJ_FLAG_FUSED_JUDGE, AJ_FLAG_PROFILE, AJ_FLAG_TOPK, AJ_KERNEL_AUTO, AJ_KERNEL_BIG, AJ_KERNEL_PAIR, AJ_KERNEL_PAIR9, AJ_KERNEL_RESIDENT, AJ_KERNEL_TALL,
    AJ_KERNEL_STREAM, AJ_KERNEL_TILE, AJ_KERNEL_WIDE, AJ_W_FP8_E4M3, AJ_W_SAME, AjError, aj_create, aj_debug_copy, aj_debug_copy_rank, aj_debug_logits, aj_debug_ptrs,
    aj_destroy, aj_kernel_name, aj_profile_read, aj_strerror, aj_verify, aj_verify_sampled, aj_verify_static, aj_verify_topk, aj_verify_tree, device_tensor,
    exported_symbols, library_path, load_library,
)
