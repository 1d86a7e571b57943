"""ctypes binding of libaj.so: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and streams
(``torch.cuda.current_stream().cuda_stream``); every step of the path runs in the library's
kernels.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# AJ_LIBRARY (environment) names another build of the library, e.g. one with profiling or ablation switches
_LIB_PATH = os.environ.get("AJ_LIBRARY") or os.path.join(_HERE, "libaj.so")

AJ_F32, AJ_BF16 = 0, 1
AJ_FLAG_DEBUG, AJ_FLAG_PROFILE, AJ_FLAG_TOPK, AJ_FLAG_FUSED_JUDGE = 1, 2, 4, 8
AJ_W_SAME, AJ_W_FP8_E4M3 = 0, 1
AJ_KERNEL_AUTO, AJ_KERNEL_TILE, AJ_KERNEL_STREAM, AJ_KERNEL_BIG, AJ_KERNEL_TALL, AJ_KERNEL_PAIR, AJ_KERNEL_PAIR9, AJ_KERNEL_RESIDENT, AJ_KERNEL_WIDE = 0, 1, 2, 3, 4, 5, 6, 7, 8

SYMBOLS = ["aj_create", "aj_verify", "aj_verify_static", "aj_verify_sampled", "aj_verify_tree", "aj_verify_topk", "aj_debug_copy_rank", "aj_destroy", "aj_debug_ptrs", "aj_debug_copy", "aj_debug_logits",
           "aj_profile_read", "aj_kernel_name", "aj_strerror", "aj_last_hip_error"]


class AjError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {aj_strerror(status)} (status {status})")


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "K", "d_t", "d_d", "V", "dtype", "feat_offset", "flags", "kernel", "w_dtype")]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libaj.so (built in-tree by ``paper_2504_20039_amd.build``). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built: run `python -m paper_2504_20039_amd.build` "
                          "(there is no fallback path)")
    # torch ships its own HIP runtime (same soname as the system one); import it first so that
    # libaj.so binds to that copy instead of bringing a second runtime into the process
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
    lib.aj_create.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(vp)]
    lib.aj_create.restype = ctypes.c_int
    lib.aj_verify.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, vp, vp, vp]
    lib.aj_verify.restype = ctypes.c_int
    lib.aj_verify_static.argtypes = [ctypes.POINTER(_Config), vp, vp, vp, vp, vp, f32, f32, vp, vp, vp]
    lib.aj_verify_static.restype = ctypes.c_int
    lib.aj_verify_sampled.argtypes = [vp, vp, vp, vp, vp, vp, f32, f32, f32, vp, vp, vp, vp]
    lib.aj_verify_sampled.restype = ctypes.c_int
    lib.aj_verify_tree.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, f32, vp, vp, vp, vp]
    lib.aj_verify_tree.restype = ctypes.c_int
    lib.aj_verify_topk.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp]
    lib.aj_verify_topk.restype = ctypes.c_int
    lib.aj_debug_copy_rank.argtypes = [vp, vp, vp]
    lib.aj_debug_copy_rank.restype = ctypes.c_int
    lib.aj_destroy.argtypes = [vp]
    lib.aj_destroy.restype = ctypes.c_int
    lib.aj_debug_ptrs.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp)]
    lib.aj_debug_ptrs.restype = ctypes.c_int
    lib.aj_debug_copy.argtypes = [vp, vp, vp, vp, vp]
    lib.aj_debug_copy.restype = ctypes.c_int
    lib.aj_debug_logits.argtypes = [vp, vp, vp, vp, vp]
    lib.aj_debug_logits.restype = ctypes.c_int
    lib.aj_profile_read.argtypes = [vp, ctypes.POINTER(f32), ctypes.POINTER(i32)]
    lib.aj_profile_read.restype = ctypes.c_int
    lib.aj_kernel_name.argtypes = [vp]
    lib.aj_kernel_name.restype = ctypes.c_char_p
    lib.aj_strerror.argtypes = [ctypes.c_int]
    lib.aj_strerror.restype = ctypes.c_char_p
    lib.aj_last_hip_error.argtypes = []
    lib.aj_last_hip_error.restype = ctypes.c_int
    _lib = lib
    return lib


def exported_symbols():
    """Names from include/aj.h that the loaded library exports."""
    lib = load_library()
    return [s for s in SYMBOLS if hasattr(lib, s)]


def aj_strerror(status: int) -> str:
    return load_library().aj_strerror(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("libaj takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libaj takes contiguous row-major tensors")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def aj_create(B, K, d_t, d_d, V, dtype=AJ_BF16, feat_offset=1, flags=0, kernel=AJ_KERNEL_AUTO, w_dtype=AJ_W_SAME):
    cfg = _Config(B, K, d_t, d_d, V, dtype, feat_offset, flags, kernel, w_dtype)
    h = ctypes.c_void_p()
    rc = load_library().aj_create(ctypes.byref(cfg), ctypes.byref(h))
    if rc != 0:
        raise AjError(rc, "aj_create")
    return h


def aj_verify(h, hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, out_len, out_tok, stream=None):
    rc = load_library().aj_verify(h, _ptr(hidden_t), _ptr(hidden_d), _ptr(W_lm), _ptr(draft_tok),
                                  _ptr(clf_w), float(clf_b), float(tau), _ptr(out_len), _ptr(out_tok),
                                  _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_verify")


def aj_verify_static(B, K, d_t, d_d, V, dtype, feat_offset, kernel, hidden_t, hidden_d, W_lm, draft_tok, clf_w,
                     clf_b, tau, out_len, out_tok, stream=None, flags=0, w_dtype=AJ_W_SAME):
    """aj_verify without a handle or any allocation (workspace in the library's static device array)."""
    cfg = _Config(B, K, d_t, d_d, V, dtype, feat_offset, flags, kernel, w_dtype)
    rc = load_library().aj_verify_static(ctypes.byref(cfg), _ptr(hidden_t), _ptr(hidden_d), _ptr(W_lm),
                                         _ptr(draft_tok), _ptr(clf_w), float(clf_b), float(tau), _ptr(out_len),
                                         _ptr(out_tok), _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_verify_static")


def aj_verify_sampled(h, hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, inv_temperature, row_key,
                      out_len, out_tok, stream=None):
    """row_key: device int64/uint64 tensor [B, K+1] (the bits are the key)."""
    rc = load_library().aj_verify_sampled(h, _ptr(hidden_t), _ptr(hidden_d), _ptr(W_lm), _ptr(draft_tok),
                                          _ptr(clf_w), float(clf_b), float(tau), float(inv_temperature),
                                          _ptr(row_key), _ptr(out_len), _ptr(out_tok), _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_verify_sampled")


def aj_verify_tree(h, hidden_t, hidden_d, W_lm, draft_tok, parent, clf_w, clf_b, tau, out_len, out_tok, out_node,
                   stream=None):
    rc = load_library().aj_verify_tree(h, _ptr(hidden_t), _ptr(hidden_d), _ptr(W_lm), _ptr(draft_tok), _ptr(parent),
                                       _ptr(clf_w), float(clf_b), float(tau), _ptr(out_len), _ptr(out_tok),
                                       _ptr(out_node), _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_verify_tree")


def aj_verify_topk(h, hidden_t, W_lm, draft_tok, top_k, out_len, out_tok, stream=None):
    rc = load_library().aj_verify_topk(h, _ptr(hidden_t), _ptr(W_lm), _ptr(draft_tok), int(top_k),
                                       _ptr(out_len), _ptr(out_tok), _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_verify_topk")


def aj_debug_copy_rank(h, B, K, stream=None):
    """Host copy of the draft tokens' ranks after aj_verify_topk: int32 [B*(K+1)]."""
    rank = np.empty(B * (K + 1), np.int32)
    rc = load_library().aj_debug_copy_rank(h, rank.ctypes.data, _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_debug_copy_rank")
    return rank


def aj_destroy(h):
    rc = load_library().aj_destroy(h)
    if rc != 0:
        raise AjError(rc, "aj_destroy")


def aj_kernel_name(h) -> str:
    return load_library().aj_kernel_name(h).decode()


def aj_debug_ptrs(h):
    """Raw device addresses (t_star, maxlogit, score-or-None) inside the handle's workspace."""
    t, m, s = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    rc = load_library().aj_debug_ptrs(h, ctypes.byref(t), ctypes.byref(m), None)
    if rc != 0:
        raise AjError(rc, "aj_debug_ptrs")
    rc = load_library().aj_debug_ptrs(h, None, None, ctypes.byref(s))
    return t.value, m.value, (s.value if rc == 0 else None)


def aj_debug_copy(h, B, K, want_score=True, stream=None):
    """Host copies (t_star int32 [B*(K+1)], maxlogit f32 [B*(K+1)], score f32 [2,B,K] or None)."""
    M = B * (K + 1)
    t_star = np.empty(M, np.int32)
    maxlogit = np.empty(M, np.float32)
    score = np.empty((2, B, K), np.float32) if want_score else None
    rc = load_library().aj_debug_copy(h, t_star.ctypes.data, maxlogit.ctypes.data,
                                      score.ctypes.data if want_score else None, _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_debug_copy")
    return t_star, maxlogit, score


def aj_debug_logits(h, hidden_t, W_lm, logits, stream=None):
    rc = load_library().aj_debug_logits(h, _ptr(hidden_t), _ptr(W_lm), _ptr(logits), _stream(stream))
    if rc != 0:
        raise AjError(rc, "aj_debug_logits")


def aj_profile_read(h, capacity=64):
    ms = (ctypes.c_float * capacity)()
    n = ctypes.c_int32(capacity)
    rc = load_library().aj_profile_read(h, ms, ctypes.byref(n))
    if rc != 0:
        raise AjError(rc, "aj_profile_read")
    return [float(ms[i]) for i in range(n.value)]


def device_tensor(a: np.ndarray, device="cuda:0"):
    """Upload a stored numpy tensor (uint16 = bf16 bits, float32, int32) without changing a bit."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)
