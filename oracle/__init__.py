"""ctypes binding of the CPU oracle (oracle/aj_oracle.c).

TEST INFRASTRUCTURE: importable only from tests/, the smoke check and the
benchmark's CPU-baseline leg.  Nothing in the product package imports this, and
this package imports nothing from the product.

Arrays are numpy: ``uint16`` = bfloat16 bits, ``float32`` = fp32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aj_oracle.c")
_LIB = os.path.join(_HERE, "libaj_oracle.so")

F32, BF16 = 0, 1
NEAR_TIE_REL = 1e-3
NEAR_THR_REL = 1e-4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (host code only, no HIP)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    if force:   # the self-test program (run under sanitizers by the tests) must at least compile
        selftest = os.path.join(os.path.dirname(_SRC), "selftest.c")
        subprocess.run(["gcc", "-O1", "-fopenmp", "-Wall", "-c", selftest, "-o", os.devnull], check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, dbl, flt = ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_float
        lib.ajo_num_threads.restype = i32
        lib.ajo_logits_row.argtypes = [i32, vp, vp, i32, i32, vp]
        lib.ajo_logits_row.restype = i32
        lib.ajo_greedy_rows.argtypes = [i32, vp, i32, vp, i32, i32, vp, vp, vp]
        lib.ajo_greedy_rows.restype = i32
        lib.ajo_judge_logit.argtypes = [i32, vp, vp, vp, i32, i32, dbl]
        lib.ajo_judge_logit.restype = dbl
        lib.ajo_threshold_logit.argtypes = [dbl]
        lib.ajo_threshold_logit.restype = dbl
        lib.ajo_walk.argtypes = [i32] * 6 + [vp] * 5 + [flt, flt] + [vp] * 6
        lib.ajo_walk.restype = i32
        lib.ajo_verify.argtypes = [i32] * 7 + [vp] * 5 + [flt, flt] + [vp] * 10
        lib.ajo_verify.restype = i32
        lib.ajo_rank_rows.argtypes = [i32, vp, i32, vp, i32, i32] + [vp] * 7
        lib.ajo_rank_rows.restype = i32
        lib.ajo_walk_topk.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        lib.ajo_walk_topk.restype = i32
        lib.ajo_verify_topk.argtypes = [i32] * 6 + [vp] * 10
        lib.ajo_verify_topk.restype = i32
        lib.ajo_walk_tree.argtypes = [i32] * 6 + [vp] * 6 + [flt, flt] + [vp] * 7
        lib.ajo_walk_tree.restype = i32
        lib.ajo_verify_tree.argtypes = [i32] * 7 + [vp] * 6 + [flt, flt] + [vp] * 10
        lib.ajo_verify_tree.restype = i32
        lib.ajo_gumbel.argtypes = [ctypes.c_uint64, i32]
        lib.ajo_gumbel.restype = dbl
        lib.ajo_sampled_rows.argtypes = [i32, vp, i32, vp, i32, i32, dbl, vp, vp, vp, vp]
        lib.ajo_sampled_rows.restype = i32
        lib.ajo_verify_sampled.argtypes = [i32] * 7 + [vp] * 5 + [flt, flt, flt, vp] + [vp] * 10
        lib.ajo_verify_sampled.restype = i32
        _lib = lib
    return _lib


def _code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"stored tensors are float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a, dtype=None):
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data


def num_threads() -> int:
    return int(_load().ajo_num_threads())


def logits_row(h_row: np.ndarray, W_lm: np.ndarray) -> np.ndarray:
    """Step 1 for one verify row: fp64 logits [V]."""
    h_row, W_lm = _c(h_row), _c(W_lm)
    V, d_t = W_lm.shape
    assert h_row.shape == (d_t,) and _code(h_row) == _code(W_lm)
    out = np.empty(V, dtype=np.float64)
    rc = _load().ajo_logits_row(_code(W_lm), _ptr(h_row), _ptr(W_lm), V, d_t, _ptr(out))
    if rc:
        raise RuntimeError(f"ajo_logits_row rc={rc}")
    return out


def greedy_rows(hidden_t: np.ndarray, W_lm: np.ndarray):
    """Steps 1-2: (t_star int32 [M], max1 f64 [M], max2 f64 [M])."""
    W_lm = _c(W_lm)
    V, d_t = W_lm.shape
    hidden_t = _c(hidden_t).reshape(-1, d_t)
    assert _code(hidden_t) == _code(W_lm)
    M = hidden_t.shape[0]
    t = np.empty(M, dtype=np.int32)
    m1 = np.empty(M, dtype=np.float64)
    m2 = np.empty(M, dtype=np.float64)
    rc = _load().ajo_greedy_rows(_code(W_lm), _ptr(hidden_t), M, _ptr(W_lm), V, d_t,
                                 _ptr(t), _ptr(m1), _ptr(m2))
    if rc:
        raise RuntimeError(f"ajo_greedy_rows rc={rc}")
    return t, m1, m2


def near_tie(max1: np.ndarray, max2: np.ndarray) -> np.ndarray:
    return (max1 - max2) < NEAR_TIE_REL * np.abs(max1)


def judge_logit(ht_row, hd_row, clf_w, clf_b: float) -> float:
    ht_row, clf_w = _c(ht_row), _c(clf_w)
    d_t = ht_row.shape[0]
    d_d = clf_w.shape[0] - d_t
    hd_row = _c(hd_row) if d_d > 0 else None
    return float(_load().ajo_judge_logit(_code(clf_w), _ptr(ht_row), _ptr(hd_row), _ptr(clf_w),
                                         d_t, d_d, float(clf_b)))


def threshold_logit(tau: float) -> float:
    return float(_load().ajo_threshold_logit(float(tau)))


class WalkResult:
    __slots__ = ("out_len", "out_tok", "mismatch", "z", "p", "near_thr")


def walk(hidden_t, hidden_d, t_star, draft_tok, clf_w, clf_b, tau, feat_offset=1) -> WalkResult:
    """Steps 3-4 given the greedy tokens t_star [B, K+1]."""
    draft_tok = _c(draft_tok, np.int32)
    B, K = draft_tok.shape
    t_star = _c(t_star, np.int32).reshape(B, K + 1)
    clf_w = _c(clf_w)
    hidden_t = _c(hidden_t).reshape(B, K + 1, -1)
    d_t = hidden_t.shape[2]
    d_d = clf_w.shape[0] - d_t
    hidden_d = _c(hidden_d).reshape(B, K + 1, d_d) if d_d > 0 else None
    r = WalkResult()
    r.out_len = np.empty(B, np.int32)
    r.out_tok = np.empty(B, np.int32)
    r.mismatch = np.empty((B, K), np.uint8)
    r.z = np.empty((B, K), np.float64)
    r.p = np.empty((B, K), np.float64)
    r.near_thr = np.empty((B, K), np.uint8)
    rc = _load().ajo_walk(B, K, d_t, d_d, _code(clf_w), feat_offset,
                          _ptr(hidden_t), _ptr(hidden_d), _ptr(t_star), _ptr(draft_tok), _ptr(clf_w),
                          float(clf_b), float(tau), _ptr(r.out_len), _ptr(r.out_tok),
                          _ptr(r.mismatch), _ptr(r.z), _ptr(r.p), _ptr(r.near_thr))
    if rc:
        raise ValueError(f"ajo_walk rc={rc}")
    return r


class VerifyResult:
    __slots__ = ("out_len", "out_tok", "t_star", "max1", "max2", "near_tie",
                 "mismatch", "z", "p", "near_thr")


def verify(hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, feat_offset=1) -> VerifyResult:
    """Steps 1-4 (the whole verification step) with all diagnostics."""
    draft_tok = _c(draft_tok, np.int32)
    B, K = draft_tok.shape
    W_lm, clf_w = _c(W_lm), _c(clf_w)
    V, d_t = W_lm.shape
    d_d = clf_w.shape[0] - d_t
    hidden_t = _c(hidden_t).reshape(B, K + 1, d_t)
    hidden_d = _c(hidden_d).reshape(B, K + 1, d_d) if d_d > 0 else None
    M = B * (K + 1)
    r = VerifyResult()
    r.out_len = np.empty(B, np.int32)
    r.out_tok = np.empty(B, np.int32)
    r.t_star = np.empty(M, np.int32)
    r.max1 = np.empty(M, np.float64)
    r.max2 = np.empty(M, np.float64)
    r.near_tie = np.empty(M, np.uint8)
    r.mismatch = np.empty((B, K), np.uint8)
    r.z = np.empty((B, K), np.float64)
    r.p = np.empty((B, K), np.float64)
    r.near_thr = np.empty((B, K), np.uint8)
    rc = _load().ajo_verify(B, K, d_t, d_d, V, _code(W_lm), feat_offset,
                            _ptr(hidden_t), _ptr(hidden_d), _ptr(W_lm), _ptr(draft_tok), _ptr(clf_w),
                            float(clf_b), float(tau), _ptr(r.out_len), _ptr(r.out_tok),
                            _ptr(r.t_star), _ptr(r.max1), _ptr(r.max2), _ptr(r.near_tie),
                            _ptr(r.mismatch), _ptr(r.z), _ptr(r.p), _ptr(r.near_thr))
    if rc:
        raise ValueError(f"ajo_verify rc={rc}")
    return r


# ---- top-K baseline (Section 4: accept a mismatching draft token within the target's top-k tokens)

class RankResult:
    __slots__ = ("t_star", "max1", "rank", "rank_lo", "rank_hi", "tok_logit")


def rank_rows(hidden_t, W_lm, tok) -> RankResult:
    """Per verify row: the greedy token and the rank of tok[r] (number of vocabulary entries ordered
    before it: larger logit first, lower index first among equals; -1 = no token, >= V = invalid)."""
    W_lm = _c(W_lm)
    V, d_t = W_lm.shape
    hidden_t = _c(hidden_t).reshape(-1, d_t)
    tok = _c(tok, np.int32).reshape(-1)
    M = hidden_t.shape[0]
    assert tok.shape == (M,) and _code(hidden_t) == _code(W_lm)
    r = RankResult()
    r.t_star = np.empty(M, np.int32)
    r.max1 = np.empty(M, np.float64)
    r.rank = np.empty(M, np.int32)
    r.rank_lo = np.empty(M, np.int32)
    r.rank_hi = np.empty(M, np.int32)
    r.tok_logit = np.empty(M, np.float64)
    rc = _load().ajo_rank_rows(_code(W_lm), _ptr(hidden_t), M, _ptr(W_lm), V, d_t, _ptr(tok),
                               _ptr(r.t_star), _ptr(r.max1), _ptr(r.rank), _ptr(r.rank_lo), _ptr(r.rank_hi),
                               _ptr(r.tok_logit))
    if rc:
        raise ValueError(f"ajo_rank_rows rc={rc}")
    return r


def walk_topk(rank, t_star, top_k: int):
    """First-reject walk of the baseline: (out_len [B], out_tok [B]) from rank / t_star [B][K+1]."""
    rank, t_star = _c(rank, np.int32), _c(t_star, np.int32)
    B, R = rank.shape
    assert t_star.shape == (B, R)
    out_len, out_tok = np.empty(B, np.int32), np.empty(B, np.int32)
    rc = _load().ajo_walk_topk(B, R - 1, int(top_k), _ptr(rank), _ptr(t_star), _ptr(out_len), _ptr(out_tok))
    if rc:
        raise ValueError(f"ajo_walk_topk rc={rc}")
    return out_len, out_tok


class TopkResult:
    __slots__ = ("out_len", "out_tok", "t_star", "max1", "rank", "rank_lo", "rank_hi")


def verify_topk(hidden_t, W_lm, draft_tok, top_k: int) -> TopkResult:
    """The whole top-K baseline step with per-row diagnostics ([B*(K+1)]; the rank entries of the bonus
    rows are 0)."""
    draft_tok = _c(draft_tok, np.int32)
    B, K = draft_tok.shape
    W_lm = _c(W_lm)
    V, d_t = W_lm.shape
    hidden_t = _c(hidden_t).reshape(B, K + 1, d_t)
    M = B * (K + 1)
    r = TopkResult()
    r.out_len, r.out_tok = np.empty(B, np.int32), np.empty(B, np.int32)
    r.t_star, r.max1 = np.empty(M, np.int32), np.empty(M, np.float64)
    r.rank, r.rank_lo, r.rank_hi = np.empty(M, np.int32), np.empty(M, np.int32), np.empty(M, np.int32)
    rc = _load().ajo_verify_topk(B, K, d_t, V, _code(W_lm), int(top_k), _ptr(hidden_t), _ptr(W_lm),
                                 _ptr(draft_tok), _ptr(r.out_len), _ptr(r.out_tok), _ptr(r.t_star),
                                 _ptr(r.max1), _ptr(r.rank), _ptr(r.rank_lo), _ptr(r.rank_hi))
    if rc:
        raise ValueError(f"ajo_verify_topk rc={rc}")
    return r


# ---- sampling mode (Appendix A: Gumbel-max reparameterisation of stochastic decoding)

def gumbel(key: int, v: int) -> float:
    """Standard Gumbel noise of vocabulary entry v under a row key (the counter-based generator of the oracle)."""
    return float(_load().ajo_gumbel(int(key) & 0xFFFFFFFFFFFFFFFF, int(v)))


def sampled_rows(hidden_t, W_lm, inv_temperature: float, row_key):
    """(y int32 [M], max1 f64 [M], max2 f64 [M]): argmax of logit / T + Gumbel(key, v) per verify row."""
    W_lm = _c(W_lm)
    V, d_t = W_lm.shape
    hidden_t = _c(hidden_t).reshape(-1, d_t)
    M = hidden_t.shape[0]
    row_key = _c(row_key, np.uint64).reshape(-1)
    assert row_key.shape == (M,) and _code(hidden_t) == _code(W_lm)
    y, m1, m2 = np.empty(M, np.int32), np.empty(M, np.float64), np.empty(M, np.float64)
    rc = _load().ajo_sampled_rows(_code(W_lm), _ptr(hidden_t), M, _ptr(W_lm), V, d_t, float(inv_temperature),
                                  _ptr(row_key), _ptr(y), _ptr(m1), _ptr(m2))
    if rc:
        raise ValueError(f"ajo_sampled_rows rc={rc}")
    return y, m1, m2


def verify_sampled(hidden_t, hidden_d, W_lm, draft_tok, clf_w, clf_b, tau, inv_temperature, row_key,
                   feat_offset=1) -> VerifyResult:
    """The whole step with the target's tokens sampled (t_star holds the sampled tokens, max1/max2 the
    perturbed scores)."""
    draft_tok = _c(draft_tok, np.int32)
    B, K = draft_tok.shape
    W_lm, clf_w = _c(W_lm), _c(clf_w)
    V, d_t = W_lm.shape
    d_d = clf_w.shape[0] - d_t
    hidden_t = _c(hidden_t).reshape(B, K + 1, d_t)
    hidden_d = _c(hidden_d).reshape(B, K + 1, d_d) if d_d > 0 else None
    row_key = _c(row_key, np.uint64).reshape(B, K + 1)
    M = B * (K + 1)
    r = VerifyResult()
    r.out_len, r.out_tok = np.empty(B, np.int32), np.empty(B, np.int32)
    r.t_star, r.max1, r.max2 = np.empty(M, np.int32), np.empty(M, np.float64), np.empty(M, np.float64)
    r.near_tie = np.empty(M, np.uint8)
    r.mismatch, r.near_thr = np.empty((B, K), np.uint8), np.empty((B, K), np.uint8)
    r.z, r.p = np.empty((B, K), np.float64), np.empty((B, K), np.float64)
    rc = _load().ajo_verify_sampled(B, K, d_t, d_d, V, _code(W_lm), feat_offset,
                                    _ptr(hidden_t), _ptr(hidden_d), _ptr(W_lm), _ptr(draft_tok), _ptr(clf_w),
                                    float(clf_b), float(tau), float(inv_temperature), _ptr(row_key),
                                    _ptr(r.out_len), _ptr(r.out_tok), _ptr(r.t_star), _ptr(r.max1), _ptr(r.max2),
                                    _ptr(r.near_tie), _ptr(r.mismatch), _ptr(r.z), _ptr(r.p), _ptr(r.near_thr))
    if rc:
        raise ValueError(f"ajo_verify_sampled rc={rc}")
    return r


# ---- draft trees (Section 3.3 "Generality": the judge on a tree-based verification stage)

class TreeResult:
    __slots__ = ("out_len", "out_tok", "out_node", "t_star", "max1", "max2", "mismatch", "z", "p", "near_thr")


def walk_tree(hidden_t, hidden_d, t_star, draft_tok, parent, clf_w, clf_b, tau, feat_offset=1) -> TreeResult:
    """Longest accepted root-to-node path per window, given the greedy tokens t_star [B][K+1]."""
    draft_tok, parent = _c(draft_tok, np.int32), _c(parent, np.int32)
    B, K = draft_tok.shape
    assert parent.shape == (B, K)
    clf_w = _c(clf_w)
    t_star = _c(t_star, np.int32).reshape(B, K + 1)
    hidden_t = _c(hidden_t).reshape(B, K + 1, -1)
    d_t = hidden_t.shape[2]
    d_d = clf_w.shape[0] - d_t
    hidden_d = _c(hidden_d).reshape(B, K + 1, d_d) if d_d > 0 else None
    r = TreeResult()
    r.out_len, r.out_tok, r.out_node = np.empty(B, np.int32), np.empty(B, np.int32), np.empty(B, np.int32)
    r.mismatch, r.near_thr = np.empty((B, K), np.uint8), np.empty((B, K), np.uint8)
    r.z, r.p = np.empty((B, K), np.float64), np.empty((B, K), np.float64)
    rc = _load().ajo_walk_tree(B, K, d_t, d_d, _code(hidden_t), feat_offset, _ptr(hidden_t), _ptr(hidden_d),
                               _ptr(t_star), _ptr(draft_tok), _ptr(parent), _ptr(clf_w), float(clf_b), float(tau),
                               _ptr(r.out_len), _ptr(r.out_tok), _ptr(r.out_node),
                               _ptr(r.mismatch), _ptr(r.z), _ptr(r.p), _ptr(r.near_thr))
    if rc:
        raise ValueError(f"ajo_walk_tree rc={rc}")
    return r


def verify_tree(hidden_t, hidden_d, W_lm, draft_tok, parent, clf_w, clf_b, tau, feat_offset=1) -> TreeResult:
    """The whole step on draft trees, with diagnostics."""
    draft_tok, parent = _c(draft_tok, np.int32), _c(parent, np.int32)
    B, K = draft_tok.shape
    W_lm, clf_w = _c(W_lm), _c(clf_w)
    V, d_t = W_lm.shape
    d_d = clf_w.shape[0] - d_t
    hidden_t = _c(hidden_t).reshape(B, K + 1, d_t)
    hidden_d = _c(hidden_d).reshape(B, K + 1, d_d) if d_d > 0 else None
    M = B * (K + 1)
    r = TreeResult()
    r.out_len, r.out_tok, r.out_node = np.empty(B, np.int32), np.empty(B, np.int32), np.empty(B, np.int32)
    r.t_star, r.max1, r.max2 = np.empty(M, np.int32), np.empty(M, np.float64), np.empty(M, np.float64)
    r.mismatch, r.near_thr = np.empty((B, K), np.uint8), np.empty((B, K), np.uint8)
    r.z, r.p = np.empty((B, K), np.float64), np.empty((B, K), np.float64)
    rc = _load().ajo_verify_tree(B, K, d_t, d_d, V, _code(W_lm), feat_offset, _ptr(hidden_t), _ptr(hidden_d),
                                 _ptr(W_lm), _ptr(draft_tok), _ptr(parent), _ptr(clf_w), float(clf_b), float(tau),
                                 _ptr(r.out_len), _ptr(r.out_tok), _ptr(r.out_node),
                                 _ptr(r.t_star), _ptr(r.max1), _ptr(r.max2),
                                 _ptr(r.mismatch), _ptr(r.z), _ptr(r.p), _ptr(r.near_thr))
    if rc:
        raise ValueError(f"ajo_verify_tree rc={rc}")
    return r
