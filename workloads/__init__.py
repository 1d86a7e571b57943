"""Seeded synthetic speculation-window workloads.

The workloads are shaped like Llama-3-class draft/target pairs (the paper's
Section 4 model pairs and window sizes); they stand in for the paper's GSM8K /
LiveCodeBench speculation windows, which need datasets and trained weights.

This package only *draws inputs*.  It contains none of the verification
method's arithmetic and imports neither the CPU oracle nor the HIP library:
whatever depends on the target's greedy tokens (the draft tokens) takes those
tokens as an argument.

Storage types: ``bf16`` tensors are numpy ``uint16`` arrays holding the raw
bfloat16 bits, ``f32`` tensors are ``float32`` arrays.
"""
from __future__ import annotations

import ctypes
import dataclasses
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libwl.so")

F32, BF16 = 0, 1

# tensor ids of the counter-based generator (one stream per tensor)
TID_HIDDEN_T = 1
TID_HIDDEN_D = 2
TID_W_LM = 3
TID_CLF_W = 4
TID_DRAFT_MATCH = 5
TID_DRAFT_ALT = 6
TID_DRAFT_RUN = 7

DEFAULT_SEED = 20039


@dataclasses.dataclass(frozen=True)
class Workload:
    """One benchmark configuration (B windows of K draft tokens + 1 bonus row)."""

    name: str
    B: int
    K: int
    d_t: int
    d_d: int
    V: int
    dtype: str            # "f32" or "bf16": storage type of hidden states, W_lm, clf_w
    p_match: float        # probability that a draft token equals the target's greedy token
    clustered: bool       # mismatches come in runs of Geometric(0.5) length
    clf_b: float
    tau: float
    taus: tuple = ()

    @property
    def M(self) -> int:
        return self.B * (self.K + 1)

    @property
    def D(self) -> int:
        return self.d_t + self.d_d

    @property
    def dtype_code(self) -> int:
        return F32 if self.dtype == "f32" else BF16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


WORKLOADS = {
    w.name: w
    for w in [
        Workload("tiny_f32", 1, 8, 256, 128, 1024, "f32", 0.7, False, 0.0, 0.5),
        Workload("8b_b1_k16", 1, 16, 4096, 2048, 128256, "bf16", 0.8, False, 0.0, 0.5),
        Workload("8b_b32_k32", 32, 32, 4096, 2048, 128256, "bf16", 0.75, True, 0.0, 0.5,
                 (0.0, 0.3, 0.5, 1.0)),
        Workload("70b_b8_k32", 8, 32, 8192, 4096, 128256, "bf16", 0.7, False, -1.0, 0.5),
        Workload("70b_b128_k64", 128, 64, 8192, 4096, 128256, "bf16", 0.5, False, 0.0, 0.6),
        # the paper's own deployment shape (Section 4.1: window 64; the serving tables: window 32): one
        # sequence, a 70B-class target, recipe of the 70B batch-8 workload
        Workload("70b_b1_k32", 1, 32, 8192, 4096, 128256, "bf16", 0.7, False, -1.0, 0.5),
        Workload("70b_b1_k64", 1, 64, 8192, 4096, 128256, "bf16", 0.7, False, -1.0, 0.5),
    ]
}


def scaled(base: Workload, **kw) -> Workload:
    """A reduced or altered copy of a workload (same recipe, other sizes)."""
    return dataclasses.replace(base, **kw)


# --------------------------------------------------------------------------- build / load

def build(force: bool = False) -> str:
    """Compile gen.c into libwl.so with gcc (host code only)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u64 = ctypes.c_uint64
        lib.wl_uniform.argtypes = [u64, u64, u64, u64, ctypes.c_void_p]
        lib.wl_uniform.restype = None
        lib.wl_normal_rows.argtypes = [u64, u64, u64, u64, u64, ctypes.c_double,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        lib.wl_normal_rows.restype = ctypes.c_int
        _lib = lib
    return _lib


# --------------------------------------------------------------------------- raw draws

def uniform(seed: int, tensor_id: int, idx0: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.float64)
    _load().wl_uniform(seed, tensor_id, idx0, n, out.ctypes.data)
    return out


def normal_rows(seed: int, tensor_id: int, row0: int, rows: int, cols: int, std: float,
                rms_norm: bool, dtype: str) -> np.ndarray:
    out = np.empty((rows, cols), dtype=np.float32 if dtype == "f32" else np.uint16)
    rc = _load().wl_normal_rows(seed, tensor_id, row0, rows, cols, float(std), int(rms_norm),
                                F32 if dtype == "f32" else BF16, out.ctypes.data)
    if rc != 0:
        raise RuntimeError("wl_normal_rows failed")
    return out


def widen(a: np.ndarray) -> np.ndarray:
    """Exact conversion of a stored tensor (bf16 bits or fp32) to float64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------- workload tensors

def hidden_t(w: Workload, seed: int, row0: int = 0, rows: int | None = None) -> np.ndarray:
    """Target final hidden states, verify rows row0.. of [B*(K+1), d_t]; unit RMS per row."""
    rows = w.M - row0 if rows is None else rows
    return normal_rows(seed, TID_HIDDEN_T, row0, rows, w.d_t, 1.0, True, w.dtype)


def hidden_d(w: Workload, seed: int, row0: int = 0, rows: int | None = None) -> np.ndarray:
    """Draft final hidden states, rows row0.. of [B*(K+1), d_d]; unit RMS per row."""
    rows = w.M - row0 if rows is None else rows
    if w.d_d == 0:
        return np.empty((rows, 0), dtype=np.float32 if w.dtype == "f32" else np.uint16)
    return normal_rows(seed, TID_HIDDEN_D, row0, rows, w.d_d, 1.0, True, w.dtype)


def w_lm(w: Workload, seed: int, row0: int = 0, rows: int | None = None) -> np.ndarray:
    """LM-head rows row0.. of [V, d_t], N(0, 0.02^2)."""
    rows = w.V - row0 if rows is None else rows
    return normal_rows(seed, TID_W_LM, row0, rows, w.d_t, 0.02, False, w.dtype)


# OCP FP8 E4M3 storage of W_lm (the FP8 LM head of the paper's 405B run, Section 4): encode / decode are
# the library's (torch CPU); the decode is exact, so the oracle can be fed the decoded values as bf16 bits.

def fp8_e4m3_encode(x: np.ndarray) -> np.ndarray:
    """float array -> E4M3 bytes (uint8), round to nearest even."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def fp8_e4m3_to_bf16_bits(b: np.ndarray) -> np.ndarray:
    """E4M3 bytes -> the same values as bf16 bits (uint16); exact, E4M3 has 4 significant bits."""
    import torch
    f = torch.from_numpy(np.ascontiguousarray(b, np.uint8)).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    u = f.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0)
    return (u >> 16).astype(np.uint16)


def w_lm_fp8(w: Workload, seed: int):
    """(E4M3 bytes [V, d_t], scale): the bf16 workload's W_lm divided by a per-tensor scale that puts its
    largest magnitude at 440 (E4M3 tops out at 448), rounded to E4M3."""
    W = widen(w_lm(w, seed))
    scale = float(np.abs(W).max() / 440.0)
    return fp8_e4m3_encode(W / scale), scale


def clf_w(w: Workload, seed: int) -> np.ndarray:
    """Judge weights [d_t + d_d], N(0, 1/(d_t+d_d)); target part first."""
    return normal_rows(seed, TID_CLF_W, 0, 1, w.D, 1.0 / math.sqrt(w.D), False, w.dtype)[0]


def draft_tokens(w: Workload, seed: int, t_star: np.ndarray) -> np.ndarray:
    """Draft tokens [B, K] given the target's greedy tokens t_star [B, K+1].

    A slot is a *match* (draft token = t_star) with probability ``p_match``;
    otherwise the token is uniform over the vocabulary minus t_star.  With
    ``clustered`` the mismatching slots come in runs: outside a run a new run
    starts with probability q = 1/7 and lasts Geometric(0.5) slots (mean 2), which
    keeps the long-run mismatch fraction at 2q/(1+q) = 0.25.
    An entry t_star < 0 means "greedy token unknown": the slot gets a uniform token.
    """
    t_star = np.asarray(t_star).reshape(w.B, w.K + 1)
    n = w.B * w.K
    u_match = uniform(seed, TID_DRAFT_MATCH, 0, n).reshape(w.B, w.K)
    u_alt = uniform(seed, TID_DRAFT_ALT, 0, n).reshape(w.B, w.K)
    u_run = uniform(seed, TID_DRAFT_RUN, 0, n).reshape(w.B, w.K)
    mismatch = np.zeros((w.B, w.K), dtype=bool)
    if not w.clustered:
        mismatch = u_match >= w.p_match
    else:
        frac = 1.0 - w.p_match
        q = frac / (2.0 - frac)                 # 2q/(1+q) = frac
        for b in range(w.B):
            left = 0
            for j in range(w.K):
                if left > 0:
                    mismatch[b, j] = True
                    left -= 1
                elif u_match[b, j] < q:
                    mismatch[b, j] = True
                    left = int(math.floor(math.log(u_run[b, j]) / math.log(0.5)))
    out = np.empty((w.B, w.K), dtype=np.int32)
    for b in range(w.B):
        for j in range(w.K):
            t = int(t_star[b, j])
            if t < 0:
                out[b, j] = min(int(u_alt[b, j] * w.V), w.V - 1)
            elif not mismatch[b, j]:
                out[b, j] = t
            else:
                r = min(int(u_alt[b, j] * (w.V - 1)), w.V - 2)
                out[b, j] = r + (1 if r >= t else 0)
    return out
