"""Shared machinery of the GPU parity tests: run libaj and the oracle on the same seeded inputs
and compare them to the stated bars.

Bars (from the benchmark spec):
  - accepted lengths and emitted tokens bit-exact, except where the oracle flags a near-tie
    (top-2 logit gap < 1e-3 |max logit|) - those rows are counted, the GPU's choice must itself be
    within that band, and the oracle's steps 3-4 are replayed with the GPU's token on those rows;
  - max logit within 1e-2 relative; judge probability within 1e-3 absolute (logit too);
  - a window whose outcome hinges on a slot with |z - logit(tau)| < 1e-4 max(1,|z|) is counted
    as near-threshold instead of compared (the two sides accumulate z in different precisions).
"""
from __future__ import annotations

import hashlib
import os

import numpy as np

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


class Inputs:
    pass


def make_inputs(w, seed):
    x = Inputs()
    x.w, x.seed = w, seed
    x.ht, x.hd = wl.hidden_t(w, seed), wl.hidden_d(w, seed)
    x.W, x.cw = wl.w_lm(w, seed), wl.clf_w(w, seed)
    return x


def _digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


class GoldenMismatch(AssertionError):
    """A stored oracle file exists but was made from other inputs than the regenerated ones."""


def read_golden(name, seed):
    """(digests, rows) of a stored oracle file, or None when there is no such file."""
    path = os.path.join(GOLDEN, f"greedy_{name}_seed{seed}.txt")
    if not os.path.exists(path):
        return None
    sha, rows = {}, []
    for line in open(path):
        if line.startswith("#"):
            continue
        p = line.split()
        if p[0] == "sha256":
            sha[p[1]] = p[2]
        else:
            rows.append((int(p[1]), float(p[2]), float(p[3])))
    return sha, rows


def load_golden(x):
    """Stored oracle greedy rows for a full-size workload; None only when no file is stored.

    A stored file whose digests or row count do not fit the regenerated inputs is an error (GoldenMismatch names
    the tensor): silently comparing fewer rows instead would hide which check ran."""
    got = read_golden(x.w.name, x.seed)
    if got is None:
        return None
    sha, rows = got
    if len(rows) != x.w.M:
        raise GoldenMismatch(f"golden file of {x.w.name} holds {len(rows)} rows, the workload has {x.w.M}")
    for name, arr in (("hidden_t", x.ht), ("W_lm", x.W), ("hidden_d", x.hd), ("clf_w", x.cw)):
        if sha.get(name) != _digest(arr):
            raise GoldenMismatch(f"golden file of {x.w.name}: regenerated {name} differs from the tensor the "
                                 f"stored oracle rows were computed from (sha256 {sha.get(name)} stored, "
                                 f"{_digest(arr)} regenerated)")
    t = np.array([r[0] for r in rows], np.int32)
    m1 = np.array([r[1] for r in rows], np.float64)
    m2 = np.array([r[2] for r in rows], np.float64)
    return t, m1, m2


def oracle_greedy(x, windows=None):
    """Oracle steps 1-2. windows=None: all rows. Else only those windows; other rows get t = -1."""
    w = x.w
    if windows is None:
        return oracle.greedy_rows(x.ht, x.W)
    t = np.full(w.M, -1, np.int32)
    m1 = np.full(w.M, np.nan)
    m2 = np.full(w.M, np.nan)
    R = w.K + 1
    for b in windows:
        tt, a, c = oracle.greedy_rows(x.ht[b * R:(b + 1) * R], x.W)
        t[b * R:(b + 1) * R], m1[b * R:(b + 1) * R], m2[b * R:(b + 1) * R] = tt, a, c
    return t, m1, m2


def run_gpu(x, draft, tau, feat_offset=1, kernel=0, clf_b=None, flags=None, repeat=1, sampled=None, w8=None):
    """One aj_verify (or, with sampled = (inv_temperature, row_key [B][K+1] uint64), aj_verify_sampled) through the
    C ABI; returns dict of host arrays.  w8: W_lm as FP8 E4M3 bytes (x.W then holds the same values as bf16 bits
    for the oracle)."""
    import torch
    import paper_2504_20039_amd as aj
    w = x.w
    clf_b = w.clf_b if clf_b is None else clf_b
    flags = aj.AJ_FLAG_DEBUG if flags is None else flags
    dev = [aj.device_tensor(a) for a in (x.ht, x.hd, x.W if w8 is None else w8, np.ascontiguousarray(draft, np.int32), x.cw)]
    out_len = torch.full((max(w.B, 1),), -7, dtype=torch.int32, device="cuda")
    out_tok = torch.full((max(w.B, 1),), -7, dtype=torch.int32, device="cuda")
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, feat_offset, flags, kernel,
                     aj.AJ_W_SAME if w8 is None else aj.AJ_W_FP8_E4M3)
    d_key = torch.from_numpy(np.ascontiguousarray(sampled[1], np.uint64).view(np.int64)).cuda() if sampled else None
    try:
        name = aj.aj_kernel_name(h)
        outs = []
        for _ in range(repeat):
            out_len.fill_(-7)
            out_tok.fill_(-7)
            if sampled:
                aj.aj_verify_sampled(h, dev[0], dev[1] if w.d_d > 0 else None, dev[2], dev[3], dev[4], clf_b, tau,
                                     sampled[0], d_key, out_len, out_tok)
            else:
                aj.aj_verify(h, dev[0], dev[1] if w.d_d > 0 else None, dev[2], dev[3], dev[4], clf_b, tau,
                             out_len, out_tok)
            torch.cuda.synchronize()
            t_star, maxlogit, score = aj.aj_debug_copy(h, w.B, w.K, want_score=bool(flags & aj.AJ_FLAG_DEBUG))
            outs.append(dict(out_len=out_len.cpu().numpy()[:w.B].copy(), out_tok=out_tok.cpu().numpy()[:w.B].copy(),
                             t_star=t_star, maxlogit=maxlogit, score=score, kernel=name))
    finally:
        aj.aj_destroy(h)
    for o in outs[1:]:
        for k in ("out_len", "out_tok", "t_star", "maxlogit"):
            assert np.array_equal(o[k], outs[0][k]), f"run-to-run difference in {k}"
    return outs[0]


def compare(x, draft, tau, greedy, gpu, feat_offset=1, clf_b=None, windows=None, scores_row=None):
    """Assert parity of one GPU result with the oracle; returns the counts that are reported.
    greedy = the oracle's (token, max, runner-up) per row; scores_row(r) = the oracle's scores of row r over the
    vocabulary (default: its logits; the sampling tests pass the perturbed scores)."""
    w = x.w
    clf_b = w.clf_b if clf_b is None else clf_b
    t, m1, m2 = greedy
    R = w.K + 1
    win = np.arange(w.B) if windows is None else np.asarray(sorted(windows))
    rows = (win[:, None] * R + np.arange(R)[None, :]).reshape(-1)
    rep = dict(rows=len(rows), windows=len(win), near_tie_rows=0, near_tie_differ=0, near_thr_windows=0,
               kernel=gpu["kernel"])
    if len(rows) == 0:
        return rep

    # ---- step 2: greedy tokens
    flag = oracle.near_tie(m1[rows], m2[rows])
    rep["near_tie_rows"] = int(flag.sum())
    g_t = gpu["t_star"][rows]
    differ = g_t != t[rows]
    assert not (differ & ~flag).any(), \
        f"greedy token differs on unflagged rows {rows[differ & ~flag][:10]}"
    t_replay = t.copy()
    for r in rows[differ]:
        lg = oracle.logits_row(x.ht[r], x.W) if scores_row is None else scores_row(r)
        assert 0 <= gpu["t_star"][r] < w.V
        assert lg[gpu["t_star"][r]] >= m1[r] - 1e-3 * abs(m1[r]), f"row {r}: GPU token is not a near-tie"
        t_replay[r] = gpu["t_star"][r]
    rep["near_tie_differ"] = int(differ.sum())
    # ---- step 1 (what is visible of it): the maximum logit
    relerr = np.abs(gpu["maxlogit"][rows] - m1[rows]) / np.abs(m1[rows])
    assert relerr.max() <= 1e-2, f"max logit off by {relerr.max():.3g} relative"
    rep["maxlogit_relerr"] = float(relerr.max())

    # ---- steps 3-4, replayed on the GPU's tokens where a flagged row differed
    t_fill = np.where(t_replay < 0, 0, t_replay)
    ref = oracle.walk(x.ht, x.hd, t_fill, draft, x.cw, clf_b, tau, feat_offset)
    mis = ref.mismatch.astype(bool)[win]
    if gpu["score"] is not None:
        gz, gp = gpu["score"][0][win], gpu["score"][1][win]
        assert np.isnan(gz[~mis]).all() and np.isnan(gp[~mis]).all(), "score set at a matching slot"
        if mis.any():
            assert np.abs(gp[mis] - ref.p[win][mis]).max() <= 1e-3
            assert np.abs(gz[mis] - ref.z[win][mis]).max() <= 1e-3
            rep["score_abserr"] = float(np.abs(gp[mis] - ref.p[win][mis]).max())
    g_len, g_tok = gpu["out_len"][win], gpu["out_tok"][win]
    o_len, o_tok = ref.out_len[win], ref.out_tok[win]
    assert ((g_len >= 0) & (g_len <= w.K)).all()
    bad = (g_len != o_len) | (g_tok != o_tok)
    if bad.any():
        nthr = ref.near_thr.astype(bool)[win]
        for i in np.nonzero(bad)[0]:
            upto = max(g_len[i], o_len[i])
            assert nthr[i, :min(upto + 1, w.K)].any(), \
                f"window {win[i]}: GPU ({g_len[i]},{g_tok[i]}) != oracle ({o_len[i]},{o_tok[i]})"
            rep["near_thr_windows"] += 1
        assert rep["near_thr_windows"] <= 1 + len(win) // 100
    # emitted token is the GPU's own greedy token at the accepted length
    assert np.array_equal(g_tok, gpu["t_star"][win * R + g_len])
    return rep


def parity_case(w, seed, tau=None, feat_offset=1, kernel=0, greedy=None, windows=None, clf_b=None,
                draft=None, repeat=1):
    """Inputs -> oracle -> GPU -> compare. Returns (report, inputs, draft, greedy, gpu)."""
    tau = w.tau if tau is None else tau
    x = make_inputs(w, seed)
    if greedy is None:
        greedy = oracle_greedy(x, windows)
    if draft is None:
        draft = wl.draft_tokens(w, seed, greedy[0])
    gpu = run_gpu(x, draft, tau, feat_offset, kernel, clf_b, repeat=repeat)
    rep = compare(x, draft, tau, greedy, gpu, feat_offset, clf_b, windows)
    return rep, x, draft, greedy, gpu
