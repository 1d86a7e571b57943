"""Pins of the CPU oracle against things other than itself (CPU only).

What pins what:
  hand example (tests/golden/hand_example.txt)  -> whole pipeline, feature row, concat order,
                                                   threshold direction, emission rule
  numpy fp64 matmul (library GEMM)              -> step 1 (ajo_logits_row, ajo_greedy_rows max)
  O(V^2) brute-force argmax + duplicate rows    -> step 2 and the lowest-index tie rule
  longest-common-prefix routine at tau = 0      -> steps 3-4 reduce to greedy speculative decoding
  tau = 1, all-match, slot-0 mismatch, clf_w=0  -> endpoints of steps 3-4
  prefix formulation without early exit         -> step 4 (ajo_walk), with numpy judge logits -> step 3
  exhaustive V=4, K=3                           -> steps 2-4 on every draft tuple
  symmetries (scale, permutation, dead half)    -> steps 1-3
  closed-form E[out_len] on synthetic windows   -> generator + steps 3-4 (statistical)
  log-odds closed forms                         -> ajo_threshold_logit
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers

def to_bf16_bits(x):
    """fp32 -> bf16 bits for values that are exactly representable (asserted)."""
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not exact in bf16"
    return (u >> 16).astype(np.uint16)


def store(x, dtype):
    return np.asarray(x, np.float32) if dtype == "f32" else to_bf16_bits(x)


def np_logits(h, W):
    return wl.widen(h) @ wl.widen(W).T            # library fp64 GEMM


def brute_argmax(l):
    """v is the greedy token iff nothing is larger and nothing equal sits before it."""
    V = len(l)
    winners = [v for v in range(V)
               if not any(l[u] > l[v] for u in range(V))
               and not any(l[u] == l[v] for u in range(v))]
    assert len(winners) == 1
    return winners[0]


def lcp_greedy(t_star, draft):
    """Textbook greedy speculative decoding: accept the common prefix, emit target token."""
    B, K = draft.shape
    out_len = np.zeros(B, np.int32)
    out_tok = np.zeros(B, np.int32)
    for b in range(B):
        n = 0
        while n < K and draft[b, n] == t_star[b, n]:
            n += 1
        out_len[b], out_tok[b] = n, t_star[b, n]
    return out_len, out_tok


def prefix_formulation(t_star, draft, z, zthr):
    """out_len = largest n <= K with every slot j < n either matching or judged unimportant."""
    B, K = draft.shape
    ok = (t_star[:, :K] == draft) | (z < zthr)
    out_len = np.array([max(n for n in range(K + 1) if ok[b, :n].all()) for b in range(B)], np.int32)
    out_tok = t_star[np.arange(B), out_len].astype(np.int32)
    return out_len, out_tok


def np_judge_z(ht, hd, cw, b, B, K, feat_offset):
    """Judge logit of every slot with numpy (library dot), [B, K]."""
    d_t = ht.shape[-1]
    x = np.concatenate([wl.widen(ht).reshape(B, K + 1, d_t),
                        wl.widen(hd).reshape(B, K + 1, -1)], axis=2)
    rows = x[:, feat_offset:feat_offset + K, :]
    return rows @ wl.widen(cw) + b


def small_case(seed, B=3, K=5, d_t=32, d_d=16, V=64, dtype="bf16", p_match=0.6, clf_b=0.0):
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], name="small", B=B, K=K, d_t=d_t, d_d=d_d, V=V,
                  dtype=dtype, p_match=p_match, clf_b=clf_b)
    ht, hd, W, cw = wl.hidden_t(w, seed), wl.hidden_d(w, seed), wl.w_lm(w, seed), wl.clf_w(w, seed)
    t, m1, m2 = oracle.greedy_rows(ht, W)
    draft = wl.draft_tokens(w, seed, t)
    return w, ht, hd, W, cw, t.reshape(B, K + 1), draft


# ----------------------------------------------------------------------------- hand example

def _parse_hand():
    vals, cases, zs = {}, [], []
    for line in open(os.path.join(GOLDEN, "hand_example.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, *rest = line.split()
        if key == "case":
            cases.append((int(rest[0]), float(rest[1]), int(rest[2]), int(rest[3])))
        elif key == "z":
            zs.append((int(rest[0]), float(rest[1]), float(rest[2])))
        else:
            vals[key] = [float(x) for x in rest]
    return vals, cases, zs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hand_example(dtype):
    vals, cases, zs = _parse_hand()
    W = store(np.array(vals["W_lm"]).reshape(4, 2), dtype)
    ht = store(np.array(vals["hidden_t"]).reshape(4, 2), dtype)
    hd = store(np.array(vals["hidden_d"]).reshape(4, 1), dtype)
    cw = store(vals["clf_w"], dtype)
    draft = np.array(vals["draft_tok"], np.int32).reshape(1, 3)
    t_expected = np.array(vals["t_star"], np.int32)
    assert len(cases) == 6 and len(zs) == 2
    for feat_offset, tau, exp_len, exp_tok in cases:
        r = oracle.verify(ht, hd, W, draft, cw, vals["clf_b"][0], tau, feat_offset=feat_offset)
        assert list(r.t_star) == list(t_expected)
        assert (int(r.out_len[0]), int(r.out_tok[0])) == (exp_len, exp_tok), (feat_offset, tau)
        assert list(r.mismatch[0]) == [0, 1, 0]
    for feat_offset, z, p in zs:
        r = oracle.verify(ht, hd, W, draft, cw, vals["clf_b"][0], 0.5, feat_offset=feat_offset)
        assert r.z[0, 1] == pytest.approx(z, abs=1e-12)
        assert r.p[0, 1] == pytest.approx(p, abs=1e-9)
        assert np.isnan(r.z[0, 0]) and np.isnan(r.z[0, 2])


# ----------------------------------------------------------------------------- step 1 / 2

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_logits_match_library_gemm(dtype):
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], dtype=dtype)
    ht, W = wl.hidden_t(w, 7), wl.w_lm(w, 7)
    ref = np_logits(ht, W)
    for r in range(w.M):
        got = oracle.logits_row(ht[r], W)
        assert np.max(np.abs(got - ref[r])) < 1e-12
    t, m1, m2 = oracle.greedy_rows(ht, W)
    assert np.array_equal(t, ref.argmax(axis=1))
    assert np.max(np.abs(m1 - ref.max(axis=1))) < 1e-12
    srt = np.sort(ref, axis=1)
    assert np.max(np.abs(m2 - srt[:, -2])) < 1e-12


def test_logits_not_transposed():
    """A rectangular W_lm with a known structure: only W[v, k] = [v == 3k] fits the definition."""
    d_t, V = 4, 12
    W = np.zeros((V, d_t), np.float32)
    for k in range(d_t):
        W[3 * k, k] = 1.0
    h = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    got = oracle.logits_row(h, W)
    exp = np.zeros(V)
    exp[[0, 3, 6, 9]] = [1, 2, 3, 4]
    assert np.array_equal(got, exp)


def test_argmax_bruteforce_and_ties():
    rng = np.random.default_rng(3)
    d_t, V = 8, 24
    for trial in range(20):
        # small integers: many exact ties, products and sums exact
        W = rng.integers(-2, 3, size=(V, d_t)).astype(np.float32)
        H = rng.integers(-2, 3, size=(6, d_t)).astype(np.float32)
        t, m1, m2 = oracle.greedy_rows(H, W)
        L = H.astype(np.float64) @ W.astype(np.float64).T
        for r in range(6):
            assert t[r] == brute_argmax(list(L[r]))
            others = np.delete(L[r], t[r])
            assert m1[r] == L[r].max() and m2[r] == others.max()
    # duplicated rows: the lowest copy wins, also at the two ends of the vocabulary
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], dtype="bf16")
    ht, W = wl.hidden_t(w, 11), wl.w_lm(w, 11).copy()
    t0, _, _ = oracle.greedy_rows(ht, W)
    W2 = W.copy()
    W2[w.V - 1] = W[t0[0]]                     # copy of row-0's winner at the last index
    W2[0] = W[t0[1]]                           # copy of row-1's winner at index 0
    t2, m1, m2 = oracle.greedy_rows(ht, W2)
    assert t2[0] == min(t0[0], w.V - 1) and t2[1] == 0
    assert m1[1] == m2[1]                      # exact tie is visible in the diagnostics
    assert oracle.near_tie(m1, m2)[1]


def test_negative_zero_ties_with_positive_zero():
    W = np.array([[-1.0], [1.0], [0.0]], np.float32)
    h = np.array([[0.0]], np.float32)          # logits (-0.0, +0.0, +0.0): all equal as IEEE values
    t, _, _ = oracle.greedy_rows(h, W)
    assert t[0] == 0


def test_single_token_vocabulary():
    W = np.array([[2.0, 1.0]], np.float32)
    h = np.array([[1.0, 1.0]], np.float32)
    t, m1, m2 = oracle.greedy_rows(h, W)
    assert t[0] == 0 and m1[0] == 3.0 and m2[0] == -np.inf


# ----------------------------------------------------------------------------- steps 3 / 4

def test_threshold_logit_closed_forms():
    assert oracle.threshold_logit(0.5) == 0.0
    assert oracle.threshold_logit(0.0) == -np.inf and oracle.threshold_logit(1.0) == np.inf
    for tau in [0.005, 0.06, 0.145, 0.23, 0.9]:
        z = oracle.threshold_logit(tau)
        assert 1.0 / (1.0 + math.exp(-z)) == pytest.approx(tau, rel=1e-14)
        assert oracle.threshold_logit(1.0 - tau) == pytest.approx(-z, rel=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("feat_offset", [0, 1])
def test_walk_matches_prefix_formulation(dtype, feat_offset):
    for seed in [1, 2, 3]:
        w, ht, hd, W, cw, t, draft = small_case(seed, B=6, K=7, dtype=dtype, p_match=0.5)
        z_np = np_judge_z(ht, hd, cw, 0.25, w.B, w.K, feat_offset)
        for tau in [0.0, 0.2, 0.5, 0.56, 0.8, 1.0]:
            r = oracle.walk(ht, hd, t, draft, cw, 0.25, tau, feat_offset=feat_offset)
            exp_len, exp_tok = prefix_formulation(t, draft, z_np, oracle.threshold_logit(np.float32(tau)))
            assert np.array_equal(r.out_len, exp_len) and np.array_equal(r.out_tok, exp_tok)
            mis = t[:, :w.K] != draft
            assert np.array_equal(r.mismatch.astype(bool), mis)
            assert np.allclose(r.z[mis], z_np[mis], atol=1e-12, rtol=0)
            assert np.allclose(r.p[mis], 1 / (1 + np.exp(-z_np[mis])), atol=1e-12, rtol=0)
            assert np.isnan(r.z[~mis]).all()
            assert np.all(r.out_len <= w.K) and np.all(r.out_len >= 0)


def test_tau0_is_greedy_speculative_decoding_and_tau1_accepts_all():
    for seed in [4, 5]:
        w, ht, hd, W, cw, t, draft = small_case(seed, B=8, K=9, p_match=0.7)
        full = oracle.verify(ht, hd, W, draft, cw, 0.0, 0.0)
        assert np.array_equal(full.t_star.reshape(w.B, w.K + 1), t)
        exp_len, exp_tok = lcp_greedy(t, draft)
        assert np.array_equal(full.out_len, exp_len) and np.array_equal(full.out_tok, exp_tok)
        # tau = 1 with a hostile classifier (huge positive logits): still everything accepted
        r = oracle.walk(ht, hd, t, draft, cw, 1e30, 1.0)
        assert np.all(r.out_len == w.K) and np.array_equal(r.out_tok, t[:, w.K])
        # tau = 0 with a classifier that calls everything unimportant: still plain greedy
        r = oracle.walk(ht, hd, t, draft, cw, -1e30, 0.0)
        assert np.array_equal(r.out_len, exp_len)


def test_boundaries_all_match_and_first_slot():
    w, ht, hd, W, cw, t, draft = small_case(6, B=4, K=6)
    allmatch = t[:, :w.K].copy()
    r = oracle.walk(ht, hd, t, allmatch, cw, 5.0, 0.3)
    assert np.all(r.out_len == w.K) and np.array_equal(r.out_tok, t[:, w.K])
    assert not r.mismatch.any()
    bad0 = allmatch.copy()
    bad0[:, 0] = (bad0[:, 0] + 1) % w.V
    r = oracle.walk(ht, hd, t, bad0, cw, 0.0, 0.0)
    assert np.all(r.out_len == 0) and np.array_equal(r.out_tok, t[:, 0])
    lastbad = allmatch.copy()
    lastbad[:, w.K - 1] = (lastbad[:, w.K - 1] + 1) % w.V
    r = oracle.walk(ht, hd, t, lastbad, cw, 0.0, 0.0)
    assert np.all(r.out_len == w.K - 1) and np.array_equal(r.out_tok, t[:, w.K - 1])
    # out-of-vocabulary draft tokens simply never match
    oov = np.full_like(allmatch, w.V + 5)
    r = oracle.walk(ht, hd, t, oov, cw, 0.0, 0.0)
    assert np.all(r.out_len == 0)


def test_zero_classifier_reduces_to_the_endpoints():
    w, ht, hd, W, cw, t, draft = small_case(8, B=5, K=8, p_match=0.5)
    zero = np.zeros_like(cw)
    exp_len, exp_tok = lcp_greedy(t, draft)
    # sigmoid(b) = 0.2689 for b = -1
    r = oracle.walk(ht, hd, t, draft, zero, -1.0, 0.3)
    assert np.all(r.out_len == w.K)
    r = oracle.walk(ht, hd, t, draft, zero, -1.0, 0.25)
    assert np.array_equal(r.out_len, exp_len) and np.array_equal(r.out_tok, exp_tok)
    assert np.allclose(r.p[r.mismatch.astype(bool)], 1 / (1 + math.e), atol=1e-15)
    # strictness: p == tau rejects (b = 0 -> p = 0.5 exactly, logit(0.5) = 0)
    r = oracle.walk(ht, hd, t, draft, zero, 0.0, 0.5)
    assert np.array_equal(r.out_len, exp_len)


def test_monotone_in_tau():
    w, ht, hd, W, cw, t, draft = small_case(9, B=16, K=12, p_match=0.5)
    prev = None
    for tau in np.linspace(0, 1, 21):
        r = oracle.walk(ht, hd, t, draft, cw, 0.0, float(tau))
        if prev is not None:
            assert np.all(r.out_len >= prev)
        prev = r.out_len.copy()
    assert np.all(prev == w.K)


def test_exhaustive_tiny_window():
    vals, _, _ = _parse_hand()
    W = np.array(vals["W_lm"], np.float32).reshape(4, 2)
    ht = np.array(vals["hidden_t"], np.float32).reshape(4, 2)
    hd = np.array(vals["hidden_d"], np.float32).reshape(4, 1)
    cw = np.array(vals["clf_w"], np.float32)
    t = np.array(vals["t_star"], np.int32).reshape(1, 4)
    for fo in [0, 1]:
        z_np = np_judge_z(ht, hd, cw, 0.0, 1, 3, fo)
        for draft in itertools.product(range(4), repeat=3):
            d = np.array(draft, np.int32).reshape(1, 3)
            for tau in [0.0, 0.25, 0.5, 0.75, 1.0]:
                r = oracle.verify(ht, hd, W, d, cw, 0.0, tau, feat_offset=fo)
                exp_len, exp_tok = prefix_formulation(t, d, z_np, oracle.threshold_logit(tau))
                assert (r.out_len[0], r.out_tok[0]) == (exp_len[0], exp_tok[0]), (fo, draft, tau)


# ----------------------------------------------------------------------------- symmetries

def test_symmetries():
    w, ht, hd, W, cw, t, draft = small_case(10, B=6, K=8, V=96, p_match=0.5)
    base = oracle.verify(ht, hd, W, draft, cw, 0.1, 0.55)
    # scaling W_lm by a power of two is exact in bf16: nothing changes
    W4 = (wl.widen(W) * 4.0).astype(np.float32)
    W4b = (W4.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(wl.widen(W4b), W4.astype(np.float64))
    s = oracle.verify(ht, hd, W4b, draft, cw, 0.1, 0.55)
    assert np.array_equal(s.out_len, base.out_len) and np.array_equal(s.out_tok, base.out_tok)
    assert np.allclose(s.max1, 4 * base.max1, rtol=1e-15)
    # relabelling the vocabulary (no exact ties here) relabels the emitted token
    assert (base.max1 > base.max2).all()
    perm = np.random.default_rng(0).permutation(w.V)          # new row i holds old row perm[i]
    inv = np.argsort(perm)                                    # old token v becomes inv[v]
    p = oracle.verify(ht, hd, W[perm], inv[draft].astype(np.int32), cw, 0.1, 0.55)
    assert np.array_equal(p.out_len, base.out_len)
    assert np.array_equal(p.out_tok, inv[base.out_tok])
    # a classifier with a dead draft half ignores hidden_d
    cw_dead = cw.copy()
    cw_dead[w.d_t:] = 0
    a = oracle.verify(ht, hd, W, draft, cw_dead, 0.1, 0.55)
    b = oracle.verify(ht, wl.hidden_d(w, 999), W, draft, cw_dead, 0.1, 0.55)
    assert np.array_equal(a.out_len, b.out_len) and np.array_equal(a.z[a.mismatch == 1], b.z[b.mismatch == 1])
    # ... and one with a dead target half ignores hidden_t in the judge
    cw_dead = cw.copy()
    cw_dead[:w.d_t] = 0
    z_np = wl.widen(hd).reshape(w.B, w.K + 1, -1)[:, 1:, :] @ wl.widen(cw)[w.d_t:] + 0.1
    a = oracle.verify(ht, hd, W, draft, cw_dead, 0.1, 0.55)
    m = a.mismatch.astype(bool)
    assert np.allclose(a.z[m], z_np[m], atol=1e-12)


# ----------------------------------------------------------------------------- statistics

def _phi(x):
    return 0.5 * (1.0 + math.erf(x / math.sqrt(2.0)))


@pytest.mark.parametrize("p_match,clf_b,tau", [(0.5, 0.0, 0.6), (0.7, -1.0, 0.5)])
def test_expected_accepted_length_closed_form(p_match, clf_b, tau):
    """iid slots: reject prob rho = (1-p_match)(1-a), a = Phi((logit tau - b)/|w|);
    E[out_len] = (1-rho)(1-(1-rho)^K)/rho for a window of K slots."""
    B, K = 600, 32
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], name="stat", B=B, K=K, d_t=64, d_d=32, V=256,
                  dtype="bf16", p_match=p_match, clf_b=clf_b, tau=tau)
    seed = 77
    ht, hd, W, cw = wl.hidden_t(w, seed), wl.hidden_d(w, seed), wl.w_lm(w, seed), wl.clf_w(w, seed)
    t, _, _ = oracle.greedy_rows(ht, W)
    draft = wl.draft_tokens(w, seed, t)
    realised = (draft == t.reshape(B, K + 1)[:, :K]).mean()
    assert abs(realised - p_match) < 4 * math.sqrt(p_match * (1 - p_match) / (B * K))
    r = oracle.walk(ht, hd, t, draft, cw, clf_b, tau)
    norm = float(np.linalg.norm(wl.widen(cw)))
    a = _phi((oracle.threshold_logit(tau) - clf_b) / norm)
    rho = (1 - p_match) * (1 - a)
    q = 1 - rho
    mean = q * (1 - q ** K) / rho
    # variance of min(Geometric, K) is below that of the untruncated geometric
    se = math.sqrt(q / rho ** 2 / B)
    assert abs(r.out_len.mean() - mean) < 4 * se, (r.out_len.mean(), mean, se)


def test_near_flags():
    w, ht, hd, W, cw, t, draft = small_case(12, B=4, K=6, p_match=0.3)
    r = oracle.verify(ht, hd, W, draft, cw, 0.0, 0.5)
    assert np.array_equal(r.near_tie.astype(bool), (r.max1 - r.max2) < 1e-3 * np.abs(r.max1))
    m = r.mismatch.astype(bool)
    assert np.array_equal(r.near_thr[m].astype(bool), np.abs(r.z[m]) < 1e-4 * np.maximum(1, np.abs(r.z[m])))
    # a slot whose logit sits on the threshold is flagged
    zero = np.zeros_like(cw)
    r = oracle.walk(ht, hd, t, draft, zero, 0.0, 0.5)
    assert r.near_thr[m].all() and not r.near_thr[~m].any()


def test_bad_arguments_are_refused():
    w, ht, hd, W, cw, t, draft = small_case(13)
    for tau in [-0.1, 1.5, float("nan")]:
        with pytest.raises(ValueError):
            oracle.walk(ht, hd, t, draft, cw, 0.0, tau)
    with pytest.raises(ValueError):
        oracle.walk(ht, hd, t, draft, cw, 0.0, 0.5, feat_offset=2)
