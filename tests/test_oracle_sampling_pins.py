"""Pins of the oracle's sampling mode (Appendix A, "Generalization to sampling": the next token is
argmax_i log P(i) + Gumbel noise drawn from a generator seeded by the random state and the context)
against things other than itself (CPU only).

  closed-form Gumbel CDF exp(-exp(-x)) (Kolmogorov-Smirnov)      -> ajo_gumbel: transform, range, uniformity of the bits
  Gumbel-max theorem: token frequencies == softmax(logit / T)   -> ajo_sampled_rows: sign of the noise, direction of T
  T -> 0 is greedy decoding; 1/T = 0 is the uniform distribution -> endpoints of the temperature
  numpy GEMM + numpy argmax on the perturbed scores              -> assembly of ajo_sampled_rows (row keys, tie rule)
  walk of the sampled tokens == ajo_walk; hand example at T -> 0 -> ajo_verify_sampled is the greedy pipeline on y
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle
import workloads as wl


def test_gumbel_matches_closed_form_cdf():
    rng = np.random.default_rng(0)
    keys = rng.integers(0, 2**63, size=40, dtype=np.uint64)
    x = np.array([oracle.gumbel(int(k), v) for k in keys for v in range(500)])
    assert np.isfinite(x).all()
    d, p = stats.kstest(x, lambda t: np.exp(-np.exp(-t)))
    assert p > 1e-3, (d, p)
    # mean = Euler-Mascheroni constant, variance = pi^2 / 6
    assert abs(x.mean() - 0.5772156649) < 4 * math.sqrt(math.pi ** 2 / 6 / len(x))
    assert abs(x.var() - math.pi ** 2 / 6) < 0.1
    # one key, consecutive vocabulary entries: no serial correlation; two keys: unrelated streams
    a = np.array([oracle.gumbel(12345, v) for v in range(20000)])
    b = np.array([oracle.gumbel(12346, v) for v in range(20000)])
    assert abs(np.corrcoef(a[:-1], a[1:])[0, 1]) < 0.03
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.03
    assert stats.kstest(a, lambda t: np.exp(-np.exp(-t))).pvalue > 1e-3
    # both halves of the 64-bit key matter: keys that differ only in the upper, or only in the lower, 32 bits
    # give unrelated streams
    base = 0x0123456789ABCDEF
    c = np.array([oracle.gumbel(base, v) for v in range(5000)])
    for bit in range(64):
        e = np.array([oracle.gumbel(base ^ (1 << bit), v) for v in range(5000)])
        assert not np.array_equal(c, e) and abs(np.corrcoef(c, e)[0, 1]) < 0.06, bit
    e = np.array([oracle.gumbel(base + 1, v) for v in range(5000)])
    assert abs(np.corrcoef(c, e)[0, 1]) < 0.06


def test_generator_bit_pattern_matches_the_worked_values():
    """tests/golden/noise_bits.txt holds (key, v) -> h, n, u worked from the generator's published text (include/aj.h)
    with unbounded integers; the oracle's noise must be -log(-log(u)) of exactly that u, and the n recovered
    from the oracle's value must be the stored integer (adjacent values of n differ by >= 6e-8 relative in
    -log u, far above fp64 rounding)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "noise_bits.txt")
    cases = [l.split() for l in open(path) if not l.startswith("#")]
    assert len(cases) >= 8
    for key_hex, v, h_hex, n, num in cases:
        key, v, h, n, num = int(key_hex, 16), int(v), int(h_hex, 16), int(n), int(num)
        assert n == h >> 9 and num == 2 * n + 1
        u = num / 16777216.0                       # exact in fp64
        g = oracle.gumbel(key, v)
        assert g == pytest.approx(-math.log(-math.log(u)), rel=1e-13, abs=1e-13), (key_hex, v)
        n_back = math.exp(-math.exp(-g)) * 8388608.0 - 0.5
        assert round(n_back) == n and abs(n_back - n) < 1e-3, (key_hex, v, n_back)


@pytest.mark.parametrize("inv_t", [1.0, 0.5, 2.5])
def test_token_frequencies_are_the_softmax(inv_t):
    V, d, N = 7, 4, 40000
    rng = np.random.default_rng(5)
    W = rng.standard_normal((V, d)).astype(np.float32)
    h = rng.standard_normal((1, d)).astype(np.float32)
    logits = (wl.widen(h) @ wl.widen(W).T)[0]
    p = np.exp(logits * inv_t - (logits * inv_t).max())
    p /= p.sum()
    H = np.repeat(h, N, axis=0)
    keys = rng.integers(0, 2**63, size=N, dtype=np.uint64)
    y, _, _ = oracle.sampled_rows(H, W, inv_t, keys)
    counts = np.bincount(y, minlength=V)
    chi2, pval = stats.chisquare(counts, N * p)
    assert pval > 1e-3, (counts, N * p)
    # a wrong direction of the temperature (T instead of 1/T) or noise subtracted instead of added would not fit
    q = np.exp(logits / inv_t - (logits / inv_t).max())
    q /= q.sum()
    if inv_t != 1.0:
        assert stats.chisquare(counts, N * q).pvalue < 1e-6


def test_temperature_endpoints():
    rng = np.random.default_rng(7)
    V, d, M = 50, 16, 64
    W = rng.standard_normal((V, d)).astype(np.float32)
    H = rng.standard_normal((M, d)).astype(np.float32)
    keys = rng.integers(0, 2**63, size=M, dtype=np.uint64)
    g = oracle.greedy_rows(H, W)[0]
    y, m1, m2 = oracle.sampled_rows(H, W, 1e9, keys)          # T -> 0: the noise cannot change the order
    assert np.array_equal(y, g)
    # 1/T = 0: pure noise, every token equally likely
    N = 20000
    y0, _, _ = oracle.sampled_rows(np.repeat(H[:1], N, axis=0), W[:8], 0.0,
                                   rng.integers(0, 2**63, size=N, dtype=np.uint64))
    assert stats.chisquare(np.bincount(y0, minlength=8)).pvalue > 1e-3
    with pytest.raises(ValueError):
        oracle.sampled_rows(H, W, -1.0, keys)


def test_assembly_against_numpy():
    rng = np.random.default_rng(9)
    V, d, M = 33, 24, 10
    W = (0.3 * rng.standard_normal((V, d))).astype(np.float32)
    W[20] = W[3]                                              # equal logits, different noise: no tie expected
    H = rng.standard_normal((M, d)).astype(np.float32)
    keys = rng.integers(0, 2**63, size=M, dtype=np.uint64)
    keys[4] = keys[5]                                         # same key, different rows
    inv_t = 1.7
    L = wl.widen(H) @ wl.widen(W).T
    G = np.array([[oracle.gumbel(int(k), v) for v in range(V)] for k in keys])
    S = L * inv_t + G
    y, m1, m2 = oracle.sampled_rows(H, W, inv_t, keys)
    assert np.array_equal(y, S.argmax(axis=1))
    np.testing.assert_allclose(m1, S.max(axis=1), rtol=1e-12)
    np.testing.assert_allclose(m2, np.sort(S, axis=1)[:, -2], rtol=1e-12)
    assert np.array_equal(G[4], G[5])                         # the noise depends on (key, v) only


def test_whole_step_is_the_greedy_pipeline_on_sampled_tokens():
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], name="s", B=6)
    seed = 3
    ht, hd, W, cw = wl.hidden_t(w, seed), wl.hidden_d(w, seed), wl.w_lm(w, seed), wl.clf_w(w, seed)
    rng = np.random.default_rng(1)
    keys = rng.integers(0, 2**63, size=(w.B, w.K + 1), dtype=np.uint64)
    inv_t = 8.0
    y, m1, m2 = oracle.sampled_rows(ht, W, inv_t, keys.reshape(-1))
    assert (y != oracle.greedy_rows(ht, W)[0]).any()          # the noise does change some tokens here
    draft = wl.draft_tokens(w, seed, y)
    for tau in (0.0, 0.4, 1.0):
        r = oracle.verify_sampled(ht, hd, W, draft, cw, 0.0, tau, inv_t, keys)
        ref = oracle.walk(ht, hd, y.reshape(w.B, w.K + 1), draft, cw, 0.0, tau)
        assert np.array_equal(r.t_star, y)
        assert np.array_equal(r.out_len, ref.out_len) and np.array_equal(r.out_tok, ref.out_tok)
    # T -> 0 reproduces the greedy step on the same inputs
    g = oracle.greedy_rows(ht, W)[0]
    draft = wl.draft_tokens(w, seed, g)
    a = oracle.verify_sampled(ht, hd, W, draft, cw, 0.0, 0.5, 1e9, keys)
    b = oracle.verify(ht, hd, W, draft, cw, 0.0, 0.5)
    assert np.array_equal(a.out_len, b.out_len) and np.array_equal(a.out_tok, b.out_tok)
