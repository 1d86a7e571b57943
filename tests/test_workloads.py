"""The seeded input generator: determinism, independence of the chunking, the recipe's statistics."""
import math

import numpy as np
import pytest
import torch

import workloads as wl


def test_same_seed_same_bytes_and_chunks_agree():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], V=300)
    a = wl.w_lm(w, 5)
    b = wl.w_lm(w, 5)
    assert a.dtype == np.uint16 and np.array_equal(a, b)
    part = wl.w_lm(w, 5, row0=117, rows=40)
    assert np.array_equal(part, a[117:157])
    assert not np.array_equal(a, wl.w_lm(w, 6))
    h = wl.hidden_t(w, 5)
    assert np.array_equal(wl.hidden_t(w, 5, row0=3, rows=2), h[3:5])
    # streams of different tensors differ
    assert not np.array_equal(wl.hidden_t(w, 5)[:, :64], wl.hidden_d(w, 5)[:, :64])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recipe_statistics(dtype):
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], dtype=dtype, B=8, K=15, d_t=512, d_d=256, V=2048)
    ht, hd, W, cw = (wl.widen(x) for x in (wl.hidden_t(w, 1), wl.hidden_d(w, 1), wl.w_lm(w, 1), wl.clf_w(w, 1)))
    tol = 3e-3 if dtype == "bf16" else 1e-6
    assert np.allclose(np.sqrt((ht ** 2).mean(axis=1)), 1.0, atol=tol)
    assert np.allclose(np.sqrt((hd ** 2).mean(axis=1)), 1.0, atol=tol)
    n = W.size
    assert abs(W.mean()) < 5 * 0.02 / math.sqrt(n)
    assert abs(W.std() - 0.02) < 0.02 * 5 / math.sqrt(2 * n) + 1e-4
    assert abs(cw.std() * math.sqrt(w.D) - 1.0) < 0.15
    # normality: fourth moment of a standard normal is 3
    z = W / 0.02
    assert abs((z ** 4).mean() - 3.0) < 0.05


def test_bf16_rounding_is_nearest_even():
    w32 = wl.scaled(wl.WORKLOADS["tiny_f32"], V=64)
    w16 = wl.scaled(w32, dtype="bf16")
    a32 = wl.w_lm(w32, 9)
    a16 = wl.w_lm(w16, 9)
    ref = torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(a16, ref)


def test_draft_tokens_iid_and_alternative_token_rule():
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=200, K=16, V=7, p_match=0.7)
    rng = np.random.default_rng(0)
    t = rng.integers(0, w.V, size=(w.B, w.K + 1)).astype(np.int32)
    d = wl.draft_tokens(w, 3, t)
    assert d.shape == (w.B, w.K) and d.dtype == np.int32
    assert np.array_equal(d, wl.draft_tokens(w, 3, t))
    match = d == t[:, :w.K]
    assert abs(match.mean() - 0.7) < 4 * math.sqrt(0.21 / match.size)
    assert d.min() >= 0 and d.max() < w.V
    # mismatching tokens are spread over the other V-1 tokens
    rel = (d - t[:, :w.K])[~match] % w.V
    counts = np.bincount(rel, minlength=w.V)
    assert counts[0] == 0 and counts[1:].min() > 0.6 * counts[1:].mean()
    # unknown greedy tokens (-1) give uniform tokens in range
    d2 = wl.draft_tokens(w, 3, np.full_like(t, -1))
    assert d2.min() >= 0 and d2.max() < w.V


def test_draft_tokens_clustered_runs():
    w = wl.scaled(wl.WORKLOADS["8b_b32_k32"], B=256, V=1000)
    t = np.random.default_rng(1).integers(0, w.V, size=(w.B, w.K + 1)).astype(np.int32)
    d = wl.draft_tokens(w, 20039, t)
    mis = d != t[:, :w.K]
    assert abs(mis.mean() - 0.25) < 0.03
    # drawn runs have mean length 2; a new run may start right after one ends (prob q = 1/7), and
    # such runs merge when observed: mean observed length 2/(1-q) = 2.33, a little less after
    # truncation at the window end
    runs = []
    for b in range(w.B):
        j = 0
        while j < w.K:
            if mis[b, j]:
                k = j
                while k < w.K and mis[b, k]:
                    k += 1
                runs.append(k - j)
                j = k
            else:
                j += 1
    assert 2.1 < np.mean(runs) < 2.5


@pytest.mark.parametrize("name", ["8b_b1_k16", "70b_b8_k32"])
def test_stored_oracle_rows_fit_the_regenerated_inputs(name):
    """The full-size GPU parity tests trust tests/golden/greedy_*.txt only if the inputs they regenerate are the
    bytes those rows were computed from.  The same digests, checked here without a GPU, for a 4096- and an
    8192-wide workload (the other two stored files share these W_lm tensors)."""
    import hashlib
    import sys
    import os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from parity import read_golden
    w = wl.WORKLOADS[name]
    sha, rows = read_golden(name, wl.DEFAULT_SEED)
    assert len(rows) == w.M
    tensors = {"hidden_t": wl.hidden_t, "W_lm": wl.w_lm, "hidden_d": wl.hidden_d, "clf_w": wl.clf_w}
    for key, make in tensors.items():
        got = hashlib.sha256(np.ascontiguousarray(make(w, wl.DEFAULT_SEED)).tobytes()).hexdigest()
        assert got == sha[key], f"{name}: regenerated {key} is not the tensor the stored oracle rows were made from"
