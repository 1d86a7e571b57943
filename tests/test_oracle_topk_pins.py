"""Pins of the oracle's top-K baseline (Section 4: accept a mismatching draft token that is within
the target's top-K tokens) against things other than itself (CPU only).

  hand example (tests/golden/hand_example_topk.txt) -> ranks, tie order, walk, emission
  numpy stable sort of the fp64 GEMM logits         -> ajo_rank_rows (rank = position in the order)
  top_k = 1  == greedy verification (tau = 0 walk)  -> the baseline reduces to Section 2's algorithm
  top_k = V  accepts everything; monotone in top_k  -> endpoints and direction
  prefix formulation without early exit             -> ajo_walk_topk
  duplicated rows, invalid tokens, rank brackets    -> tie rule, edge cases, rank_lo <= rank <= rank_hi
"""
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example_topk.txt")


def bf16(x):
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0)
    return (u >> 16).astype(np.uint16)


def load_example():
    ex = {"cases": [], "ties": []}
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "case":
            v = [int(x) for x in t[1:]]
            ex["cases"].append((v[0:3], v[3], v[4], v[5], v[6:9]))
        elif t[0] == "tie_row":
            ex["ties"].append((int(t[1]), int(t[3]), int(t[5])))
        else:
            ex[t[0]] = [float(x) for x in t[1:]]
    return ex


def sorted_rank(logits_row, tok):
    """Position of tok when the vocabulary is sorted by logit (descending), equal logits by index."""
    order = np.lexsort((np.arange(len(logits_row)), -logits_row))      # library sort; last key is primary
    return int(np.nonzero(order == tok)[0][0])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hand_example(dtype):
    ex = load_example()
    conv = (lambda a: np.asarray(a, np.float32)) if dtype == "f32" else bf16
    W = conv(np.array(ex["W_lm"]).reshape(4, 2))
    H = conv(np.array(ex["hidden_t"]).reshape(4, 2))
    for draft, top_k, out_len, out_tok, ranks in ex["cases"]:
        r = oracle.verify_topk(H, W, np.array([draft], np.int32), top_k)
        assert list(r.t_star) == [int(x) for x in ex["t_star"]]
        assert (int(r.out_len[0]), int(r.out_tok[0])) == (out_len, out_tok), (draft, top_k)
        assert list(r.rank[:3]) == ranks and r.rank[3] == 0
    for row, tok, rank in ex["ties"]:
        t = np.full(4, -1, np.int32)
        t[row] = tok
        assert oracle.rank_rows(H, W, t).rank[row] == rank


def random_case(seed, B=3, K=6, d=24, V=97, dtype=np.float32):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((B * (K + 1), d)).astype(dtype)
    W = (0.1 * rng.standard_normal((V, d))).astype(dtype)
    draft = rng.integers(0, V, size=(B, K)).astype(np.int32)
    return H, W, draft


def test_rank_is_position_in_library_sort():
    H, W, draft = random_case(1)
    B, K = draft.shape
    W[11] = W[5]                     # exact duplicates: equal logits in every row
    W[90] = W[5]
    tok = np.full((B, K + 1), -1, np.int32)
    tok[:, :K] = draft
    tok[0, 0], tok[0, 1], tok[0, 2] = 5, 11, 90
    L = wl.widen(H) @ wl.widen(W).T
    r = oracle.rank_rows(H, W, tok)
    np.testing.assert_allclose(r.tok_logit.reshape(B, K + 1)[:, :K],
                               np.take_along_axis(L.reshape(B, K + 1, -1)[:, :K], draft_fix(tok, K), 2)[..., 0], rtol=1e-12)
    for row in range(B * (K + 1)):
        t = tok.reshape(-1)[row]
        assert r.t_star[row] == np.lexsort((np.arange(W.shape[0]), -L[row]))[0]
        if t < 0:
            assert r.rank[row] == 0
        else:
            assert r.rank[row] == sorted_rank(L[row], t), row
            assert r.rank_lo[row] <= r.rank[row] <= r.rank_hi[row]
    # the three copies of one row are ordered by index
    rk = r.rank.reshape(B, K + 1)
    assert rk[0, 1] == sorted_rank(L[1], 11) and sorted_rank(L[1], 11) == sorted_rank(L[1], 5) + 1


def draft_fix(tok, K):
    return tok[:, :K, None].astype(np.int64)


def test_top1_is_greedy_verification_and_topV_accepts_all():
    for seed in range(4):
        H, W, draft = random_case(seed, B=5, K=7)
        B, K = draft.shape
        V, d = W.shape
        g = oracle.greedy_rows(H, W)[0].reshape(B, K + 1)
        draft[:, :3] = g[:, :3]                  # a matching prefix, then mostly mismatches
        draft[1] = g[1, :K]                      # an all-match window
        # greedy verification = judge walk with tau = 0 (no override), any classifier
        cw = np.zeros(d + 8, np.float32)
        ref = oracle.verify(H, np.zeros((B * (K + 1), 8), np.float32), W, draft, cw, 0.0, 0.0)
        r1 = oracle.verify_topk(H, W, draft, 1)
        assert np.array_equal(r1.out_len, ref.out_len) and np.array_equal(r1.out_tok, ref.out_tok)
        assert r1.out_len[1] == K and r1.out_tok[1] == g[1, K]
        rV = oracle.verify_topk(H, W, draft, V)
        assert (rV.out_len == K).all() and np.array_equal(rV.out_tok, g[:, K])
        prev = r1.out_len
        for k in (2, 4, 8, 16, 32, 64, V):
            cur = oracle.verify_topk(H, W, draft, k).out_len
            assert (cur >= prev).all()
            prev = cur


def test_walk_matches_prefix_formulation():
    rng = np.random.default_rng(3)
    B, K = 50, 9
    rank = rng.integers(0, 6, size=(B, K + 1)).astype(np.int32)
    t_star = rng.integers(0, 1000, size=(B, K + 1)).astype(np.int32)
    for top_k in (1, 2, 3, 6, 7):
        out_len, out_tok = oracle.walk_topk(rank, t_star, top_k)
        ok = rank[:, :K] < top_k
        want = np.array([max(n for n in range(K + 1) if ok[b, :n].all()) for b in range(B)])
        assert np.array_equal(out_len, want)
        assert np.array_equal(out_tok, t_star[np.arange(B), want])


def test_invalid_tokens_and_bad_arguments():
    H, W, draft = random_case(7, B=2, K=4)
    V = W.shape[0]
    draft[0, 1] = V + 5            # outside the vocabulary: in no top-k
    draft[1, 0] = -3
    r = oracle.verify_topk(H, W, draft, V)
    assert r.out_len[0] == 1 and r.out_len[1] == 0
    assert r.rank.reshape(2, 5)[0, 1] == V and r.rank.reshape(2, 5)[1, 0] == V
    with pytest.raises(ValueError):
        oracle.verify_topk(H, W, draft, 0)


def test_rank_brackets_open_only_near_ties():
    # a row whose logits are far apart has lo == rank == hi; a planted near-tie opens the bracket
    H = np.zeros((1, 4), np.float32)
    H[0] = [1, 0, 0, 0]
    W = np.zeros((5, 4), np.float32)
    W[:, 0] = [4.0, 3.0, 2.0, 2.0 + 1e-5, -1.0]       # band = 1e-4 * 4
    for tok, rank, lo, hi in ((2, 3, 2, 3), (3, 2, 2, 3), (1, 1, 1, 1), (4, 4, 4, 4)):
        r = oracle.rank_rows(H, W, np.array([tok], np.int32))
        assert (r.rank[0], r.rank_lo[0], r.rank_hi[0]) == (rank, lo, hi), tok
