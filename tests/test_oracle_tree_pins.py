"""Pins of the oracle's draft-tree verification (Section 3.3 "Generality": the judge on a tree-based verification
stage) against things other than itself (CPU only).

  hand example (tests/golden/hand_example_tree.txt)      -> edge rule, row indexing, depth tie rule, emission
  a chain (parent[j] = j - 1) is the linear walk          -> reduces to ajo_walk
  tau = 0: textbook greedy tree verification              -> independent routine following matching children
  tau = 1: every node accepted                            -> deepest node of the tree, lowest index
  brute force over all root-to-node paths                 -> accepted[] recursion and the choice of the path
  monotone in tau; bad parent arrays are refused
"""
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example_tree.txt")


def bf16(x):
    x = np.asarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0)
    return (u >> 16).astype(np.uint16)


def load_example():
    ex = {"case": [], "case2": []}
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] in ("case", "case2"):
            ex[t[0]].append((float(t[1]), int(t[2]), int(t[3]), int(t[4])))
        else:
            ex[t[0]] = [float(x) for x in t[1:]]
    return ex


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hand_example(dtype):
    ex = load_example()
    conv = (lambda a: np.asarray(a, np.float32)) if dtype == "f32" else bf16
    W = conv(np.array(ex["W_lm"]).reshape(4, 2))
    ht = conv(np.array(ex["hidden_t"]).reshape(6, 2))
    hd = conv(np.array(ex["hidden_d"]).reshape(6, 1))
    cw = conv(ex["clf_w"])
    for key, par, tok in (("case", "parent", "draft_tok"), ("case2", "parent2", "draft_tok2")):
        parent = np.array([ex[par]], np.int32)
        draft = np.array([ex[tok]], np.int32)
        for tau, out_len, out_node, out_tok in ex[key]:
            r = oracle.verify_tree(ht, hd, W, draft, parent, cw, ex["clf_b"][0], tau)
            assert list(r.t_star) == [int(x) for x in ex["t_star"]]
            assert (int(r.out_len[0]), int(r.out_node[0]), int(r.out_tok[0])) == (out_len, out_node, out_tok), (key, tau)


def random_tree(rng, K):
    return np.array([rng.integers(-1, j) for j in range(K)], np.int32)      # parent[j] in [-1, j)


def setup(seed, B=6, K=9):
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], name="t", B=B, K=K)
    ht, hd, W, cw = wl.hidden_t(w, seed), wl.hidden_d(w, seed), wl.w_lm(w, seed), wl.clf_w(w, seed)
    t = oracle.greedy_rows(ht, W)[0].reshape(B, K + 1)
    rng = np.random.default_rng(seed)
    parent = np.stack([random_tree(rng, K) for _ in range(B)])
    # tokens: the target's prediction at the parent's row with probability 0.6, else another token
    draft = np.empty((B, K), np.int32)
    for b in range(B):
        for j in range(K):
            want = t[b, parent[b, j] + 1]
            draft[b, j] = want if rng.random() < 0.6 else (want + 1 + rng.integers(w.V - 1)) % w.V
    return w, ht, hd, W, cw, t, parent, draft


def test_chain_is_the_linear_walk():
    w, ht, hd, W, cw, t, _, _ = setup(1)
    chain = np.tile(np.arange(-1, w.K - 1, dtype=np.int32), (w.B, 1))
    draft = wl.draft_tokens(w, 1, t.reshape(-1))
    for tau in (0.0, 0.3, 0.6, 1.0):
        a = oracle.walk_tree(ht, hd, t, draft, chain, cw, 0.0, tau)
        b = oracle.walk(ht, hd, t, draft, cw, 0.0, tau)
        assert np.array_equal(a.out_len, b.out_len) and np.array_equal(a.out_tok, b.out_tok)
        assert np.array_equal(a.out_node, b.out_len - 1)
        assert np.array_equal(a.mismatch, b.mismatch)
        np.testing.assert_array_equal(a.z, b.z)
    for fo in (0, 1):
        a = oracle.walk_tree(ht, hd, t, draft, chain, cw, 0.0, 0.4, feat_offset=fo)
        b = oracle.walk(ht, hd, t, draft, cw, 0.0, 0.4, feat_offset=fo)
        assert np.array_equal(a.out_len, b.out_len)


def greedy_tree(t_row, parent, tok):
    """Textbook greedy tree verification: from the root follow a child whose token is the target's
    prediction; with duplicate matching siblings every such branch is explored and the deepest kept."""
    K = len(parent)
    best = (0, -1)

    def go(node, depth):
        nonlocal best
        if depth > best[0] or (depth == best[0] and depth > 0 and node < best[1]):
            best = (depth, node)
        for c in range(K):
            if parent[c] == node and tok[c] == t_row[node + 1]:
                go(c, depth + 1)
    go(-1, 0)
    return best


def test_tau_zero_is_greedy_tree_verification_and_tau_one_accepts_all():
    for seed in range(5):
        w, ht, hd, W, cw, t, parent, draft = setup(seed)
        r0 = oracle.verify_tree(ht, hd, W, draft, parent, cw, 0.0, 0.0)
        r1 = oracle.verify_tree(ht, hd, W, draft, parent, cw, 0.0, 1.0)
        for b in range(w.B):
            depth, node = greedy_tree(t[b], parent[b], draft[b])
            assert (r0.out_len[b], r0.out_node[b]) == (depth, node)
            assert r0.out_tok[b] == t[b, node + 1]
            d = np.zeros(w.K, int)
            for j in range(w.K):
                d[j] = 1 + (d[parent[b, j]] if parent[b, j] >= 0 else 0)
            assert r1.out_len[b] == d.max() and r1.out_node[b] == int(np.argmax(d))


def test_brute_force_over_paths_and_monotone():
    for seed in range(4):
        w, ht, hd, W, cw, t, parent, draft = setup(seed + 10, B=4, K=8)
        prev = None
        for tau in (0.0, 0.2, 0.5, 0.8, 1.0):
            r = oracle.verify_tree(ht, hd, W, draft, parent, cw, 0.0, tau)
            zthr = oracle.threshold_logit(tau)
            for b in range(w.B):
                best = (0, -1)
                for j in range(w.K):
                    path, n = [], j
                    while n >= 0:
                        path.append(n)
                        n = parent[b, n]
                    ok = True
                    for n in path:            # every edge on the way must match or be judged unimportant
                        if draft[b, n] != t[b, parent[b, n] + 1]:
                            row = b * (w.K + 1) + n + 1
                            z = oracle.judge_logit(ht[row], hd[row], cw, 0.0)
                            ok &= z < zthr
                    if ok and len(path) > best[0]:
                        best = (len(path), j)
                assert (r.out_len[b], r.out_node[b]) == best, (seed, tau, b)
                assert r.out_tok[b] == t[b, best[1] + 1]
            if prev is not None:
                assert (r.out_len >= prev).all()
            prev = r.out_len


def test_bad_parents_are_refused():
    w, ht, hd, W, cw, t, parent, draft = setup(3)
    p = parent.copy(); p[0, 2] = 2
    with pytest.raises(ValueError):
        oracle.walk_tree(ht, hd, t, draft, p, cw, 0.0, 0.5)
    p = parent.copy(); p[1, 0] = 0
    with pytest.raises(ValueError):
        oracle.walk_tree(ht, hd, t, draft, p, cw, 0.0, 0.5)
    p = parent.copy(); p[2, 3] = -2
    with pytest.raises(ValueError):
        oracle.walk_tree(ht, hd, t, draft, p, cw, 0.0, 0.5)
