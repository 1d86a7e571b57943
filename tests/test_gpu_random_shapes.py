"""Seeded random shapes through every entry point (automatic dispatch) against the oracle: row counts around the
dispatch boundaries, hidden sizes that select every LM-head kernel, vocabularies with ragged tiles."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import compare, make_inputs, run_gpu
import test_gpu_topk as tk
import test_gpu_tree as tr

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("stream", [11, 12, 13, 14])
def test_random_shapes(stream):
    rng = np.random.default_rng(stream)
    for it in range(12):
        d_t = int(rng.choice([64, 128, 192, 256, 320, 512, 768, 1024, 1280, 2048, 4096]))
        m = int(rng.choice([1, 5, 17, 31, 32, 33, 50, 64, 65, 100, 128, 129, 200, 256, 257, 288, 289, 320, 321, 400, 600]))
        K = int(rng.integers(1, min(64, m) + 1))
        B = max(1, m // (K + 1))
        V = int(rng.choice([17, 100, 255, 256, 257, 1000, 2049, 5000]))
        d_d = int(rng.choice([0, 8, 64, 256]))
        w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="rnd", B=B, K=K, d_t=d_t, d_d=d_d, V=V,
                      p_match=float(rng.choice([0.3, 0.6, 0.9])))
        seed, tau = int(rng.integers(1, 1000)), float(rng.choice([0.0, 0.2, 0.5, 0.8, 1.0]))
        case = f"B={B} K={K} d_t={d_t} d_d={d_d} V={V} seed={seed} tau={tau}"
        x = make_inputs(w, seed)
        greedy = oracle.greedy_rows(x.ht, x.W)
        # the judge path
        draft = wl.draft_tokens(w, seed, greedy[0])
        compare(x, draft, tau, greedy, run_gpu(x, draft, tau, repeat=2))
        # the top-K baseline
        dk = tk.planted_drafts(x, seed)
        for k, o in tk.run_topk(x, dk, [1, 3, V])[0].items():
            tk.check(x, dk, o, k)
        # sampling mode
        keys = rng.integers(0, 2**63, size=(B, K + 1), dtype=np.uint64)
        inv_t = float(rng.choice([0.5, 1.0, 3.0]))
        ref = oracle.sampled_rows(x.ht, x.W, inv_t, keys.reshape(-1))
        ds = wl.draft_tokens(w, seed, ref[0])

        def scores_row(r):
            return oracle.logits_row(x.ht[r], x.W) * inv_t + np.array([oracle.gumbel(int(keys.reshape(-1)[r]), v) for v in range(V)])
        compare(x, ds, tau, ref, run_gpu(x, ds, tau, sampled=(inv_t, keys)), scores_row=scores_row)
        # draft trees
        parent = tr.random_trees(rng, B, K, str(rng.choice(["chain", "star", "bushy", "random"])))
        dt = tr.tree_drafts(rng, greedy[0].reshape(B, K + 1), parent, V, 0.6)
        tr.check(x, dt, parent, tau, tr.run_tree(x, dt, parent, tau), greedy)
        print("ok", case, flush=True)
