"""GPU parity of draft-tree verification (Section 3.3 "Generality") through the C ABI, against the oracle.

Bars as in the chain path: greedy tokens bit-exact except oracle-flagged near-ties (replayed), judge scores
within 1e-3, accepted node / depth / emitted token bit-exact (a window whose outcome hinges on a near-threshold
score is counted instead, as in tests/parity.py)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import make_inputs

pytestmark = pytest.mark.gpu


def random_trees(rng, B, K, shape):
    parent = np.empty((B, K), np.int32)
    for b in range(B):
        for j in range(K):
            if shape == "chain":
                parent[b, j] = j - 1
            elif shape == "star":
                parent[b, j] = -1
            elif shape == "bushy":               # EAGLE-like: a few branches per level
                parent[b, j] = -1 if j < 3 else rng.integers(max(-1, j - 7), j)
            else:
                parent[b, j] = rng.integers(-1, j)
    return parent


def tree_drafts(rng, t, parent, V, p_match):
    B, K = parent.shape
    draft = np.empty((B, K), np.int32)
    for b in range(B):
        for j in range(K):
            want = t[b, parent[b, j] + 1]
            draft[b, j] = want if rng.random() < p_match else (want + 1 + rng.integers(V - 1)) % V
    return draft


def run_tree(x, draft, parent, tau, feat_offset=1, kernel=0, clf_b=0.0):
    import torch
    import paper_2504_20039_amd as aj
    w = x.w
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, feat_offset, aj.AJ_FLAG_DEBUG, kernel)
    dev = [aj.device_tensor(a) for a in (x.ht, x.hd, x.W, np.ascontiguousarray(draft, np.int32),
                                         np.ascontiguousarray(parent, np.int32), x.cw)]
    outs = [torch.full((w.B,), -9, dtype=torch.int32, device="cuda") for _ in range(3)]
    aj.aj_verify_tree(h, dev[0], dev[1] if w.d_d > 0 else None, dev[2], dev[3], dev[4], dev[5], clf_b, tau,
                      outs[0], outs[1], outs[2])
    torch.cuda.synchronize()
    t_star, maxlogit, score = aj.aj_debug_copy(h, w.B, w.K)
    aj.aj_destroy(h)
    return dict(out_len=outs[0].cpu().numpy(), out_tok=outs[1].cpu().numpy(), out_node=outs[2].cpu().numpy(),
                t_star=t_star, maxlogit=maxlogit, score=score)


def check(x, draft, parent, tau, gpu, greedy, feat_offset=1, clf_b=0.0):
    w = x.w
    t, m1, m2 = greedy
    flag = oracle.near_tie(m1, m2)
    differ = gpu["t_star"] != t
    assert not (differ & ~flag).any()
    assert np.abs(gpu["maxlogit"] - m1).max() <= 1e-2 * np.abs(m1).min()
    # replay on the GPU's tokens (they differ from the oracle's only on flagged rows)
    ref = oracle.walk_tree(x.ht, x.hd, gpu["t_star"].reshape(w.B, w.K + 1), draft, parent, x.cw, clf_b, tau, feat_offset)
    mis = ref.mismatch.astype(bool)
    gz, gp = gpu["score"]
    assert np.isnan(gz[~mis]).all()
    if mis.any():
        assert np.abs(gz[mis] - ref.z[mis]).max() <= 1e-3 and np.abs(gp[mis] - ref.p[mis]).max() <= 1e-3
    bad = (gpu["out_len"] != ref.out_len) | (gpu["out_node"] != ref.out_node) | (gpu["out_tok"] != ref.out_tok)
    for b in np.nonzero(bad)[0]:
        assert ref.near_thr[b].any(), (b, gpu["out_len"][b], ref.out_len[b])
    assert bad.sum() <= 1 + w.B // 100
    # what holds for any outcome: the emitted token is the greedy token of the accepted node's row
    assert np.array_equal(gpu["out_tok"], gpu["t_star"].reshape(w.B, -1)[np.arange(w.B), gpu["out_node"] + 1])
    return int(differ.sum())


@pytest.mark.parametrize("shape", ["chain", "star", "bushy", "random"])
@pytest.mark.parametrize("dims", [
    dict(B=1, K=8, d_t=256, d_d=128, V=1024, dtype="f32"),
    dict(B=6, K=15, d_t=512, d_d=256, V=3000),
    dict(B=3, K=63, d_t=1024, d_d=0, V=2000),           # target-only features, as in the paper's EAGLE runs
])
def test_tree_shapes(shape, dims):
    base = "tiny_f32" if dims.get("dtype") == "f32" else "8b_b1_k16"
    w = wl.scaled(wl.WORKLOADS[base], name="tree", **dims)
    x = make_inputs(w, 21)
    greedy = oracle.greedy_rows(x.ht, x.W)
    rng = np.random.default_rng(4)
    parent = random_trees(rng, w.B, w.K, shape)
    draft = tree_drafts(rng, greedy[0].reshape(w.B, w.K + 1), parent, w.V, 0.6)
    prev = None
    for tau in (0.0, 0.3, 0.6, 1.0):
        for fo in (1, 0):
            gpu = run_tree(x, draft, parent, tau, feat_offset=fo)
            check(x, draft, parent, tau, gpu, greedy, feat_offset=fo)
            if fo == 1:
                if prev is not None:
                    assert (gpu["out_len"] >= prev).all()
                prev = gpu["out_len"]
    if shape == "chain":                                # the chain is the linear entry point, bit for bit
        from parity import run_gpu
        lin = run_gpu(x, draft, 0.3)
        tr = run_tree(x, draft, parent, 0.3)
        assert np.array_equal(lin["out_len"], tr["out_len"]) and np.array_equal(lin["out_tok"], tr["out_tok"])
        assert np.array_equal(tr["out_node"], tr["out_len"] - 1)


def test_full_size_eagle_like_window_and_bad_calls():
    """8B-shaped target, target-only features, window of 8 nodes (the paper's EAGLE-2 setting), batch 4."""
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="eagle", B=4, K=8, d_d=0)
    x = make_inputs(w, wl.DEFAULT_SEED)
    greedy = oracle.greedy_rows(x.ht, x.W)
    rng = np.random.default_rng(8)
    parent = random_trees(rng, w.B, w.K, "bushy")
    draft = tree_drafts(rng, greedy[0].reshape(w.B, w.K + 1), parent, w.V, 0.5)
    for tau in (0.0, 0.5):
        gpu = run_tree(x, draft, parent, tau)
        check(x, draft, parent, tau, gpu, greedy)
    # malformed parents are clamped, not followed out of the window; null pointers are refused
    weird = parent.copy()
    weird[0, 3], weird[1, 0] = 100, -5
    gpu = run_tree(x, draft, weird, 0.5)
    assert ((gpu["out_node"] >= -1) & (gpu["out_node"] < w.K)).all()
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code)
    o = [torch.zeros(w.B, dtype=torch.int32, device="cuda") for _ in range(3)]
    dev = [aj.device_tensor(a) for a in (x.ht, x.W, draft, parent, x.cw)]
    with pytest.raises(aj.AjError) as e:
        aj.aj_verify_tree(h, dev[0], None, dev[1], dev[2], None, dev[4], 0.0, 0.5, o[0], o[1], o[2])
    assert e.value.status == -1
    with pytest.raises(aj.AjError):
        aj.aj_verify_tree(h, dev[0], None, dev[1], dev[2], dev[3], dev[4], 0.0, 0.5, o[0], o[1], None)
    aj.aj_destroy(h)
