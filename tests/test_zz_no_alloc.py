"""aj_verify_static (the entry point that allocates nothing) against aj_create + aj_verify: same kernels, so the
outputs must be bit-identical; two calls in a row share the static device workspace, the second one smaller."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _inputs(w, seed):
    import oracle
    import workloads as wl
    ht, hd, W, cw = wl.hidden_t(w, seed), wl.hidden_d(w, seed), wl.w_lm(w, seed), wl.clf_w(w, seed)
    t, _, _ = oracle.greedy_rows(ht, W)
    return ht, hd, W, wl.draft_tokens(w, seed, t), cw


def _both(w, seed):
    """(out_len, out_tok) of the handle path and of the static path on the same device tensors."""
    import torch
    import paper_2504_20039_amd as aj
    ht, hd, W, draft, cw = _inputs(w, seed)
    dev = [aj.device_tensor(a) for a in (ht, hd, W, draft, cw)]
    res = []
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code)
    for static in (False, True):
        out_len = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
        out_tok = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
        if static:
            aj.aj_verify_static(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, 1, aj.AJ_KERNEL_AUTO, *dev, w.clf_b, w.tau,
                                out_len, out_tok)
        else:
            aj.aj_verify(h, *dev, w.clf_b, w.tau, out_len, out_tok)
        torch.cuda.synchronize()
        res.append((out_len.cpu().numpy(), out_tok.cpu().numpy()))
    aj.aj_destroy(h)
    return res, (ht, hd, W, draft, cw)


def test_static_entry_point_matches_the_handle_path_on_two_calls_in_a_row():
    import oracle
    import workloads as wl
    base = wl.WORKLOADS["tiny_f32"]
    # first a 264-row call on the 288-row large-tile kernel, then a smaller one (34 rows, streaming tiles) that
    # reuses the front of the same static workspace
    first = wl.scaled(base, dtype="bf16", B=8, K=32, d_t=1024, d_d=256, V=5000)
    second = wl.scaled(base, dtype="bf16", B=2, K=16, d_t=1024, d_d=256, V=3001)
    for w, seed in ((first, 11), (second, 12)):
        (ref, got), (ht, hd, W, draft, cw) = _both(w, seed)
        assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1]), (w, ref, got)
        assert (got[0] >= 0).all() and (got[0] <= w.K).all()
        # and the oracle's outcome, off oracle-flagged near-ties
        t, m1, m2 = oracle.greedy_rows(ht, W)
        if not oracle.near_tie(m1, m2).any():
            o = oracle.walk(ht, hd, t, draft, cw, w.clf_b, w.tau)
            assert np.array_equal(got[0], o.out_len) and np.array_equal(got[1], o.out_tok)


def test_static_entry_point_refuses_what_it_cannot_hold():
    import torch
    import paper_2504_20039_amd as aj
    x = torch.zeros(64, dtype=torch.int32, device="cuda")
    args = (x, x, x, x, x, 0.0, 0.5, x, x)
    # 128 windows x 65 rows of a 128256-entry vocabulary: 33 MB of per-block maxima, beyond the static 8 MiB
    with pytest.raises(aj.AjError) as e:
        aj.aj_verify_static(128, 64, 8192, 4096, 128256, aj.AJ_BF16, 1, aj.AJ_KERNEL_AUTO, *args)
    assert e.value.status == -5 and "static" in str(e.value)
    # flags need a handle
    with pytest.raises(aj.AjError) as e:
        aj.aj_verify_static(1, 8, 256, 128, 1024, aj.AJ_BF16, 1, aj.AJ_KERNEL_AUTO, *args, flags=aj.AJ_FLAG_DEBUG)
    assert e.value.status == -1
