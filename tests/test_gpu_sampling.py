"""GPU parity of sampling-mode verification (Appendix A: Gumbel-max with a seeded generator) through the C ABI.

Bars as in the greedy path, on the perturbed scores logit / T + G: sampled tokens bit-exact except rows the
oracle flags as near-ties (top-2 gap of the perturbed scores < 1e-3 |max|), which are counted, checked to lie in
the band, and replayed; the perturbed maximum within 1e-2 relative (seen: ~1e-6: the GPU takes the two
logarithms of the noise in fp32, the oracle in fp64); accepted lengths and emitted tokens bit-exact.
"""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import compare, make_inputs, run_gpu

pytestmark = pytest.mark.gpu


def keys_for(w, seed):
    rng = np.random.default_rng(seed)
    k = rng.integers(0, 2**63, size=(w.B, w.K + 1), dtype=np.uint64)
    k[0, 0] |= np.uint64(1) << np.uint64(63)        # a key with the top bit set
    return k


def sampling_case(w, seed, inv_t, kernel=0, tau=None, repeat=1):
    x = make_inputs(w, seed)
    keys = keys_for(w, seed + 100)
    ref = oracle.sampled_rows(x.ht, x.W, inv_t, keys.reshape(-1))
    draft = wl.draft_tokens(w, seed, ref[0])
    tau = w.tau if tau is None else tau
    gpu = run_gpu(x, draft, tau, kernel=kernel, repeat=repeat, sampled=(inv_t, keys))

    def scores_row(r):
        lg = oracle.logits_row(x.ht[r], x.W) * inv_t
        return lg + np.array([oracle.gumbel(int(keys.reshape(-1)[r]), v) for v in range(w.V)])
    rep = compare(x, draft, tau, ref, gpu, scores_row=scores_row)
    return rep, x, keys, ref, gpu


def test_tiny_f32_and_the_noise_matters():
    w = wl.WORKLOADS["tiny_f32"]
    rep, x, keys, ref, gpu = sampling_case(w, 20039, 4.0, repeat=2)
    g = oracle.greedy_rows(x.ht, x.W)[0]
    assert (ref[0] != g).any()                       # some sampled tokens differ from the greedy ones
    # T -> 0 on the GPU gives the greedy tokens
    draft = wl.draft_tokens(w, 20039, g)
    hot = run_gpu(x, draft, w.tau, sampled=(1e9, keys))
    assert np.array_equal(hot["t_star"], g)
    # 1/T = 0: pure noise; the oracle agrees bit for bit (no logits involved beyond a zero product)
    cold = run_gpu(x, draft, w.tau, sampled=(0.0, keys))
    assert np.array_equal(cold["t_star"], oracle.sampled_rows(x.ht, x.W, 0.0, keys.reshape(-1))[0])


@pytest.mark.parametrize("kernel", [0, 1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("shape", [
    dict(B=1, K=16, d_t=4096, d_d=64, V=5003),         # 16-row streaming kernel, ragged vocabulary
    dict(B=2, K=15, d_t=384, d_d=64, V=20000),         # streaming regime at another hidden size
    dict(B=2, K=15, d_t=2048, d_d=64, V=3000),         # 16-row streaming kernel, one stage per tile
    dict(B=3, K=16, d_t=1024, d_d=64, V=2500),         # general 128x128 kernel
    dict(B=9, K=31, d_t=512, d_d=64, V=3001),          # M=288: 256-row kernels (2 row tiles) and the 8-wave one
    dict(B=1, K=64, d_t=1024, d_d=64, V=3001),         # M=65: accumulator-resident kernel, five row blocks
    dict(B=8, K=32, d_t=512, d_d=64, V=3001),          # M=264: the wide kernel's 17 row blocks
    dict(B=20, K=31, d_t=256, d_d=64, V=1100),         # M=640
    dict(B=4, K=24, d_t=512, d_d=64, V=3000),          # M=100: the 128-row streaming tile
])
def test_bf16_shapes_all_kernels(kernel, shape):
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="smp", p_match=0.6, **shape)
    try:
        aj.aj_destroy(aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, 1, 0, kernel))
    except aj.AjError as e:
        assert e.status == -1
        pytest.skip(f"kernel variant {kernel} does not take this shape")
    for inv_t in (1.0, 3.0):
        rep, x, keys, ref, gpu = sampling_case(w, 7, inv_t, kernel=kernel, repeat=2)
        assert rep["maxlogit_relerr"] < 1e-4
        assert rep["near_tie_rows"] <= 0.1 * w.M + 3


def test_same_key_same_noise_and_bad_calls():
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="smp", B=2, K=8, d_t=512, d_d=64, V=4000)
    x = make_inputs(w, 5)
    x.ht[w.K + 1:] = x.ht[:w.K + 1]                  # two identical windows ...
    keys = keys_for(w, 1)
    keys[1] = keys[0]                                # ... with identical keys sample identical tokens
    y = oracle.sampled_rows(x.ht, x.W, 2.0, keys.reshape(-1))[0].reshape(2, -1)
    assert np.array_equal(y[0], y[1])
    draft = wl.draft_tokens(w, 5, y.reshape(-1))
    gpu = run_gpu(x, draft, 0.5, sampled=(2.0, keys))
    t = gpu["t_star"].reshape(2, -1)
    assert np.array_equal(t[0], t[1]) and np.array_equal(t, y)
    keys2 = keys.copy()
    keys2[1] ^= np.uint64(1)                         # one bit of the key changes the noise
    t2 = run_gpu(x, draft, 0.5, sampled=(2.0, keys2))["t_star"].reshape(2, -1)
    assert np.array_equal(t2[0], t[0]) and not np.array_equal(t2[1], t[1])
    assert np.array_equal(t2.reshape(-1), oracle.sampled_rows(x.ht, x.W, 2.0, keys2.reshape(-1))[0])

    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code)
    dev = [aj.device_tensor(a) for a in (x.ht, x.hd, x.W, draft, x.cw)]
    d_key = torch.from_numpy(keys.view(np.int64)).cuda()
    o1, o2 = torch.zeros(2, dtype=torch.int32, device="cuda"), torch.zeros(2, dtype=torch.int32, device="cuda")
    for bad in (-1.0, float("nan"), float("inf")):
        with pytest.raises(aj.AjError) as e:
            aj.aj_verify_sampled(h, dev[0], dev[1], dev[2], dev[3], dev[4], 0.0, 0.5, bad, d_key, o1, o2)
        assert e.value.status == -1
    with pytest.raises(aj.AjError):
        aj.aj_verify_sampled(h, dev[0], dev[1], dev[2], dev[3], dev[4], 0.0, 0.5, 1.0, None, o1, o2)
    aj.aj_destroy(h)


def test_full_size_default_workload():
    """The bench default at full size: every sampled token of the 17 rows against the oracle."""
    w = wl.WORKLOADS["8b_b1_k16"]
    rep, x, keys, ref, gpu = sampling_case(w, wl.DEFAULT_SEED, 1.0, repeat=2)
    print(rep)
    assert gpu["kernel"] == "lm_head_stream16_bf16"


@pytest.mark.parametrize("name,windows", [("70b_b8_k32", (0, 7)), ("70b_b128_k64", (127,))])
def test_full_size_sampled_windows(name, windows):
    """The large workloads in the launch configuration bench.py times: sampled tokens, perturbed maxima and
    outcomes of a few windows against the oracle (windows are independent), properties on all windows."""
    w = wl.WORKLOADS[name]
    seed = wl.DEFAULT_SEED
    x = make_inputs(w, seed)
    keys = keys_for(w, 5)
    R = w.K + 1
    inv_t = 1.0
    t = np.full(w.M, -1, np.int32)
    m1, m2 = np.full(w.M, np.nan), np.full(w.M, np.nan)
    for b in windows:
        sl = slice(b * R, (b + 1) * R)
        t[sl], m1[sl], m2[sl] = oracle.sampled_rows(x.ht[sl], x.W, inv_t, keys[b])
    draft = wl.draft_tokens(w, seed, t)              # windows without oracle rows get uniform tokens
    gpu = run_gpu(x, draft, w.tau, sampled=(inv_t, keys))

    def scores_row(r):
        lg = oracle.logits_row(x.ht[r], x.W) * inv_t
        return lg + np.array([oracle.gumbel(int(keys.reshape(-1)[r]), v) for v in range(w.V)])
    rep = compare(x, draft, w.tau, (t, m1, m2), gpu, windows=windows, scores_row=scores_row)
    print(rep)
    assert ((gpu["out_len"] >= 0) & (gpu["out_len"] <= w.K)).all()
    assert np.array_equal(gpu["out_tok"], gpu["t_star"][np.arange(w.B) * R + gpu["out_len"]])
    assert ((gpu["t_star"] >= 0) & (gpu["t_star"] < w.V)).all()
