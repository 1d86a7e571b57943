"""GPU parity with W_lm stored as OCP FP8 E4M3 (the FP8 LM head of the paper's 405B run, Section 4) through the C
ABI.  The kernel widens the bytes exactly to bf16, so the oracle is fed the decoded weights as bf16 bits and the
bars are those of the bf16 path (products exact, fp32 accumulation order the only difference)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import compare, make_inputs, run_gpu

pytestmark = pytest.mark.gpu


def fp8_case(w, seed, tau=None, repeat=1, sampled=None):
    x = make_inputs(w, seed)
    w8, scale = wl.w_lm_fp8(w, seed)
    x.W = wl.fp8_e4m3_to_bf16_bits(w8)              # what the kernel computes with, exactly
    greedy = oracle.greedy_rows(x.ht, x.W) if sampled is None else \
        oracle.sampled_rows(x.ht, x.W, sampled[0], sampled[1].reshape(-1))
    draft = wl.draft_tokens(w, seed, greedy[0])
    tau = w.tau if tau is None else tau
    gpu = run_gpu(x, draft, tau, repeat=repeat, w8=w8, sampled=sampled)
    scores_row = None
    if sampled is not None:
        keys = sampled[1].reshape(-1)

        def scores_row(r):
            return oracle.logits_row(x.ht[r], x.W) * sampled[0] + np.array([oracle.gumbel(int(keys[r]), v) for v in range(w.V)])
    rep = compare(x, draft, tau, greedy, gpu, scores_row=scores_row)
    assert gpu["kernel"] == ("lm_head_stream16_fp8w" if w.M <= 32 and w.d_t == 4096 else
                             "lm_head_resident_fp8w" if w.M <= 112 or (w.M <= 128 and w.d_t % 512) else "lm_head_wide_fp8w")
    return rep, x, w8, gpu


@pytest.mark.parametrize("shape", [
    dict(B=1, K=16, V=5003),           # ragged vocabulary
    dict(B=2, K=15, V=9000),           # all 32 rows
    dict(B=1, K=4, V=40),              # fewer tiles than workgroups
    dict(B=3, K=7, V=70001),           # more tiles than workgroups: several per workgroup
    dict(B=1, K=32, V=5003, d_t=8192),     # 33 rows at the 70B hidden size: the accumulator-resident kernel
    dict(B=1, K=64, V=140000, d_t=1024),   # 65 rows; more vocabulary than one pass holds
    dict(B=4, K=31, V=3000, d_t=768),      # 128 rows: all eight row blocks of the accumulator-resident kernel
    dict(B=4, K=31, V=3000, d_t=512),      # 128 rows at a multiple of 512: the wide kernel's smallest tile
    dict(B=2, K=15, V=1000, d_t=2048),     # 32 rows at a hidden size the 16-row-tile kernel does not take in FP8
    dict(B=8, K=32, V=3000, d_t=1024),     # 264 rows: the wide kernel, 17 row blocks (the last one in VGPRs), ragged last tile
    dict(B=3, K=42, V=70001, d_t=512),     # 129 rows: 9 row blocks, one trip of the slab loop, more tiles than workgroups
    dict(B=4, K=59, V=1000, d_t=1536),     # 240 rows: 15 row blocks (the short fragment window)
    dict(B=4, K=51, V=2000, d_t=512),      # 208 rows: 13 row blocks
])
def test_fp8_weights(shape):
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="fp8", p_match=0.6, **shape)
    for tau in (0.0, 0.5, 1.0):
        rep, x, w8, gpu = fp8_case(w, 13, tau=tau, repeat=2)
        assert rep["maxlogit_relerr"] < 1e-4
    # all logits through the same kernel
    import torch
    import paper_2504_20039_amd as aj
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16, 1, 0, 0, aj.AJ_W_FP8_E4M3)
    logits = torch.empty((w.M, w.V), dtype=torch.float32, device="cuda")
    aj.aj_debug_logits(h, aj.device_tensor(x.ht), aj.device_tensor(w8), logits)
    torch.cuda.synchronize()
    aj.aj_destroy(h)
    ref = wl.widen(x.ht) @ wl.widen(x.W).T
    assert np.abs(logits.cpu().numpy() - ref).max() <= 1e-4 * np.abs(ref).max()


# the 16-row-tile kernel; the accumulator-resident one; the wide one
@pytest.mark.parametrize("B,K,d_t", [(2, 15, 4096), (4, 31, 256), (8, 32, 512), (3, 47, 1024)])
def test_every_fp8_code_is_widened_exactly(B, K, d_t):
    """One-hot hidden rows turn the logit dump into a read-out of the weights as the kernel sees them: every finite
    E4M3 code (subnormals, both zeros, +-448) must come out as the format defines it, bit for bit."""
    import torch
    import paper_2504_20039_amd as aj
    M, V = B * (K + 1), 512
    v, k = np.meshgrid(np.arange(V), np.arange(d_t), indexing="ij")
    w8 = ((v + 3 * k) % 256).astype(np.uint8)
    w8[(w8 & 0x7F) == 0x7F] = 0x38                    # the two NaN codes -> 1.0
    ht = np.zeros((M, d_t), np.uint16)
    ht[np.arange(M), (np.arange(M) * 7) % d_t] = 0x3F80      # bf16 1.0 at column 7r of row r
    h = aj.aj_create(B, K, d_t, 64, V, aj.AJ_BF16, 1, 0, 0, aj.AJ_W_FP8_E4M3)
    logits = torch.empty((M, V), dtype=torch.float32, device="cuda")
    aj.aj_debug_logits(h, aj.device_tensor(ht), aj.device_tensor(w8), logits)
    torch.cuda.synchronize()
    aj.aj_destroy(h)
    want = wl.widen(wl.fp8_e4m3_to_bf16_bits(w8))[:, (np.arange(M) * 7) % d_t].T      # [M][V]
    got = logits.cpu().numpy()
    assert set(np.unique(w8)) >= set(range(0, 0x7F)) | set(range(0x80, 0xFF))
    assert np.array_equal(got.view(np.uint32) & 0x7FFFFFFF, want.astype(np.float32).view(np.uint32) & 0x7FFFFFFF)
    assert np.array_equal(got, want)


def test_fp8_sampling_and_full_size():
    w = wl.WORKLOADS["8b_b1_k16"]
    rep, x, w8, gpu = fp8_case(w, wl.DEFAULT_SEED, repeat=2)
    print(rep)
    keys = np.random.default_rng(2).integers(0, 2**63, size=(w.B, w.K + 1), dtype=np.uint64)
    # the weights are scaled by 1/scale: fold the scale into the temperature so that T = 1 in the original units
    _, scale = wl.w_lm_fp8(w, wl.DEFAULT_SEED)
    fp8_case(w, wl.DEFAULT_SEED, sampled=(scale, keys))


def test_fp8_sampling_wide():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="fp8", p_match=0.6, B=8, K=32, V=3000, d_t=1024)
    keys = np.random.default_rng(5).integers(0, 2**63, size=(w.B, w.K + 1), dtype=np.uint64)
    _, scale = wl.w_lm_fp8(w, 13)
    fp8_case(w, 13, sampled=(scale, keys))


def test_fp8_refusals():
    import paper_2504_20039_amd as aj
    ok = dict(B=1, K=16, d_t=4096, d_d=64, V=1000)
    for bad in (dict(d_t=4096 + 64), dict(B=17), dict(B=8, d_t=768), dict(dtype=aj.AJ_F32), dict(flags=aj.AJ_FLAG_TOPK), dict(kernel=aj.AJ_KERNEL_PAIR),
                dict(w_dtype=7)):
        a = dict(ok, dtype=aj.AJ_BF16, flags=0, kernel=0, w_dtype=aj.AJ_W_FP8_E4M3)
        a.update(bad)
        with pytest.raises(aj.AjError) as e:
            aj.aj_create(a["B"], a["K"], a["d_t"], a["d_d"], a["V"], a["dtype"], 1, a["flags"], a["kernel"], a["w_dtype"])
        assert e.value.status == -1, bad
