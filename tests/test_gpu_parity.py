"""GPU parity: libaj (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import compare, make_inputs, oracle_greedy, parity_case, run_gpu

pytestmark = pytest.mark.gpu

TINY = wl.WORKLOADS["tiny_f32"]
KERNELS_BF16 = [1, 2, 3, 4, 5, 6, 7, 8] # AJ_KERNEL_TILE, _STREAM, _BIG, _TALL, _PAIR, _PAIR9, _RESIDENT, _WIDE (forced); 0 = AUTO is covered too


def _skip_unless_supported(w, kernel):
    """A forced LM-head variant refuses shapes it cannot run (AJ_EINVAL at aj_create)."""
    import paper_2504_20039_amd as aj
    try:
        aj.aj_destroy(aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, 1, 0, kernel))
    except aj.AjError as e:
        assert e.status == -1
        pytest.skip(f"kernel variant {kernel} does not take this shape")


def test_tiny_f32_workload_with_all_logits():
    import torch
    import paper_2504_20039_amd as aj
    for seed in (20039, 1, 2):
        rep, x, draft, greedy, gpu = parity_case(TINY, seed, repeat=2)
        assert rep["near_thr_windows"] == 0
    # the unfused view of step 1: every logit within 1e-2 of the row's scale
    h = aj.aj_create(TINY.B, TINY.K, TINY.d_t, TINY.d_d, TINY.V, aj.AJ_F32)
    logits = torch.empty((TINY.M, TINY.V), dtype=torch.float32, device="cuda")
    aj.aj_debug_logits(h, aj.device_tensor(x.ht), aj.device_tensor(x.W), logits)
    torch.cuda.synchronize()
    aj.aj_destroy(h)
    for r in range(TINY.M):
        ref = oracle.logits_row(x.ht[r], x.W)
        assert np.abs(logits[r].cpu().numpy() - ref).max() <= 1e-2 * np.abs(ref).max()
        assert np.abs(logits[r].cpu().numpy() - ref).max() <= 1e-5


@pytest.mark.parametrize("kernel", [0] + KERNELS_BF16)
@pytest.mark.parametrize("shape", [
    dict(B=1, K=8, d_t=256, d_d=128, V=1024),          # the tiny workload in bf16
    dict(B=5, K=33, d_t=520, d_d=136, V=1000),         # ragged everywhere: M=170, V%128, d%32
    dict(B=3, K=16, d_t=1024, d_d=512, V=2500),
    dict(B=2, K=1, d_t=64, d_d=8, V=130),
    dict(B=9, K=31, d_t=2048, d_d=256, V=777),         # M=288 spans several row tiles
    dict(B=1, K=16, d_t=1024, d_d=256, V=5000),        # one skinny row block, several vocabulary tiles per CU
    dict(B=2, K=15, d_t=384, d_d=128, V=70000),        # M=32 exactly; more tiles than workgroups
    dict(B=20, K=31, d_t=512, d_d=64, V=3000),         # M=640: 3 row tiles x 12 column tiles of the large kernel
    dict(B=10, K=31, d_t=256, d_d=64, V=1100),         # M=320: one 320-row tile of the 8-wave kernel
    dict(B=19, K=31, d_t=128, d_d=64, V=600),          # M=608: two 320-row tiles vs three 256-row tiles
    dict(B=1, K=16, d_t=4096, d_d=256, V=5003),        # the register-resident streaming kernel, ragged vocabulary
    dict(B=2, K=15, d_t=2048, d_d=128, V=9000),        # ... at d_t = 2048, all 32 rows
    dict(B=1, K=4, d_t=4096, d_d=64, V=40),            # ... fewer tiles than workgroups
    dict(B=9, K=31, d_t=512, d_d=64, V=60000),         # 2 x 235 large tiles: workgroups with two tiles and with one
    dict(B=4, K=24, d_t=512, d_d=64, V=3000),          # M=100: the 128-row streaming tile
    dict(B=2, K=31, d_t=8192, d_d=64, V=1500),         # M=64 exactly at the 70B hidden size
    dict(B=1, K=32, d_t=8192, d_d=64, V=9000),         # M=33: three row blocks of the accumulator-resident kernel
    dict(B=1, K=64, d_t=2048, d_d=64, V=140000),       # M=65; more vocabulary than one pass of 256 workgroups holds
    dict(B=4, K=31, d_t=768, d_d=64, V=3001),          # M=128: all eight row blocks, three k slabs
    dict(B=7, K=15, d_t=256, d_d=64, V=530),           # M=112, a single k slab, a ragged last vocabulary block
    dict(B=8, K=32, d_t=1024, d_d=64, V=3000),         # M=264: 17 row blocks of the wide kernel (one in VGPRs)
    dict(B=3, K=42, d_t=256, d_d=64, V=70000),         # M=129: 9 row blocks, one trip of four slabs, 274 tiles on 256 workgroups
    dict(B=8, K=31, d_t=512, d_d=64, V=1000),          # M=256: 16 row blocks
    dict(B=4, K=32, d_t=256, d_d=64, V=257),           # M=132, a second vocabulary tile of ONE row: every wave of it starts early
    dict(B=4, K=29, d_t=512, d_d=64, V=256),           # M=120: the wide kernel's 8 row blocks, exactly one vocabulary tile
    dict(B=6, K=31, d_t=256, d_d=64, V=319),           # M=192, 63 rows in the last tile: one wave with a range of its own
])
def test_bf16_shapes_all_kernels(kernel, shape):
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="shape", p_match=0.6, **shape)
    _skip_unless_supported(w, kernel)
    rep, x, draft, greedy, gpu = parity_case(w, 3, kernel=kernel, repeat=2)
    # all logits through the same kernel
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16, 1, 0, kernel)
    logits = torch.empty((w.M, w.V), dtype=torch.float32, device="cuda")
    aj.aj_debug_logits(h, aj.device_tensor(x.ht), aj.device_tensor(x.W), logits)
    torch.cuda.synchronize()
    aj.aj_destroy(h)
    ref = wl.widen(x.ht) @ wl.widen(x.W).T
    assert np.abs(logits.cpu().numpy() - ref).max() <= 1e-2 * np.abs(ref).max(axis=1).min()


@pytest.mark.parametrize("tau", [0.0, 0.3, 0.5, 1.0])
@pytest.mark.parametrize("feat_offset", [1, 0])
def test_tau_sweep_clustered(tau, feat_offset):
    w = wl.scaled(wl.WORKLOADS["8b_b32_k32"], name="sweep", B=24, d_t=512, d_d=256, V=4096)
    rep, x, draft, greedy, gpu = parity_case(w, 5, tau=tau, feat_offset=feat_offset)
    t = greedy[0].reshape(w.B, w.K + 1)
    if tau == 1.0:
        assert (gpu["out_len"] == w.K).all() and np.array_equal(gpu["out_tok"], gpu["t_star"].reshape(w.B, -1)[:, w.K])
    if tau == 0.0 and rep["near_tie_differ"] == 0:
        lcp = np.array([next((j for j in range(w.K) if draft[b, j] != t[b, j]), w.K) for b in range(w.B)])
        assert np.array_equal(gpu["out_len"], lcp)


def test_monotone_in_tau_on_gpu():
    w = wl.scaled(wl.WORKLOADS["70b_b8_k32"], name="mono", B=16, d_t=256, d_d=128, V=2048, p_match=0.5, clf_b=0.0)
    x = make_inputs(w, 8)
    greedy = oracle_greedy(x)
    draft = wl.draft_tokens(w, 8, greedy[0])
    prev = None
    for tau in (0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 1.0):
        gpu = run_gpu(x, draft, tau)
        compare(x, draft, tau, greedy, gpu)
        if prev is not None:
            assert (gpu["out_len"] >= prev).all()
        prev = gpu["out_len"]


def _edge_inputs(seed=4, B=4, **kw):
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="edge", B=B, K=12, d_t=256, d_d=64, V=1500, **kw)
    x = make_inputs(w, seed)
    return w, x, oracle_greedy(x)


def test_edge_draft_patterns():
    w, x, greedy = _edge_inputs()
    t = greedy[0].reshape(w.B, w.K + 1)
    allmatch = t[:, :w.K].copy()
    cases = {"all_match": allmatch}
    d = allmatch.copy(); d[:, 0] = (d[:, 0] + 1) % w.V; cases["slot0"] = d
    d = allmatch.copy(); d[:, w.K - 1] = (d[:, w.K - 1] + 1) % w.V; cases["last_slot"] = d
    cases["all_mismatch"] = (allmatch + 1) % w.V
    cases["out_of_vocab"] = np.full_like(allmatch, w.V + 3)
    cases["negative"] = np.full_like(allmatch, -1)
    for name, draft in cases.items():
        for tau in (0.0, 0.5, 1.0):
            gpu = run_gpu(x, draft, tau)
            compare(x, draft, tau, greedy, gpu)
            if name == "all_match":
                assert (gpu["out_len"] == w.K).all() and np.array_equal(gpu["out_tok"], t[:, w.K])
            if name in ("slot0", "all_mismatch", "out_of_vocab", "negative") and tau == 0.0:
                assert (gpu["out_len"] == 0).all() and np.array_equal(gpu["out_tok"], t[:, 0])


@pytest.mark.parametrize("kernel", [0] + KERNELS_BF16)
def test_argmax_at_vocabulary_ends_and_exact_ties(kernel):
    w, x, greedy = _edge_inputs(seed=6, B=2)        # 26 verify rows: every variant takes it
    _skip_unless_supported(w, kernel)
    R = w.K + 1
    # make row 0's hidden state a big multiple of a chosen W_lm row's sign pattern: that row wins
    Wd = wl.widen(x.W)
    def plant(row, v):
        h = np.sign(Wd[v]) + (Wd[v] == 0)
        x.ht[row] = ((h.astype(np.float32)).view(np.uint32) >> 16).astype(np.uint16)
    plant(0, 0)
    plant(1, w.V - 1)
    plant(2, 700)
    # exact duplicates of the winners, at higher and lower indices
    x.W[w.V - 2] = x.W[0]          # row 0: tie between 0 and V-2 -> 0
    x.W[5] = x.W[w.V - 1]          # row 1: tie between 5 and V-1 -> 5
    x.W[900] = x.W[700]            # row 2: tie between 700 and 900 (different vocabulary blocks) -> 700
    x.W[701] = x.W[700]            # and inside the same block -> 700
    greedy = oracle_greedy(x)
    assert list(greedy[0][:3]) == [0, 5, 700]
    draft = wl.draft_tokens(w, 6, greedy[0])
    gpu = run_gpu(x, draft, 0.5, kernel=kernel, repeat=2)
    # exact ties are flagged near-ties for the oracle, but the lowest-index rule is ours to keep:
    assert list(gpu["t_star"][:3]) == [0, 5, 700]
    compare(x, draft, 0.5, greedy, gpu)


def test_single_token_vocabulary_and_k1():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="v1", B=3, K=1, d_t=64, d_d=16, V=1)
    rep, x, draft, greedy, gpu = parity_case(w, 2)
    assert (gpu["t_star"] == 0).all() and (gpu["out_len"] == 1).all()


def test_target_only_judge():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="tonly", B=6, K=10, d_t=512, d_d=0, V=900, p_match=0.4)
    for tau in (0.3, 0.6):
        parity_case(w, 9, tau=tau)


@pytest.mark.parametrize("shape", [
    dict(B=1, K=32, d_t=1024, d_d=256, V=5000),        # 33 rows; the judge row is the first of a wave's block
    dict(B=4, K=31, d_t=512, d_d=64, V=3001),          # 128 rows; ragged vocabulary: the judge block follows a partial one
    dict(B=3, K=15, d_t=256, d_d=0, V=530),            # target-only features: the judge is the fused row alone
    dict(B=1, K=64, d_t=768, d_d=128, V=140000),       # several passes over the vocabulary; the judge block in the last
    dict(B=2, K=7, d_t=2048, d_d=64, V=16352),         # the vocabulary fills 511 of 512 blocks of one pass
])
def test_fused_judge_row(shape):
    """AJ_FLAG_FUSED_JUDGE: the judge's target half comes out of the LM-head pass as one more operand row; scores within
    1e-3 of the oracle on every mismatching slot, outcomes bit-exact, for both feature rows and a tau sweep."""
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="fused", p_match=0.4, **shape)
    x = make_inputs(w, 21)
    greedy = oracle_greedy(x)
    draft = wl.draft_tokens(w, 21, greedy[0])
    for feat_offset in (1, 0):
        for tau in (0.0, 0.4, 0.7, 1.0):
            gpu = run_gpu(x, draft, tau, feat_offset, flags=aj.AJ_FLAG_DEBUG | aj.AJ_FLAG_FUSED_JUDGE, repeat=2)
            assert gpu["kernel"] == "lm_head_resident_bf16"
            rep = compare(x, draft, tau, greedy, gpu, feat_offset)
            plain = run_gpu(x, draft, tau, feat_offset)
            assert np.array_equal(plain["out_len"], gpu["out_len"]) or rep["near_thr_windows"] > 0
    # shapes the fused row is not built for are refused at create
    for bad in (dict(B=8, K=32), dict(d_t=w.d_t + 64)):
        a = dict(B=w.B, K=w.K, d_t=w.d_t)
        a.update(bad)
        with pytest.raises(aj.AjError) as e:
            aj.aj_create(a["B"], a["K"], a["d_t"], w.d_d, w.V, aj.AJ_BF16, 1, aj.AJ_FLAG_FUSED_JUDGE)
        assert e.value.status == -1


def test_long_window():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="long", B=2, K=200, d_t=128, d_d=64, V=300, p_match=0.9,
                  clf_b=-2.0)
    rep, x, draft, greedy, gpu = parity_case(w, 10, tau=0.5)
    assert gpu["out_len"].max() > 64            # the scan went past one ballot


def test_empty_batch_and_bad_calls():
    import torch
    import paper_2504_20039_amd as aj
    h = aj.aj_create(0, 8, 256, 128, 1024, aj.AJ_BF16)
    aj.aj_verify(h, None, None, None, None, None, 0.0, 0.5, None, None)   # B = 0: nothing to do
    aj.aj_destroy(h)
    h = aj.aj_create(1, 8, 256, 128, 1024, aj.AJ_BF16)
    z = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    i = torch.zeros(64, dtype=torch.int32, device="cuda")
    W = torch.zeros((1024, 256), dtype=torch.bfloat16, device="cuda")
    for tau in (-0.5, 1.5, float("nan")):
        with pytest.raises(aj.AjError):
            aj.aj_verify(h, z, z, W, i, z, 0.0, tau, i, i)
    with pytest.raises(aj.AjError):
        aj.aj_verify(h, None, z, W, i, z, 0.0, 0.5, i, i)
    with pytest.raises(aj.AjError):
        aj.aj_verify(h, z[1:], z, W, i, z, 0.0, 0.5, i, i)              # misaligned
    with pytest.raises(aj.AjError):
        aj.aj_debug_copy(h, 1, 8, want_score=True)                      # AJ_FLAG_DEBUG not set
    aj.aj_destroy(h)


def test_non_default_stream():
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(TINY, dtype="bf16", B=4)
    x = make_inputs(w, 12)
    greedy = oracle_greedy(x)
    draft = wl.draft_tokens(w, 12, greedy[0])
    ref = oracle.walk(x.ht, x.hd, greedy[0], draft, x.cw, w.clf_b, w.tau)
    dev = [aj.device_tensor(a) for a in (x.ht, x.hd, x.W, draft, x.cw)]
    out_len = torch.zeros(w.B, dtype=torch.int32, device="cuda")
    out_tok = torch.zeros(w.B, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        aj.aj_verify(h, *dev, w.clf_b, w.tau, out_len, out_tok)
    s.synchronize()
    aj.aj_destroy(h)
    assert np.array_equal(out_len.cpu().numpy(), ref.out_len) and np.array_equal(out_tok.cpu().numpy(), ref.out_tok)


def test_maximum_window_length():
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="kmax", B=1, K=1023, d_t=64, d_d=8, V=200, p_match=0.97,
                  clf_b=-3.0)
    rep, x, draft, greedy, gpu = parity_case(w, 21, tau=0.5)
    assert 0 <= gpu["out_len"][0] <= 1023


def test_handle_reuse_with_other_inputs_and_two_handles():
    """A handle keeps no state between calls: results depend on the current arguments only."""
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="reuse", B=3, K=9, d_t=256, d_d=64, V=3000, p_match=0.5)
    xs = [make_inputs(w, s) for s in (31, 32)]
    refs, drafts = [], []
    for x in xs:
        g = oracle_greedy(x)
        d = wl.draft_tokens(w, x.seed, g[0])
        refs.append(oracle.walk(x.ht, x.hd, g[0], d, x.cw, w.clf_b, w.tau))
        drafts.append(d)
        assert not oracle.near_tie(g[1], g[2]).any()
    dev = [[aj.device_tensor(a) for a in (x.ht, x.hd, x.W, d, x.cw)] for x, d in zip(xs, drafts)]
    h1 = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16)
    h2 = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16)
    outs = [[torch.zeros(w.B, dtype=torch.int32, device="cuda") for _ in range(2)] for _ in range(4)]
    # h1: inputs 0, then inputs 1, then inputs 0 again; h2: inputs 1 in between - all enqueued back to back
    aj.aj_verify(h1, *dev[0], w.clf_b, w.tau, *outs[0])
    aj.aj_verify(h2, *dev[1], w.clf_b, w.tau, *outs[1])
    aj.aj_verify(h1, *dev[1], w.clf_b, w.tau, *outs[2])
    aj.aj_verify(h1, *dev[0], w.clf_b, w.tau, *outs[3])
    torch.cuda.synchronize()
    aj.aj_destroy(h1)
    aj.aj_destroy(h2)
    for o, r in zip(outs, (refs[0], refs[1], refs[1], refs[0])):
        assert np.array_equal(o[0].cpu().numpy(), r.out_len) and np.array_equal(o[1].cpu().numpy(), r.out_tok)


def test_profile_events_and_kernel_names():
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="prof", B=1, K=16, d_t=4096, d_d=64, V=4096)
    x = make_inputs(w, 3)
    dev = [aj.device_tensor(a) for a in (x.ht, x.hd, x.W, np.zeros((w.B, w.K), np.int32), x.cw)]
    o = [torch.zeros(w.B, dtype=torch.int32, device="cuda") for _ in range(2)]
    h = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16, 1, aj.AJ_FLAG_PROFILE)
    assert aj.aj_kernel_name(h) == "lm_head_stream16_bf16"
    assert aj.aj_profile_read(h) == []
    for _ in range(5):
        aj.aj_verify(h, *dev, 0.0, 0.5, *o)
    ms = aj.aj_profile_read(h)
    assert len(ms) == 5 and all(0.0 < t < 50.0 for t in ms)
    aj.aj_destroy(h)
    plain = aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, aj.AJ_BF16)
    with pytest.raises(aj.AjError):
        aj.aj_profile_read(plain)
    aj.aj_destroy(plain)
    for M_B, d_t, name in ((8, 4096, "lm_head_wide_bf16"), (8, 4096 + 64, "lm_head_big_bf16"), (4, 4096, "lm_head_wide_bf16"), (3, 4096, "lm_head_resident_bf16"), (4, 4096 + 128, "lm_head_stream_bf16"), (5, 4096, "lm_head_wide_bf16"), (5, 4096 + 128, "lm_head_big_bf16"),
                           (4, 4096 + 8, "lm_head_tile_bf16"), (9, 4096, "lm_head_pair9_bf16"), (10, 4096, "lm_head_tall_bf16"),
                           (33, 4096, "lm_head_pair9_bf16"), (33, 4096 + 64, "lm_head_tall_bf16"),
                           (260, 4096, "lm_head_pair_bf16")):
        hh = aj.aj_create(M_B, 31, d_t, 64, 4096, aj.AJ_BF16)     # 256, 256, 128, 128, 160, 160, 128, 288, 320, 1056, 1056, 8320 verify rows
        assert aj.aj_kernel_name(hh) == name, (M_B, aj.aj_kernel_name(hh))
        aj.aj_destroy(hh)


@pytest.mark.parametrize("kernel,shape", [
    (2, dict(B=1, K=16, d_t=4096, d_d=64, V=20000)),
    (3, dict(B=8, K=31, d_t=512, d_d=64, V=5000)),
    (4, dict(B=9, K=31, d_t=512, d_d=64, V=5000)),
    (5, dict(B=9, K=31, d_t=768, d_d=64, V=5000)),
    (6, dict(B=9, K=31, d_t=768, d_d=64, V=5000)),
    (7, dict(B=3, K=31, d_t=768, d_d=64, V=20000)),
    (8, dict(B=8, K=32, d_t=768, d_d=64, V=70000)),
])
def test_run_to_run_bit_identical(kernel, shape):
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="det", p_match=0.5, **shape)
    parity_case(w, 17, kernel=kernel, repeat=100)


@pytest.mark.parametrize("d_t", [512, 320, 200])       # whole-line kernels; 64-byte-piece kernels; general kernel only
@pytest.mark.parametrize("B,K", [(1, 31), (1, 32), (2, 31), (5, 12), (4, 31), (3, 42), (8, 31), (1, 256), (9, 31),
                                 (17, 16), (10, 31), (3, 106), (16, 31), (19, 26), (18, 31), (1, 576)])
def test_dispatch_boundaries(B, K, d_t):
    """Row counts on both sides of every dispatch boundary (32|33, 64|65, 128|129, 256|257, 288|289, 320|321,
    512|513, 576|577), whatever kernel AUTO picks at each hidden size."""
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="edge", p_match=0.6, B=B, K=K, d_t=d_t, d_d=64, V=1500)
    rep, x, draft, greedy, gpu = parity_case(w, 29, repeat=2)
    assert rep["near_thr_windows"] == 0
