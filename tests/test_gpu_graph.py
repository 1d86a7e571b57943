"""aj_verify and aj_verify_static enqueue kernels only (no allocation, no memset, no synchronisation), so a caller can
capture them in a HIP graph.  A graph of one call is replayed several times, with the program's own eager work and
synchronisations between the replays and with new inputs written into the captured buffers, and every replay is checked
against the eager call on the same inputs."""
import numpy as np
import pytest

import workloads as wl
from parity import make_inputs, oracle_greedy

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,static", [
    (dict(B=1, K=16, d_t=4096, d_d=64, V=5003), False),      # one-launch tail, 16-row-tile kernel
    (dict(B=1, K=64, d_t=1024, d_d=64, V=9000), False),      # split tail, accumulator-resident kernel
    (dict(B=4, K=32, d_t=512, d_d=64, V=3000), False),       # wide kernel
    (dict(B=4, K=32, d_t=512, d_d=64, V=3000), True),        # the entry point that allocates nothing
])
def test_a_captured_call_replays_like_the_eager_one(shape, static):
    import torch
    import paper_2504_20039_amd as aj
    w = wl.scaled(wl.WORKLOADS["8b_b1_k16"], name="graph", p_match=0.85, **shape)
    x = make_inputs(w, 11)
    greedy = oracle_greedy(x)
    drafts = [np.ascontiguousarray(wl.draft_tokens(w, seed, greedy[0]), np.int32) for seed in (11, 12, 13)]
    ht, hd, W, cw = (aj.device_tensor(a) for a in (x.ht, x.hd, x.W, x.cw))
    d_draft = aj.device_tensor(drafts[0])
    h = None if static else aj.aj_create(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, 1, 0, 0)

    def call(draft, ol, ot):
        if static:
            aj.aj_verify_static(w.B, w.K, w.d_t, w.d_d, w.V, w.dtype_code, 1, 0, ht, hd, W, draft, cw, w.clf_b, w.tau, ol, ot)
        else:
            aj.aj_verify(h, ht, hd, W, draft, cw, w.clf_b, w.tau, ol, ot)

    try:
        eager = []
        for dr in drafts:
            ol = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
            ot = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
            call(aj.device_tensor(dr), ol, ot)
            torch.cuda.synchronize()
            eager.append((ol.cpu().numpy().copy(), ot.cpu().numpy().copy()))
        if w.B >= 4:      # (the replays below are told apart by their results)
            assert any(not np.array_equal(eager[0][0], e[0]) or not np.array_equal(eager[0][1], e[1]) for e in eager[1:])

        g_len = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
        g_tok = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            call(d_draft, g_len, g_tok)              # a warm-up on the capture stream
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            call(d_draft, g_len, g_tok)
        for rnd in range(2):
            for i, dr in enumerate(drafts):
                d_draft.copy_(torch.from_numpy(dr).cuda())
                g_len.fill_(-7)                      # eager work of the program between the replays
                g_tok.fill_(-7)
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                assert np.array_equal(g_len.cpu().numpy(), eager[i][0]), (rnd, i)
                assert np.array_equal(g_tok.cpu().numpy(), eager[i][1]), (rnd, i)
    finally:
        if h is not None:
            aj.aj_destroy(h)
