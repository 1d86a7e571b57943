"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle's greedy rows (the expensive steps 1-2) come from tests/golden/, written by
make_golden.py from the oracle alone and guarded by digests of the regenerated inputs: if a stored
file does not fit the regenerated inputs the test FAILS and names the tensor (tests/test_workloads.py
checks the same digests without a GPU).  Only for a workload with no stored file does the test compute
oracle rows on the spot, for two sampled windows, and compare those windows alone (outputs of
different windows are independent); the report line says which of the two ran."""
import numpy as np
import pytest

import workloads as wl
from parity import compare, load_golden, make_inputs, oracle_greedy, run_gpu

pytestmark = pytest.mark.gpu

FULL = ["8b_b1_k16", "8b_b32_k32", "70b_b8_k32", "70b_b128_k64", "70b_b1_k32", "70b_b1_k64"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_parity(name):
    w = wl.WORKLOADS[name]
    seed = wl.DEFAULT_SEED
    x = make_inputs(w, seed)
    greedy = load_golden(x)          # raises when a stored file does not fit the inputs
    windows = None
    source = "stored oracle rows, all windows"
    if greedy is None:
        source = "no stored file: oracle on the spot, windows 0 and B-1"
        windows = sorted({0, w.B - 1})
        greedy = oracle_greedy(x, windows)
    draft = wl.draft_tokens(w, seed, greedy[0])
    for tau in (w.taus or (w.tau,)):
        gpu = run_gpu(x, draft, tau, repeat=2 if tau == w.tau else 1)
        rep = compare(x, draft, tau, greedy, gpu, windows=windows)
        print(f"\n[{name} tau={tau}] ({source}) {rep}", flush=True)
        assert rep["windows"] == (w.B if windows is None else len(windows))
        R = w.K + 1
        # properties that hold at any size, on every window
        assert ((gpu["out_len"] >= 0) & (gpu["out_len"] <= w.K)).all()
        assert np.array_equal(gpu["out_tok"], gpu["t_star"][np.arange(w.B) * R + gpu["out_len"]])
        if tau == 1.0:
            assert (gpu["out_len"] == w.K).all()
        if tau == 0.0:
            ts = gpu["t_star"].reshape(w.B, R)
            lcp = np.array([next((j for j in range(w.K) if draft[b, j] != ts[b, j]), w.K) for b in range(w.B)])
            assert np.array_equal(gpu["out_len"], lcp)
