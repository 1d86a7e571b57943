"""Write the stored oracle results for the full-size workloads.

Calls only oracle/ and workloads/ (never the HIP library).  For each workload and
seed it stores what is expensive to recompute - the oracle's greedy token, maximum
logit and runner-up logit of every verify row (steps 1-2) - together with SHA-256
digests of the input tensors, so that a test can tell whether it regenerated the
very same inputs before it trusts the stored rows.  Steps 3-4 are cheap and are
recomputed by the tests from these rows with oracle.walk.

usage: python tests/golden/make_golden.py [workload ...]     (default: all bf16 full-size ones)
"""
import hashlib
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle                      # noqa: E402
import workloads as wl             # noqa: E402


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def path_for(name: str, seed: int) -> str:
    return os.path.join(HERE, f"greedy_{name}_seed{seed}.txt")


def make(name: str, seed: int) -> None:
    w = wl.WORKLOADS[name]
    t0 = time.time()
    ht, W = wl.hidden_t(w, seed), wl.w_lm(w, seed)
    print(f"[{name}] inputs generated in {time.time() - t0:.1f}s; oracle on {w.M} rows, "
          f"{oracle.num_threads()} threads", flush=True)
    t0 = time.time()
    t, m1, m2 = oracle.greedy_rows(ht, W)
    dt = time.time() - t0
    print(f"[{name}] oracle steps 1-2: {dt:.1f}s", flush=True)
    with open(path_for(name, seed), "w") as f:
        f.write(f"# oracle greedy rows (steps 1-2) for workload {name}, seed {seed}\n")
        f.write("# written by tests/golden/make_golden.py from oracle/ and workloads/ only\n")
        f.write(f"# oracle_seconds {dt:.1f} threads {oracle.num_threads()}\n")
        f.write(f"sha256 hidden_t {digest(ht)}\n")
        f.write(f"sha256 W_lm {digest(W)}\n")
        f.write(f"sha256 hidden_d {digest(wl.hidden_d(w, seed))}\n")
        f.write(f"sha256 clf_w {digest(wl.clf_w(w, seed))}\n")
        f.write("# row t_star max1 max2\n")
        for r in range(w.M):
            f.write(f"{r} {int(t[r])} {float(m1[r])!r} {float(m2[r])!r}\n")


if __name__ == "__main__":
    names = sys.argv[1:] or ["8b_b1_k16", "70b_b8_k32", "8b_b32_k32", "70b_b128_k64"]
    for n in names:
        make(n, wl.DEFAULT_SEED)
