"""Writes tests/golden/lbs_block_cfg<C>_<layer>.json: the oracle's COMPLETE local block shuffle
(Algorithm 1 run to termination) of one block of a full-size matrix.

  config 2, q/k/v/o 4096 x 4096, blocks of 64, block 17
  config 5, qkv/out 9216 x 9216, blocks of 128, block 40

Scores come from the first T_SUB = 1024 rows of the configuration's calibration set (the oracle
computes them completely), the global naive shuffle runs over all K channels, and the block's
search is run with the row sums of eq. (5) taken in the oracle's plain order and, as a cross-check
that the result does not hinge on that order, in 16 interleaved sub-sums and exactly (math.fsum).

Calls only the CPU oracle and the seeded input generators.  Run from the repository root (the
second case takes a few hours of CPU time):
    python tests/golden/make_lbs_block_golden.py 2
    python tests/golden/make_lbs_block_golden.py 5
"""
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402
from oracle import esparse_oracle as orc  # noqa: E402

T_SUB = 1024
CASES = {2: ("qkvo", 64, 17), 5: ("qkv_out", 128, 40)}


def sha(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def main(cfg: int, orders):
    layer, B, blk = CASES[cfg]
    t0 = time.time()
    W = wl.weights(cfg, layer).numpy()
    Xc = wl.calibration(cfg, layer, T=T_SUB).numpy()
    N, K = W.shape
    alpha = wl.default_alpha(T_SUB)
    s = orc.channel_score(Xc, alpha, 100)
    theta0 = orc.global_naive_shuffle(W, s, 4)
    print(f"[{time.time() - t0:7.1f}s] scores + GNS done", flush=True)
    ch0 = theta0[blk * B:(blk + 1) * B]
    Wb = W[:, ch0].astype(np.float64)
    results = {}
    for order in orders:
        sub, nsw = orc.local_block_shuffle_vectorised(Wb, s[ch0], np.arange(B), 2, 4, B, order=order)
        results[str(order)] = (ch0[sub].tolist(), int(nsw[0]))
        print(f"[{time.time() - t0:7.1f}s] order {order}: {int(nsw[0])} swaps", flush=True)
    first = results[str(orders[0])]
    agree = all(r == first for r in results.values())
    assert agree, "the block's result depends on the order of the row sums"
    out = {
        "cfg": cfg, "layer": layer, "N": N, "K": K, "B": B, "block": blk, "T_sub": T_SUB, "alpha": alpha,
        "inputs_sha256": {"W": sha(W), "Xc": sha(Xc)},
        "score_sha256": sha(s),
        "theta0_sha256": sha(theta0),
        "theta0_block": ch0.tolist(),
        "theta_block": first[0],
        "swaps": first[1],
        "row_sum_orders_cross_checked": [str(o) for o in orders],
    }
    path = os.path.join(ROOT, "tests", "golden", f"lbs_block_cfg{cfg}_{layer}.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path, flush=True)


if __name__ == "__main__":
    main(int(sys.argv[1]), ["sequential", ("lanes", 16), "exact"])
