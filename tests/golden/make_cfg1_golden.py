"""Writes tests/golden/cfg1_oracle.json: the oracle's results on workload configuration 1
(single 512x512 fp16 layer, 256 calibration tokens, 2:4, GNS + LBS with blocks of 64).

Calls only the CPU oracle (and the seeded input generators).  Run from the repository root:
    python tests/golden/make_cfg1_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402
from oracle import esparse_oracle as orc  # noqa: E402


def sha(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def main():
    W = wl.weights(1, "linear").numpy()
    Xc = wl.calibration(1, "linear").numpy()
    X = wl.activations(1, "linear", 16).numpy()
    alpha = wl.default_alpha(Xc.shape[0])
    theta, mask, s, swaps = orc.prune(Xc, W, 2, 4, 64, alpha)
    # eq. (5) fixes no order for its sum over the rows: the result must not hinge on the oracle's choice
    theta0 = orc.global_naive_shuffle(W, s, 4)
    orders = ["sequential", ("lanes", 16), "exact"]
    for order in orders[1:]:
        t2, s2 = orc.local_block_shuffle_vectorised(W, s, theta0, 2, 4, 64, order=order)
        assert (t2 == theta).all() and (s2 == swaps).all(), f"result depends on the row-sum order ({order})"
    values, meta = orc.compress_vectorised(W, theta, mask, 2, 4)
    nv, nm = orc.native_tiling(values, meta, *W.shape)
    out = {
        "inputs_sha256": {"W": sha(W), "Xc": sha(Xc), "X": sha(X)},
        "alpha": alpha,
        "theta": theta.tolist(),
        "swaps": swaps.tolist(),
        "score_sha256": sha(s),
        "mask_sha256": sha(mask),
        "values_sha256": sha(values),
        "meta_sha256": sha(meta),
        "native_values_sha256": sha(nv),
        "native_meta_sha256": sha(nm),
        "retained": orc.retained_metric(W, s, theta, 2, 4),
        "row_sum_orders_cross_checked": [str(o) for o in orders],
    }
    path = os.path.join(ROOT, "tests", "golden", "cfg1_oracle.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
