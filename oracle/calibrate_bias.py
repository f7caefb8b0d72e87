"""Calibrate the gate-bias scale ``alpha`` of each skewed workload (run once, by hand).

For every workload with a ``target_ratio`` this bisects ``alpha`` until the
oracle's gate sends ``target_ratio`` times the mean load to the busiest expert
(within 2 %), and writes the constants to
``paper_2602_11686_amd/bias_alpha.json``.  Only the oracle's gate is called;
the HIP path is never involved.  The stored file is an *input* recipe constant
(like a seed), not an expected output.

    python -m oracle.calibrate_bias          # only the workloads that have no stored constant yet
    python -m oracle.calibrate_bias --all    # every workload again
"""
from __future__ import annotations

import json
import os

import numpy as np

from oracle import oracle as O
from paper_2602_11686_amd import inputs as I


def ratio_for(w, X, Wg, alpha):
    b = I.gate_bias(w, alpha).astype(np.float32)
    ids, _, _ = O.gate_topk(X, Wg, b, w.k)
    counts = np.bincount(ids.ravel(), minlength=w.E)
    return counts.max() / (w.T * w.k / w.E), counts


def main():
    import sys
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                        "paper_2602_11686_amd", "bias_alpha.json")
    out = {}
    if "--all" not in sys.argv[1:] and os.path.exists(path):
        with open(path) as fh:
            out = json.load(fh)
    for name, w in I.WORKLOADS.items():
        if w.target_ratio is None or name in out:
            continue
        X = I.widen(I.tokens(w))
        Wg = I.widen(I.gate_weight(w))
        lo, hi = 0.0, 8.0
        for _ in range(40):
            mid = 0.5 * (lo + hi)
            r, counts = ratio_for(w, X, Wg, mid)
            if abs(r / w.target_ratio - 1.0) < 0.005:
                break
            if r < w.target_ratio:
                lo = mid
            else:
                hi = mid
        alpha = float(np.float32(mid))
        r, counts = ratio_for(w, X, Wg, alpha)
        out[name] = {"alpha": alpha, "max_over_mean": float(r), "empty_experts": int((counts == 0).sum()),
                     "counts_sorted": sorted((int(c) for c in counts), reverse=True)}
        print(name, out[name]["alpha"], out[name]["max_over_mean"], out[name]["empty_experts"], flush=True)
    with open(path, "w") as fh:
        json.dump(out, fh, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
