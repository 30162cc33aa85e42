"""Write tests/golden/tiny_layer.json: the oracle's outputs on one tiny seeded layer.

Calls only oracle/ (and numpy).  The values are the oracle's own (a regression fixture), not the
paper's: the paper prints no worked example.  Run from the repository root:

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import oracle as orc  # noqa: E402


def main():
    rng = np.random.default_rng(2208_11580)
    d, R, N = 8, 3, 40
    X = (rng.standard_normal((d, d)) @ rng.standard_normal((d, N))).round(3)
    W = (0.1 * rng.standard_normal((R, d))).round(4)
    H = orc.hessian(X, damp_rel=0.01)
    A = orc.invert(H)
    pr = orc.prune_rows(A, W)
    counts = orc.global_select(pr["loss"], 12)
    Wp = orc.reconstruct(A, W, counts)
    grids = [orc.minmax_grid(W[i], 3) for i in range(R)]
    q = orc.quant_rows(A, W, [g[0] for g in grids], [g[1] for g in grids], 7)
    nm = orc.prune_rows(A, W, nm=(2, 4))
    out = dict(d=d, R=R, N=N, X=X.tolist(), W=W.tolist(), damp_rel=0.01, k=12, bits=3,
               prune_order=pr["order"].tolist(), prune_loss=pr["loss"].tolist(), counts=counts.tolist(),
               W_pruned=Wp.tolist(), quant_order=q["order"].tolist(), quant_codes=q["codes"].tolist(),
               W_quant=q["W"].tolist(), nm24_order=nm["order"].tolist(), W_nm24=nm["W"].tolist())
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_layer.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
