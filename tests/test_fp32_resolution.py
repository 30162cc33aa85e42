"""What an inverse Hessian stored in fp32 can resolve (the bound FP32_ORDER_GAP of tests/parity.py).

A literal Algorithm 3 (arxiv 2208.11580, Sec. 5 / Appendix) is run on the CPU with the row's copy of
H^-1 held in fp32 -- one rounding per entry and step, the least any fp32 implementation does -- and
the weights and the diagonal in fp64, fed from the fp32 rows.  The oracle follows the same order in
fp64 from the same fp32 input.  The relative difference of the two sides' candidate scores grows
along the row: it passes 1e-6 well before the end (so "identical order wherever the gap exceeds
1e-6" cannot hold at every step of a long row for fp32 storage, whatever the kernel) and stays below
2^-15.  No GPU code is involved."""
import numpy as np

import obc_inputs
from tests.parity import FP32_ORDER_GAP, ORDER_GAP


def _scores(w, dg, grid):
    dl, of, mq = grid
    c = np.clip(np.rint((w - of) / dl), 0, mq)
    e = of + dl * c - w
    with np.errstate(all="ignore"):      # eliminated entries hold stale values and are masked by the caller
        return e * e / dg


def test_fp32_matrix_storage_limits_the_order_rule(orc):
    d = 512
    W, X, _ = obc_inputs.make_layer("conv256x2304", device="cpu", d_row=3, d_col=d, n_samples=6000)
    A32 = orc.invert(orc.hessian(X.numpy())).astype(np.float32)
    A64 = A32.astype(np.float64)
    checkpoints = (256, 128, 32, 8, 4)
    worst = {m: 0.0 for m in checkpoints}
    for i in range(3):
        w0 = W[i].numpy().astype(np.float64)
        grid = (float(np.float32((w0.max() - w0.min()) / 15)), float(w0.min()), 15)
        # ---- literal Algorithm 3, matrix in fp32
        A = A32.copy()
        w, dg = w0.copy(), np.diag(A64).copy()
        live = np.ones(d, bool)
        order, snaps = [], {}
        for t in range(d):
            if d - t in checkpoints:
                snaps[d - t] = (w.copy(), dg.copy(), live.copy())
            s = _scores(w, dg, grid)
            s[~live] = np.inf
            p = int(np.argmin(s))
            order.append(p)
            dl, of, mq = grid
            tq = of + dl * np.clip(np.rint((w[p] - of) / dl), 0, mq)
            col = A[p].copy()
            cd = col.astype(np.float64)
            g = (w[p] - tq) / dg[p]
            w -= cd * g
            w[p] = tq
            A -= np.outer(col * np.float32(1.0 / dg[p]), col)         # fp32: one rounding per entry
            dg = dg - cd * cd / dg[p]
            live[p] = False
        order = np.asarray(order, np.int32)
        # ---- the oracle along the same order, state at the checkpoints
        for m in checkpoints:
            r = orc.quant_row(A64, w0, grid, k_steps=d - m, forced=order)
            ws, dgs, lv = snaps[m]
            L = np.flatnonzero(lv)
            so = _scores(r.w[L], np.diag(r.A)[L], grid)
            ss = _scores(ws[L], dgs[L], grid)
            ok = so > 1e-12 * so.max()
            worst[m] = max(worst[m], float(np.max(np.abs(ss[ok] - so[ok]) / so[ok])))
    print("relative score error of fp32 storage by live size:", worst)
    assert max(worst[m] for m in (32, 8, 4)) > ORDER_GAP
    assert max(worst.values()) < FP32_ORDER_GAP
    assert worst[4] + worst[8] > worst[256]          # it grows along the row
