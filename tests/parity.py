"""GPU-vs-oracle comparison protocol for the row solvers.

The oracle is fed exactly what the GPU solver was fed (the fp32 inverse Hessian, weights and grid,
up-cast to fp64).  Tolerances (stated by the build's target):

* order / masks: identical wherever the oracle's candidate gap exceeds 1e-6 relative.  At a
  mismatch the GPU's pick must score within 1e-6 relative of the oracle's minimum in the oracle's
  own state; the oracle then follows the GPU's order (swapping two near-tied picks gives the same
  state two steps later), so one benign swap does not cascade.
  What an inverse Hessian stored in fp32 can resolve is coarser than that late in a long row: every
  elimination rounds the matrix at 2^-24 of its entries, the rows of the matrix move the weights,
  and the OBQ score (q(w) - w)^2 / [H^-1]_pp takes a difference of nearby numbers.  A literal fp32
  Algorithm 1 on the CPU (tests/test_fp32_resolution.py) shows relative score errors of several
  1e-6 in the last steps of a row.  A pick whose gap lies between 1e-6 and FP32_ORDER_GAP = 2^-15
  is therefore not failed outright: it is counted (``beyond_gap``, with the largest gap seen), the
  oracle follows it like a near-tie, and ``assert_order_rule`` requires such picks to be rarer than
  one in BEYOND_GAP_ONE_IN steps of the sample.  A pick beyond 2^-15 fails at once.
* surviving weights: ||w_gpu - w_orc||_2 <= 1e-4 ||w_orc||_2 per row
* loss changes: the row's accumulated loss within 1e-3 relative
* quantized codes: exact, except where the oracle's pre-rounding value lies within 1e-4 of a
  half-integer at the moment of choice (fp32 and fp64 cannot agree there)
"""
import numpy as np

ORDER_GAP = 1e-6
FP32_ORDER_GAP = 2.0 ** -15
BEYOND_GAP_ONE_IN = 16384
W_RTOL = 1e-4
LOSS_RTOL = 1e-3
HALF_EPS = 1e-4


class RowParity:
    def __init__(self):
        self.rows = 0
        self.steps = 0
        self.order_mismatch_rows = 0
        self.near_ties = 0
        self.beyond_gap = 0
        self.max_gap = 0.0
        self.code_exempt = 0
        self.max_w_err = 0.0
        self.max_loss_err = 0.0

    def __repr__(self):
        return ("RowParity(rows=%d steps=%d rows_with_swaps=%d near_ties=%d beyond_1e-6=%d max_gap=%.2e "
                "code_exempt=%d max_w_err=%.2e max_loss_err=%.2e)" % (
                    self.rows, self.steps, self.order_mismatch_rows, self.near_ties, self.beyond_gap,
                    self.max_gap, self.code_exempt, self.max_w_err, self.max_loss_err))

    def assert_order_rule(self):
        """Picks beyond the 1e-6 gap (all within FP32_ORDER_GAP, or check_row has failed already)
        must be rarer than one in BEYOND_GAP_ONE_IN sampled steps."""
        assert self.beyond_gap * BEYOND_GAP_ONE_IN <= self.steps, repr(self)


def check_row(orc, stats, mode, Hinv32, w32, g_order, g_loss, g_w, k_steps, nm=(0, 0), grid=None,
              g_codes=None, live=None, g_trace=None, outlier=False):
    """Compare one GPU row with the oracle.  All g_* are numpy arrays of the GPU outputs."""
    A = np.asarray(Hinv32, np.float64)
    w = np.asarray(w32, np.float64)
    d = w.shape[0]
    S = np.arange(d) if live is None else np.flatnonzero(np.asarray(live) != 0)
    sub = live is not None and S.size < d
    if sub:
        # survivors only: the oracle works on the dense sub-problem, whose inverse it forms by
        # direct inversion of the sub-Hessian; here the sub-Hessian is inv(A)[S, S]
        H = np.linalg.inv(A)
        H = 0.5 * (H + H.T)
        A = orc.invert(H[np.ix_(S, S)])
        w = w[S]
        remap = -np.ones(d, np.int64)
        remap[S] = np.arange(S.size)
        g_order_l = remap[np.asarray(g_order[:k_steps], np.int64)]
        assert np.all(g_order_l >= 0), "GPU picked a dead index"
    else:
        g_order_l = np.asarray(g_order[:k_steps], np.int64)
    assert len(set(g_order_l.tolist())) == k_steps, "GPU order repeats an index"

    def run(forced):
        if mode == "prune":
            return orc.prune_row(A, w, k_steps=k_steps, nm=nm, forced=forced, want_trace=g_trace is not None)
        return orc.quant_row(A, w, grid, k_steps=k_steps, forced=forced, outlier=outlier)

    r = run(None)
    stats.rows += 1
    stats.steps += k_steps
    if not np.array_equal(r.order, g_order_l):
        stats.order_mismatch_rows += 1
        r = run(g_order_l.astype(np.int32))
        scale = float(np.max(r.min_score)) if k_steps else 0.0
        gap = r.pick_score - r.min_score
        # (with the outlier heuristic the oracle's minimum runs over the outliers only, so a pick
        # from outside that set can also score lower: both signs of the gap are checked)
        beyond = np.abs(gap) > ORDER_GAP * r.min_score + 1e-12 * scale
        bad = np.abs(gap) > FP32_ORDER_GAP * r.min_score + 1e-12 * scale
        assert not np.any(bad), "GPU pick beyond what fp32 storage explains at steps %s (gaps %s)" % (
            np.flatnonzero(bad)[:5], (gap / np.maximum(r.min_score, 1e-300))[bad][:5])
        stats.near_ties += int(np.count_nonzero((gap > 0) & ~beyond))
        stats.beyond_gap += int(np.count_nonzero(beyond))
        if np.any(beyond):
            stats.max_gap = max(stats.max_gap, float(np.max((np.abs(gap) / np.maximum(r.min_score, 1e-300))[beyond])))
    # weights
    gw = np.asarray(g_w, np.float64)
    gw_l = gw[S] if sub else gw
    if sub:
        dead = np.setdiff1d(np.arange(d), S)
        assert np.all(gw[dead] == 0.0)
    ref = r.w
    nrm = np.linalg.norm(ref)
    err = np.linalg.norm(gw_l - ref)
    if nrm > 0:
        stats.max_w_err = max(stats.max_w_err, err / nrm)
        assert err <= W_RTOL * nrm, "weights differ: rel %.3e" % (err / nrm)
    else:
        assert err == 0.0
    chosen = g_order_l
    if mode == "prune":
        assert np.all(gw_l[chosen] == 0.0), "pruned weights must be exactly zero"
    # losses
    gl = np.asarray(g_loss[:k_steps], np.float64)
    tot = r.loss.sum()
    if tot > 0:
        e = abs(gl.sum() - tot) / tot
        stats.max_loss_err = max(stats.max_loss_err, e)
        assert e <= LOSS_RTOL, "accumulated loss differs: rel %.3e" % e
    assert np.allclose(gl, r.loss, rtol=5e-3, atol=1e-6 * (np.max(r.loss) if k_steps else 0.0))
    # codes
    if mode == "quant" and g_codes is not None:
        gc = np.asarray(g_codes)
        gc_l = gc[S] if sub else gc
        if sub:
            assert np.all(gc[np.setdiff1d(np.arange(d), S)] == -1)
        diff = np.flatnonzero(gc_l != r.codes)
        if diff.size:
            # the step at which each differing index was chosen
            step_of = np.empty(len(w), np.int64)
            step_of[r.order] = np.arange(k_steps)
            frac = np.abs(r.pre_round[step_of[diff]] - np.floor(r.pre_round[step_of[diff]]) - 0.5)
            assert np.all(frac < HALF_EPS), "codes differ away from a rounding boundary at %s" % diff[:5]
            stats.code_exempt += diff.size
        delta, offset, maxq = grid
        assert gc_l.min() >= 0 and gc_l.max() <= maxq
        # the stored weight is the grid value (fp64 arithmetic on the fp32 grid) rounded to fp32
        deq = (np.float64(offset) + np.float64(delta) * gc_l.astype(np.float64)).astype(np.float32)
        assert np.array_equal(gw_l.astype(np.float32), deq)
    if g_trace is not None and mode == "prune":
        gt = np.asarray(g_trace[:k_steps], np.float64)
        if sub:
            assert np.all(gt[:, np.setdiff1d(np.arange(d), S)] == 0.0)
            gt = gt[:, S]
        num = np.linalg.norm(gt - r.trace, axis=1)
        den = np.linalg.norm(r.trace, axis=1)
        ok = num <= W_RTOL * den + 1e-30
        assert np.all(ok), "trace differs at steps %s" % np.flatnonzero(~ok)[:5]
    return r


def check_block_row(orc, Hinv32, w32, c, g_order, g_loss, g_w, k_blocks, g_trace=None):
    """Block pruning (blocks of c): compare one GPU row with the oracle, same protocol as check_row
    with blocks as the unit.  Returns True when the oracle had to follow a near-tie swap."""
    A = np.asarray(Hinv32, np.float64)
    w = np.asarray(w32, np.float64)
    g = np.asarray(g_order[:k_blocks], np.int32)
    assert len(set(g.tolist())) == k_blocks, "GPU order repeats a block"
    want_trace = g_trace is not None
    r = orc.block_prune_row(A, w, c, k_blocks=k_blocks, want_trace=want_trace)
    swapped = not np.array_equal(r.order, g)
    if swapped:
        r = orc.block_prune_row(A, w, c, k_blocks=k_blocks, forced=g, want_trace=want_trace)
        gap = r.pick_score - r.min_score
        bad = gap > ORDER_GAP * r.min_score + 1e-12 * r.min_score.max()
        assert not np.any(bad), "GPU block beyond the 1e-6 gap at steps %s" % np.flatnonzero(bad)[:5]
    gw = np.asarray(g_w, np.float64)
    nrm = np.linalg.norm(r.w)
    assert np.linalg.norm(gw - r.w) <= W_RTOL * nrm + 1e-30
    if k_blocks:
        P = np.concatenate([np.arange(b * c, b * c + c) for b in g])
        assert np.all(gw[P] == 0.0), "pruned blocks must be exactly zero"
        gl = np.asarray(g_loss[:k_blocks], np.float64)
        tot = r.loss.sum()
        assert abs(gl.sum() - tot) <= LOSS_RTOL * tot
        assert np.allclose(gl, r.loss, rtol=5e-3, atol=1e-6 * r.loss.max())
    if want_trace:
        gt = np.asarray(g_trace[:k_blocks], np.float64)
        num = np.linalg.norm(gt - r.trace, axis=1)
        assert np.all(num <= W_RTOL * np.linalg.norm(r.trace, axis=1) + 1e-30)
    return swapped


def check_rows(orc, stats, mode, Hinv32, W32, g_order, g_loss, g_w, k_steps, nm=(0, 0), grids=None,
               g_codes=None, n_threads=16):
    """Several rows at once: the oracle's multi-row driver (one row per host thread) runs them
    all; a row whose order and codes equal the GPU's is compared with that run directly, any other
    row goes through check_row (forced replay, near-tie rule, rounding-boundary rule).

    grids = (delta[rows], offset[rows], maxq) for mode "quant".  g_* hold the sampled rows only.
    """
    A = np.asarray(Hinv32, np.float64)
    W = np.asarray(W32, np.float64)
    n, d = W.shape
    if mode == "prune":
        ro = orc.prune_rows(A, W, k_steps=k_steps, nm=nm, n_threads=n_threads)
    else:
        assert k_steps == d
        ro = orc.quant_rows(A, W, np.asarray(grids[0], np.float64), np.asarray(grids[1], np.float64), grids[2],
                            n_threads=n_threads)
    for i in range(n):
        go = np.asarray(g_order[i][:k_steps], np.int64)
        same = np.array_equal(go, ro["order"][i])
        if same and mode == "quant" and g_codes is not None:
            same = np.array_equal(np.asarray(g_codes[i]), ro["codes"][i])
        if not same:
            grid = None if mode == "prune" else (float(grids[0][i]), float(grids[1][i]), grids[2])
            check_row(orc, stats, mode, Hinv32, W32[i], g_order[i], g_loss[i], g_w[i], k_steps, nm=nm, grid=grid,
                      g_codes=None if g_codes is None else g_codes[i])
            continue
        stats.rows += 1
        stats.steps += k_steps
        gw = np.asarray(g_w[i], np.float64)
        ref = ro["W"][i]
        nrm, err = np.linalg.norm(ref), np.linalg.norm(gw - ref)
        if nrm > 0:
            stats.max_w_err = max(stats.max_w_err, err / nrm)
            assert err <= W_RTOL * nrm, "row %d: weights differ: rel %.3e" % (i, err / nrm)
        else:
            assert err == 0.0
        if mode == "prune":
            assert np.all(gw[go] == 0.0), "pruned weights must be exactly zero"
        gl = np.asarray(g_loss[i][:k_steps], np.float64)
        tot = ro["loss"][i].sum()
        if tot > 0:
            e = abs(gl.sum() - tot) / tot
            stats.max_loss_err = max(stats.max_loss_err, e)
            assert e <= LOSS_RTOL, "row %d: accumulated loss differs: rel %.3e" % (i, e)
        assert np.allclose(gl, ro["loss"][i], rtol=5e-3, atol=1e-6 * (np.max(ro["loss"][i]) if k_steps else 0.0))
        if mode == "quant":
            delta, offset, maxq = float(grids[0][i]), float(grids[1][i]), grids[2]
            gc = np.asarray(g_codes[i])
            deq = (np.float64(offset) + np.float64(delta) * gc.astype(np.float64)).astype(np.float32)
            assert np.array_equal(gw.astype(np.float32), deq)
    return ro
