"""Pins for the CPU oracle: every check compares it with something other than itself.

Each pin names what fixes the expected value (paper: arxiv 2208.11580):

* closed-form least squares on the surviving support (Sec. 3 eq. (2); Sec. 4 Step 2: a row's
  final weights depend only on which weights were removed; OBS formulas are exact, Sec. 3),
  solved on H with numpy, never touching H^-1
* the loss identity  sum_t dL_t = 1/2 (w - w_hat)^T H (w - w_hat) = ||w X - w_hat X||^2
* brute force over every candidate, d <= 8 (the greedy choice of eq. (3) / eq. (7))
* Lemma 1 against direct inversion of the reduced Hessian
* quant(.) == 0 reduces OBQ to pruning (Sec. 5, after eq. (7))
* a diagonal Hessian reduces everything to textbook routines (magnitude pruning,
  round-to-nearest, top-N per block, global magnitude pruning)
* Appendix Algorithm 2 equals OBS run on the whole matrix (Sec. 4 Step 2)
* invariances (H -> cH, column permutation)
"""
import itertools

import numpy as np
import pytest

RTOL = 1e-9


def _problem(seed, d, n=None, R=1, damp=0.01, cond=30.0):
    rng = np.random.default_rng(seed)
    n = n or 4 * d
    A = rng.standard_normal((d, d)) @ np.diag(np.logspace(0, -np.log10(cond), d))
    X = A @ rng.standard_normal((d, n))
    W = rng.standard_normal((R, d)) * 0.1
    return W, X


def _ls_on_support(H, w, fixed_idx, fixed_val):
    """argmin_v 1/2 (v-w)^T H (v-w)  s.t. v[fixed_idx] = fixed_val, solved on H itself."""
    d = len(w)
    P = np.asarray(fixed_idx, dtype=int)
    S = np.setdiff1d(np.arange(d), P)
    v = np.zeros(d)
    v[P] = fixed_val
    if S.size:
        # stationarity on the free block: H_SS (v_S - w_S) + H_SP (v_P - w_P) = 0
        v[S] = w[S] - np.linalg.solve(H[np.ix_(S, S)], H[np.ix_(S, P)] @ (v[P] - w[P]))
    return v


def _quad(H, a, b):
    e = a - b
    return 0.5 * e @ H @ e


# ----------------------------------------------------------------------------- Hessian, inverse
def test_hessian_is_twice_sum_of_outer_products(orc):
    rng = np.random.default_rng(1)
    X = rng.standard_normal((5, 11)).astype(np.float32)
    H0 = np.zeros((5, 5))
    for n in range(X.shape[1]):
        x = X[:, n].astype(np.float64)
        H0 += 2.0 * np.outer(x, x)
    assert np.allclose(orc.hessian(X, damp_rel=-1), H0, rtol=1e-13, atol=0)
    lam = 0.01 * np.mean(np.diag(H0))
    assert np.allclose(orc.hessian(X, damp_rel=0.01), H0 + lam * np.eye(5), rtol=1e-13, atol=0)


def test_hessian_is_the_hessian_of_the_row_loss(orc):
    # second finite difference of f(v) = ||v X - w X||^2 along random directions equals u^T H u
    rng = np.random.default_rng(2)
    X = rng.standard_normal((6, 40))
    H = orc.hessian(X, damp_rel=-1)
    w = rng.standard_normal(6)
    f = lambda v: np.sum(((v - w) @ X) ** 2)
    for _ in range(4):
        u = rng.standard_normal(6)
        h = 1e-3
        second = (f(w + h * u) - 2 * f(w) + f(w - h * u)) / h**2
        assert np.isclose(second, u @ H @ u, rtol=1e-6)


def test_inverse_matches_lapack_and_identity(orc):
    for d in (1, 2, 7, 33, 96):
        _, X = _problem(10 + d, d)
        H = orc.hessian(X)
        A = orc.invert(H)
        assert np.allclose(A, A.T, rtol=0, atol=0)
        assert np.allclose(A @ H, np.eye(d), atol=1e-8)
        assert np.allclose(A, np.linalg.inv(H), rtol=1e-7, atol=1e-12 * np.abs(A).max())


def test_inverse_rejects_non_spd(orc):
    H = np.array([[1.0, 2.0], [2.0, 1.0]])
    with pytest.raises(orc.OracleError) as e:
        orc.invert(H)
    assert e.value.code == orc.ORC_NOT_SPD


# ----------------------------------------------------------------------------- P1 closed form
@pytest.mark.parametrize("d,k", [(6, 3), (24, 24), (40, 17), (64, 50)])
def test_pruned_row_equals_least_squares_on_support(orc, d, k):
    W, X = _problem(100 + d, d)
    H = orc.hessian(X)
    r = orc.prune_row(orc.invert(H), W[0], k_steps=k, want_trace=True)
    assert len(set(r.order.tolist())) == k
    for t in (0, k // 2, k - 1):
        P = r.order[: t + 1]
        ref = _ls_on_support(H, W[0], P, np.zeros(len(P)))
        assert np.allclose(r.trace[t], ref, rtol=1e-7, atol=1e-10)
        assert np.all(r.trace[t][P] == 0.0)
    assert np.array_equal(r.trace[k - 1], r.w)


def test_nm_row_equals_least_squares_and_pattern(orc):
    d = 32
    W, X = _problem(7, d)
    H = orc.hessian(X)
    for (n, m) in ((2, 4), (4, 8), (1, 4)):
        r = orc.prune_row(orc.invert(H), W[0], nm=(n, m))
        assert len(r.order) == d // m * (m - n)
        zeros = (r.w == 0.0).reshape(-1, m).sum(axis=1)
        assert np.all(zeros == m - n)
        ref = _ls_on_support(H, W[0], r.order, np.zeros(len(r.order)))
        assert np.allclose(r.w, ref, rtol=1e-7, atol=1e-10)


def test_quantized_row_free_weights_are_least_squares(orc):
    d, k = 20, 9
    W, X = _problem(8, d)
    H = orc.hessian(X)
    grid = orc.minmax_grid(W[0], 3)
    r = orc.quant_row(orc.invert(H), W[0], grid, k_steps=k)
    P = r.order
    ref = _ls_on_support(H, W[0], P, r.w[P])
    assert np.allclose(r.w, ref, rtol=1e-7, atol=1e-10)


# ----------------------------------------------------------------------------- P2 loss identity
@pytest.mark.parametrize("mode", ["prune", "nm", "quant"])
def test_loss_trace_sums_to_quadratic_form_and_output_error(orc, mode):
    d = 28
    W, X = _problem(21, d, n=3 * d)
    w = W[0]
    for damp in (-1, 0.01):
        H = orc.hessian(X, damp_rel=damp)
        A = orc.invert(H)
        if mode == "prune":
            r = orc.prune_row(A, w, k_steps=19)
        elif mode == "nm":
            r = orc.prune_row(A, w, nm=(2, 4))
        else:
            r = orc.quant_row(A, w, orc.minmax_grid(w, 2))
        assert np.all(r.loss >= 0)
        assert np.isclose(r.loss.sum(), _quad(H, w, r.w), rtol=1e-8)
        if damp < 0:
            direct = np.sum((w @ X - r.w @ X) ** 2)
            assert np.isclose(r.loss.sum(), direct, rtol=1e-8)


def test_each_loss_change_is_the_step_increase_of_the_quadratic(orc):
    d = 12
    W, X = _problem(22, d)
    H = orc.hessian(X)
    r = orc.prune_row(orc.invert(H), W[0], want_trace=True)
    prev = W[0]
    total = 0.0
    for t in range(d):
        now = _quad(H, W[0], r.trace[t])
        assert np.isclose(now - total, r.loss[t], rtol=1e-6, atol=1e-12)
        total = now
        prev = r.trace[t]


# ----------------------------------------------------------------------------- P3 brute force
@pytest.mark.parametrize("seed", range(6))
def test_greedy_choice_matches_brute_force_pruning(orc, seed):
    d = 5 + seed % 4  # 5..8
    W, X = _problem(300 + seed, d)
    H = orc.hessian(X)
    w0 = W[0]
    r = orc.prune_row(orc.invert(H), w0, want_trace=True)
    removed = []
    base = 0.0
    for t in range(d):
        best, best_cost = None, None
        for p in range(d):
            if p in removed:
                continue
            v = _ls_on_support(H, w0, removed + [p], np.zeros(len(removed) + 1))
            cost = _quad(H, w0, v)
            if best is None or cost < best_cost:
                best, best_cost = p, cost
        assert r.order[t] == best
        assert np.isclose(r.loss[t], best_cost - base, rtol=1e-6, atol=1e-13)
        removed.append(best)
        base = best_cost


@pytest.mark.parametrize("seed", range(6))
def test_greedy_choice_matches_brute_force_quantization(orc, seed):
    d = 5 + seed % 4
    W, X = _problem(400 + seed, d)
    H = orc.hessian(X)
    w0 = W[0]
    delta, offset, maxq = orc.minmax_grid(w0, 2)
    r = orc.quant_row(orc.invert(H), w0, (delta, offset, maxq), want_trace=True)
    fixed, vals = [], []
    cur = w0.copy()
    base = 0.0
    for t in range(d):
        best, best_cost, best_q = None, None, None
        for p in range(d):
            if p in fixed:
                continue
            # quantize the *current* value of weight p (numpy's rint is half-to-even)
            q = offset + delta * float(np.clip(np.rint((cur[p] - offset) / delta), 0, maxq))
            v = _ls_on_support(H, w0, fixed + [p], np.array(vals + [q]))
            cost = _quad(H, w0, v)
            if best is None or cost < best_cost:
                best, best_cost, best_q = p, cost, q
        assert r.order[t] == best
        assert np.isclose(r.loss[t], best_cost - base, rtol=1e-6, atol=1e-13)
        fixed.append(best)
        vals.append(best_q)
        cur = _ls_on_support(H, w0, fixed, np.array(vals))
        assert np.allclose(r.trace[t], cur, rtol=1e-7, atol=1e-10)
        base = best_cost


# ----------------------------------------------------------------------------- P4 Lemma 1
def test_reduced_inverse_equals_inverse_of_reduced_hessian(orc):
    d, k = 30, 13
    W, X = _problem(31, d)
    H = orc.hessian(X)
    r = orc.prune_row(orc.invert(H), W[0], k_steps=k)
    M = np.flatnonzero(r.live)
    assert len(M) == d - k and set(M) == set(range(d)) - set(r.order.tolist())
    direct = np.linalg.inv(H[np.ix_(M, M)])
    assert np.allclose(r.A[np.ix_(M, M)], direct, rtol=1e-7, atol=1e-12 * np.abs(direct).max())


def test_lemma1_single_removal_on_nonsymmetric_matrix(orc):
    # Lemma 1 holds for any invertible matrix; a symmetric example would hide a transposed operand.
    # Feed a non-symmetric "inverse" and check the oracle's elimination against direct inversion.
    rng = np.random.default_rng(5)
    d = 6
    Hn = rng.standard_normal((d, d)) + 4 * np.eye(d)
    Hn_inv = np.linalg.inv(Hn)
    # make index 2 the first pick: every weight is 1 except a zero at index 2 (score 0)
    w = np.ones(d)
    w[2] = 0.0
    r = orc.prune_row(Hn_inv + 0.0, w, k_steps=1)
    # the positive-diagonal requirement may not hold for a random matrix; choose one where it does
    assert r.order[0] == 2
    M = [0, 1, 3, 4, 5]
    direct = np.linalg.inv(Hn[np.ix_(M, M)])
    assert np.allclose(r.A[np.ix_(M, M)], direct, rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------- P5 quant == 0
def test_obq_with_zero_grid_is_pruning(orc):
    d = 26
    W, X = _problem(41, d)
    A = orc.invert(orc.hessian(X))
    rp = orc.prune_row(A, W[0])
    rq = orc.quant_row(A, W[0], (1.0, 0.0, 0))  # single grid point 0
    assert np.array_equal(rp.order, rq.order)
    assert np.array_equal(rp.loss, rq.loss)
    assert np.array_equal(rp.w, rq.w)
    assert np.all(rq.codes == 0)


# ----------------------------------------------------------------------------- P6 diagonal Hessian
def test_diagonal_hessian_reduces_to_textbook_routines(orc):
    rng = np.random.default_rng(51)
    d = 24
    h = rng.uniform(0.5, 2.0, d)
    A = np.diag(1.0 / h)
    w = rng.standard_normal(d)
    # pruning: ascending h_j w_j^2, no compensation
    r = orc.prune_row(A, w, k_steps=10)
    expect = np.argsort(h * w * w, kind="stable")[:10]
    assert np.array_equal(r.order, expect)
    keep = np.setdiff1d(np.arange(d), expect)
    assert np.array_equal(r.w[keep], w[keep]) and np.all(r.w[expect] == 0)
    assert np.allclose(r.loss, 0.5 * (h * w * w)[expect], rtol=1e-12)
    # OBQ: round-to-nearest of every weight, independent of order
    grid = orc.minmax_grid(w, 3)
    rq = orc.quant_row(A, w, grid)
    rtn = np.clip(np.rint((w - grid[1]) / grid[0]), 0, grid[2]).astype(int)
    assert np.array_equal(rq.codes, rtn)
    assert np.array_equal(rq.w, grid[1] + grid[0] * rtn)
    # 2:4 with identity Hessian: keep the two largest magnitudes of every block of four
    r24 = orc.prune_row(np.eye(d), w, nm=(2, 4))
    for b in range(d // 4):
        blk = np.abs(w[4 * b : 4 * b + 4])
        kept = np.flatnonzero(r24.w[4 * b : 4 * b + 4] != 0)
        assert set(kept) == set(np.argsort(blk)[2:])


def test_global_select_with_diagonal_hessian_is_global_magnitude_pruning(orc):
    rng = np.random.default_rng(52)
    R, d, k = 5, 12, 23
    W = rng.standard_normal((R, d))
    res = orc.prune_rows(np.eye(d), W)
    counts = orc.global_select(res["loss"], k)
    mask = orc.mask_from_counts(res["order"], counts, d)
    thresh = np.sort(np.abs(W).ravel())[k - 1]
    assert mask.sum() == k
    assert np.array_equal(mask.astype(bool), np.abs(W) <= thresh)


# ----------------------------------------------------------------------------- P7 Algorithm 2
@pytest.mark.parametrize("seed,k", [(0, 7), (1, 1), (2, 14), (3, 15), (4, 0)])
def test_global_select_equals_obs_on_the_whole_matrix(orc, seed, k):
    R, d = 3, 5
    W, X = _problem(600 + seed, d, R=R)
    H = orc.hessian(X)
    A = orc.invert(H)
    res = orc.prune_rows(A, W, want_trace=True)
    counts = orc.global_select(res["loss"], k)
    assert counts.sum() == k
    # literal OBS on the flattened matrix: block-diagonal Hessian, one weight at a time
    big = orc.prune_row(np.kron(np.eye(R), A), W.ravel(), k_steps=k)
    whole_mask = np.zeros(R * d, np.uint8)
    whole_mask[big.order] = 1
    assert np.array_equal(orc.mask_from_counts(res["order"], counts, d), whole_mask.reshape(R, d))
    assert np.allclose(orc.reconstruct(A, W, counts), big.w.reshape(R, d), rtol=1e-8, atol=1e-12)
    for i in range(R):
        if counts[i] > 0:
            assert np.array_equal(orc.reconstruct(A, W, counts)[i], res["trace"][i, counts[i] - 1])


def test_global_select_follows_next_loss_not_sorted_losses(orc):
    # non-monotone traces: Algorithm 2 can only take a row's losses in order
    L = np.array([[5.0, 1.0, 9.0], [2.0, 8.0, 0.5]])
    assert orc.global_select(L, 1).tolist() == [0, 1]
    assert orc.global_select(L, 2).tolist() == [1, 1]   # 5 < 8
    assert orc.global_select(L, 3).tolist() == [2, 1]   # then the 1 behind the 5
    assert orc.global_select(L, 4).tolist() == [2, 2]   # 8 < 9
    assert orc.global_select(L, 5).tolist() == [2, 3]   # 0.5 < 9
    assert orc.global_select(L, 6).tolist() == [3, 3]
    # ties go to the lowest row
    T = np.array([[1.0, 1.0], [1.0, 1.0]])
    assert orc.global_select(T, 1).tolist() == [1, 0]
    assert orc.global_select(T, 3).tolist() == [2, 1]


# ----------------------------------------------------------------------------- P8 invariances
def test_scaling_and_permutation_invariance(orc):
    d = 18
    W, X = _problem(71, d)
    H = orc.hessian(X)
    A = orc.invert(H)
    w = W[0]
    r = orc.prune_row(A, w, want_trace=True)
    c = 4.0  # power of two: exact in floating point
    rc = orc.prune_row(orc.invert(c * H), w, want_trace=True)
    assert np.array_equal(r.order, rc.order)
    assert np.allclose(rc.loss, c * r.loss, rtol=1e-9)
    assert np.allclose(rc.trace, r.trace, rtol=1e-9, atol=1e-14)
    perm = np.random.default_rng(3).permutation(d)
    rp = orc.prune_row(orc.invert(H[np.ix_(perm, perm)]), w[perm], want_trace=True)
    assert np.array_equal(perm[rp.order], r.order)
    assert np.allclose(rp.trace, r.trace[:, perm], rtol=1e-8, atol=1e-13)
    # a grid no weight sits on exactly (the min-max grid has two zero-error ties, which
    # the lowest-index rule would break differently after a permutation)
    g = orc.minmax_grid(w, 4)
    grid = (g[0] * 1.07, g[1] - 0.013, g[2])
    q = orc.quant_row(A, w, grid)
    qp = orc.quant_row(orc.invert(H[np.ix_(perm, perm)]), w[perm], grid)
    assert np.array_equal(perm[qp.order], q.order)
    assert np.array_equal(qp.codes, q.codes[perm])


# ----------------------------------------------------------------------------- P9 / P10
def test_quantized_codes_lie_on_the_grid(orc):
    d = 48
    W, X = _problem(81, d)
    A = orc.invert(orc.hessian(X))
    for bits in (2, 3, 4):
        delta, offset, maxq = orc.minmax_grid(W[0], bits)
        r = orc.quant_row(A, W[0], (delta, offset, maxq))
        assert sorted(r.order.tolist()) == list(range(d))
        assert r.codes.min() >= 0 and r.codes.max() <= maxq
        assert np.array_equal(r.w, offset + delta * r.codes)
        assert np.all(np.diff(np.cumsum(r.loss)) >= 0)
    # OBQ is not plain rounding: with a correlated Hessian at least one code differs from RTN
    rtn = np.clip(np.rint((W[0] - offset) / delta), 0, maxq).astype(int)
    assert np.any(rtn != r.codes)
    # and it does not do worse than RTN on the layer objective
    H = orc.hessian(X)
    assert _quad(H, W[0], r.w) <= _quad(H, W[0], offset + delta * rtn) * (1 + 1e-12)


def test_quantizer_rounds_half_to_even_and_clamps(orc):
    assert orc.quant_code(0.5, 1.0, 0.0, 15) == 0
    assert orc.quant_code(1.5, 1.0, 0.0, 15) == 2
    assert orc.quant_code(2.5, 1.0, 0.0, 15) == 2
    assert orc.quant_code(-3.0, 1.0, 0.0, 15) == 0
    assert orc.quant_code(99.0, 1.0, 0.0, 15) == 15
    assert orc.quant_code(0.26, 0.1, 0.05, 3) == 2
    assert orc.minmax_grid(np.array([2.0, 2.0]), 4) == (1.0, 2.0, 15)


def test_zero_weight_is_taken_first_with_zero_update(orc):
    d = 10
    W, X = _problem(91, d)
    A = orc.invert(orc.hessian(X))
    w = W[0].copy()
    w[6] = 0.0
    w[3] = 0.0
    r = orc.prune_row(A, w, k_steps=2, want_trace=True)
    assert r.order.tolist() == [3, 6]           # both score 0: lowest index first
    assert np.all(r.loss == 0.0)
    assert np.array_equal(r.trace[1], w)


def test_forced_order_replays_and_reports_scores(orc):
    d = 14
    W, X = _problem(95, d)
    A = orc.invert(orc.hessian(X))
    r = orc.prune_row(A, W[0])
    rf = orc.prune_row(A, W[0], forced=r.order)
    assert np.array_equal(rf.loss, r.loss) and np.array_equal(rf.pick_score, rf.min_score)
    swapped = r.order.copy()
    swapped[[0, 1]] = swapped[[1, 0]]
    rs = orc.prune_row(A, W[0], forced=swapped)
    assert rs.pick_score[0] > rs.min_score[0]
    # two steps later the state is the same whatever the order of the two removals
    assert np.allclose(rs.w, r.w, rtol=1e-9, atol=1e-14)


# ----------------------------------------------------------------------------- compound
def test_compound_row_is_obq_on_the_reduced_problem(orc):
    d = 24
    W, X = _problem(97, d)
    H = orc.hessian(X)
    A = orc.invert(H)
    rp = orc.prune_row(A, W[0], nm=(2, 4))
    w_out, codes, rq = orc.compound_row(H, rp.w, rp.live, 4)
    S = np.flatnonzero(rp.live)
    assert np.all(w_out[rp.live == 0] == 0) and np.all(codes[rp.live == 0] == -1)
    assert np.all(codes[S] >= 0)
    # continuing Algorithm 3 on the oracle's own reduced inverse (Lemma 1) gives the same run
    grid = orc.minmax_grid(rp.w[S], 4)
    cont = orc.quant_row(rp.A[np.ix_(S, S)], rp.w[S], grid)
    assert np.array_equal(cont.order, rq.order)
    assert np.array_equal(cont.codes, rq.codes)
    assert np.allclose(cont.w, rq.w, rtol=1e-9)


# ----------------------------------------------------------------------------- rows driver
def test_rows_driver_equals_single_rows_and_is_deterministic(orc):
    R, d = 7, 16
    W, X = _problem(99, d, R=R)
    A = orc.invert(orc.hessian(X))
    res = orc.prune_rows(A, W, n_threads=3)
    res2 = orc.prune_rows(A, W, n_threads=1)
    assert res["threads"] == 3 and res2["threads"] == 1
    for i in range(R):
        r = orc.prune_row(A, W[i])
        assert np.array_equal(res["order"][i], r.order)
        assert np.array_equal(res["loss"][i], r.loss)
    assert np.array_equal(res["order"], res2["order"]) and np.array_equal(res["loss"], res2["loss"])
    grids = [orc.minmax_grid(W[i], 4) for i in range(R)]
    q = orc.quant_rows(A, W, [g[0] for g in grids], [g[1] for g in grids], 15)
    for i in range(R):
        r = orc.quant_row(A, W[i], grids[i])
        assert np.array_equal(q["codes"][i], r.codes) and np.array_equal(q["W"][i], r.w)


# ----------------------------------------------------------------------------- regression fixture
def test_oracle_reproduces_its_golden_fixture(orc):
    """tests/golden/tiny_layer.json (written by make_golden.py from the oracle alone) still holds."""
    import json
    import os

    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tiny_layer.json")))
    X, W = np.array(g["X"]), np.array(g["W"])
    A = orc.invert(orc.hessian(X, damp_rel=g["damp_rel"]))
    pr = orc.prune_rows(A, W)
    assert pr["order"].tolist() == g["prune_order"]
    assert np.allclose(pr["loss"], g["prune_loss"], rtol=1e-10)
    counts = orc.global_select(pr["loss"], g["k"])
    assert counts.tolist() == g["counts"]
    assert np.allclose(orc.reconstruct(A, W, counts), g["W_pruned"], rtol=1e-10, atol=1e-15)
    grids = [orc.minmax_grid(W[i], g["bits"]) for i in range(g["R"])]
    q = orc.quant_rows(A, W, [x[0] for x in grids], [x[1] for x in grids], (1 << g["bits"]) - 1)
    assert q["codes"].tolist() == g["quant_codes"] and q["order"].tolist() == g["quant_order"]
    nm = orc.prune_rows(A, W, nm=(2, 4))
    assert nm["order"].tolist() == g["nm24_order"]


# ----------------------------------------------------------------------------- outlier heuristic
def _narrow_grid(orc, w, bits):
    g = orc.minmax_grid(w, bits)
    # a grid covering only the middle of the weight range: several weights start as outliers
    return (0.55 * g[0], g[1] + 0.22 * g[0] * g[2], g[2])


def test_outlier_heuristic_is_inactive_without_outliers(orc):
    d = 22
    W, X = _problem(501, d)
    A = orc.invert(orc.hessian(X))
    g = orc.minmax_grid(W[0], 4)
    wide = (3.0 * g[0], g[1] - g[0] * g[2], g[2])        # range three times the weights' range
    a = orc.quant_row(A, W[0], wide, want_trace=True)
    b = orc.quant_row(A, W[0], wide, outlier=True, want_trace=True)
    # no weight ever leaves the grid's range here, so there is never an outlier
    err = np.abs(a.trace - (wide[1] + wide[0] * np.clip(np.rint((a.trace - wide[1]) / wide[0]), 0, wide[2])))
    assert err.max() <= wide[0] / 2
    assert np.array_equal(a.order, b.order) and np.array_equal(a.codes, b.codes)
    assert np.array_equal(a.loss, b.loss) and np.array_equal(a.w, b.w)


@pytest.mark.parametrize("seed", range(5))
def test_outlier_heuristic_matches_restricted_brute_force(orc, seed):
    """Reading of Sec. 5 'Quantization Outliers': while any live weight has |q(w)-w| > delta/2 the
    greedy choice runs over those weights only; the pick minimises the loss increase among them."""
    d = 6 + seed % 3
    W, X = _problem(520 + seed, d)
    H = orc.hessian(X)
    w0 = W[0]
    delta, offset, maxq = _narrow_grid(orc, w0, 2)
    r = orc.quant_row(orc.invert(H), w0, (delta, offset, maxq), outlier=True, want_trace=True)
    q = lambda v: offset + delta * float(np.clip(np.rint((v - offset) / delta), 0, maxq))
    fixed, vals, cur, base = [], [], w0.copy(), 0.0
    saw_outlier_step = False
    for t in range(d):
        live = [p for p in range(d) if p not in fixed]
        outl = [p for p in live if abs(q(cur[p]) - cur[p]) > delta / 2]
        cands = outl if outl else live
        saw_outlier_step |= bool(outl)
        best, best_cost, best_q = None, None, None
        for p in cands:
            v = _ls_on_support(H, w0, fixed + [p], np.array(vals + [q(cur[p])]))
            cost = _quad(H, w0, v)
            if best is None or cost < best_cost:
                best, best_cost, best_q = p, cost, q(cur[p])
        assert r.order[t] == best
        assert np.isclose(r.loss[t], best_cost - base, rtol=1e-6, atol=1e-13)
        fixed.append(best)
        vals.append(best_q)
        cur = _ls_on_support(H, w0, fixed, np.array(vals))
        assert np.allclose(r.trace[t], cur, rtol=1e-7, atol=1e-10)
        base = best_cost
    assert saw_outlier_step
    assert np.isclose(r.loss.sum(), _quad(H, w0, r.w), rtol=1e-8)          # loss identity still holds
    assert np.array_equal(r.w, offset + delta * r.codes)                   # codes on the grid


def test_outlier_heuristic_lowers_the_error_on_a_clipping_grid(orc):
    d = 40
    W, X = _problem(540, d)
    H = orc.hessian(X)
    A = orc.invert(H)
    grid = _narrow_grid(orc, W[0], 3)
    plain = orc.quant_row(A, W[0], grid)
    heur = orc.quant_row(A, W[0], grid, outlier=True)
    assert not np.array_equal(plain.order, heur.order)
    assert _quad(H, W[0], heur.w) < _quad(H, W[0], plain.w)


def test_symmetric_grid_is_symmetric_about_zero(orc):
    w = np.array([-0.31, 0.12, 0.05, 0.27, -0.02])
    for bits in (2, 3, 4, 8):
        delta, offset, maxq = orc.symmetric_grid(w, bits)
        levels = offset + delta * np.arange(maxq + 1)
        assert np.isclose(levels[0], -0.31) and np.isclose(levels[-1], 0.31)
        assert np.allclose(levels, -levels[::-1])
    assert orc.symmetric_grid(np.zeros(3), 4) == (1.0, -0.0, 15) or orc.symmetric_grid(np.zeros(3), 4)[0] == 1.0


# ----------------------------------------------------------------------------- sequential re-fit
def test_refit_is_linear_regression(orc):
    # appendix "Sequential Quantization with OBQ": without dampening the re-fit is the least-squares
    # solution of W X = Y, here obtained from the library's SVD-based routine on the raw data
    rng = np.random.default_rng(5)
    d_col, d_row, n = 12, 5, 60
    X = rng.standard_normal((d_col, n))
    Y = rng.standard_normal((d_row, n))
    W = orc.refit(orc.hessian(X, damp_rel=-1.0), orc.cross(X, Y))
    ref = np.linalg.lstsq(X.T, Y.T, rcond=None)[0].T
    assert W.shape == (d_row, d_col)
    assert np.allclose(W, ref, rtol=1e-9, atol=1e-12)
    # stationarity: the residual is orthogonal to every input feature
    assert np.allclose((W @ X - Y) @ X.T, 0.0, atol=1e-9)


def test_refit_recovers_weights_of_a_noise_free_layer(orc):
    rng = np.random.default_rng(6)
    d_col, d_row, n = 10, 4, 40
    X = rng.standard_normal((d_col, n))
    W0 = rng.standard_normal((d_row, d_col))
    W = orc.refit(orc.hessian(X, damp_rel=-1.0), orc.cross(X, W0 @ X))
    assert np.allclose(W, W0, rtol=1e-9, atol=1e-11)


def test_dampened_refit_zeroes_the_gradient_of_the_dampened_quadratic(orc):
    # with H = 2 X X^T + lam I the re-fit minimises ||W X - Y||^2 + lam/2 ||W||^2, whose gradient
    # 2 (W X - Y) X^T + lam W is written out here from the data
    rng = np.random.default_rng(7)
    d_col, d_row, n = 9, 3, 30
    X = rng.standard_normal((d_col, n))
    Y = rng.standard_normal((d_row, n))
    H = orc.hessian(X, damp_rel=0.05)
    lam = 0.05 * np.mean(2.0 * np.sum(X * X, axis=1))
    W = orc.refit(H, orc.cross(X, Y))
    grad = 2.0 * (W @ X - Y) @ X.T + lam * W
    assert np.allclose(grad, 0.0, atol=1e-9)
    # and it is a minimum: any perturbation raises the objective
    def obj(V):
        return np.sum((V @ X - Y) ** 2) + 0.5 * lam * np.sum(V * V)
    for _ in range(5):
        assert obj(W + 1e-3 * rng.standard_normal(W.shape)) > obj(W)


# ----------------------------------------------------------------------------- block pruning
def _block_setup(seed, d, c):
    W, X = _problem(seed, d)
    H = 2.0 * X @ X.T
    H += 0.01 * np.mean(np.diag(H)) * np.eye(d)
    return W[0], H, np.linalg.inv(H)


@pytest.mark.parametrize("c,k", [(2, 3), (4, 2), (4, 4), (8, 1)])
def test_block_pruned_row_equals_least_squares_on_support(orc, c, k):
    # Sec. 4 "Block-Sparsity": after k block steps the survivors are the exact minimiser of the
    # layer's quadratic with the chosen blocks held at zero, and zeros come in aligned blocks
    d = 16
    w, H, A = _block_setup(21 + c, d, c)
    r = orc.block_prune_row(A, w, c, k_blocks=k)
    P = np.concatenate([np.arange(b * c, b * c + c) for b in r.order])
    assert len(set(r.order.tolist())) == k
    assert np.all(r.w[P] == 0.0)
    ref = _ls_on_support(H, w, P, np.zeros(P.size))
    assert np.allclose(r.w, ref, rtol=1e-8, atol=1e-11)
    # the recorded losses add up to the true increase of the quadratic
    assert np.isclose(r.loss.sum(), _quad(H, r.w, w), rtol=1e-8)


def test_block_score_is_the_least_squares_cost_of_removing_the_block(orc):
    # eq. (5): the first step's choice is the block whose removal (with optimal compensation)
    # costs least; brute force over all blocks with the constrained least-squares solution
    d, c = 12, 4
    for seed in range(4):
        w, H, A = _block_setup(40 + seed, d, c)
        costs = []
        for b in range(d // c):
            P = np.arange(b * c, b * c + c)
            costs.append(_quad(H, _ls_on_support(H, w, P, np.zeros(c)), w))
        r = orc.block_prune_row(A, w, c, k_blocks=1)
        assert r.order[0] == int(np.argmin(costs))
        assert np.isclose(r.loss[0], min(costs), rtol=1e-8)
        assert np.isclose(r.min_score[0], 2.0 * min(costs), rtol=1e-8)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_block_greedy_matches_brute_force_every_step(orc, seed):
    # every step's choice, not only the first: given the blocks already taken, the next block is
    # the one with the smallest total least-squares cost increase
    d, c = 12, 3
    w, H, A = _block_setup(60 + seed, d, c)
    r = orc.block_prune_row(A, w, c)
    taken = []
    prev = 0.0
    for t in range(d // c):
        best, best_cost = None, None
        for b in range(d // c):
            if b in taken:
                continue
            P = np.concatenate([np.arange(x * c, x * c + c) for x in taken + [b]])
            cost = _quad(H, _ls_on_support(H, w, P, np.zeros(P.size)), w)
            if best is None or cost < best_cost:
                best, best_cost = b, cost
        assert r.order[t] == best
        assert np.isclose(r.loss[t], best_cost - prev, rtol=1e-7, atol=1e-12)
        taken.append(best)
        prev = best_cost


def test_block_size_one_is_algorithm_1(orc):
    d = 14
    w, H, A = _block_setup(70, d, 1)
    a = orc.block_prune_row(A, w, 1, want_trace=True)
    b = orc.prune_row(A, w, want_trace=True)
    assert np.array_equal(a.order, b.order)
    assert np.allclose(a.loss, b.loss, rtol=1e-12)
    assert np.allclose(a.trace, b.trace, rtol=1e-12, atol=1e-15)


def test_block_step_equals_single_steps_over_its_indices(orc):
    # removing a block at once (eq. (5)) and removing its indices one after another with the
    # single-weight update (eq. (3)) reach the same weights; the single losses add up to the block's
    d, c = 16, 4
    w, H, A = _block_setup(80, d, c)
    r = orc.block_prune_row(A, w, c, k_blocks=2)
    forced = np.concatenate([np.arange(b * c, b * c + c) for b in r.order]).astype(np.int32)
    s = orc.prune_row(A, w, k_steps=2 * c, forced=forced)
    assert np.allclose(s.w, r.w, rtol=1e-9, atol=1e-13)
    assert np.allclose(s.loss.reshape(2, c).sum(axis=1), r.loss, rtol=1e-9)
    # and the reduced inverse agrees on the survivors (Lemma 1 applied in either grouping)
    S = np.flatnonzero(r.live)
    assert np.allclose(r.A[np.ix_(S, S)], s.A[np.ix_(S, S)], rtol=1e-9, atol=1e-14)
    assert np.allclose(r.A[np.ix_(S, S)], np.linalg.inv(H[np.ix_(S, S)]), rtol=1e-7)


def test_block_rows_driver_and_argument_checks(orc):
    d, c = 12, 4
    W, X = _problem(90, d, R=5)
    A = np.linalg.inv(2.0 * X @ X.T + 0.1 * np.eye(d))
    res = orc.block_prune_rows(A, W, c, k_blocks=2, n_threads=2)
    for i in range(5):
        r = orc.block_prune_row(A, W[i], c, k_blocks=2)
        assert np.array_equal(res["order"][i], r.order)
        assert np.array_equal(res["W"][i], r.w)
        assert np.array_equal(res["loss"][i], r.loss)
    with pytest.raises(Exception):
        orc.block_prune_row(A, W[0], 5)          # d not a multiple of c
    with pytest.raises(Exception):
        orc.block_prune_row(A, W[0], 4, k_blocks=4)


# ----------------------------------------------------------------------------- layer objective
def test_layer_error_is_the_sum_of_squared_output_differences(orc):
    """Sec. 3 eq. (2): ||W X - W^ X||^2, spelled out per output row and per sample."""
    rng = np.random.default_rng(70)
    R, d, n = 3, 5, 7
    W = rng.standard_normal((R, d))
    Wh = W + 0.3 * rng.standard_normal((R, d))
    X = rng.standard_normal((d, n))
    total = 0.0
    for i in range(R):
        for s in range(n):
            y = sum(W[i, j] * X[j, s] for j in range(d))
            yh = sum(Wh[i, j] * X[j, s] for j in range(d))
            total += (y - yh) ** 2
    assert np.isclose(orc.layer_error(W, Wh, X), total, rtol=1e-12)
    # hand value: W - W^ = [[1, -2]], X = [[1, 2], [3, 4]]: outputs differ by (-5, -6): 25 + 36
    assert orc.layer_error(np.array([[2.0, 0.0]]), np.array([[1.0, 2.0]]), np.array([[1.0, 2.0], [3.0, 4.0]])) == 61.0
    # one row's share and the whole layer's are not the same thing (sum over rows), nor is it a norm
    # without the square
    assert orc.layer_error(W, Wh, X) > orc.layer_error(W[:1], Wh[:1], X)
    assert np.isclose(orc.layer_error(W, W + 2.0 * (Wh - W), X), 4.0 * total, rtol=1e-12)
    assert orc.layer_error(W, W, X) == 0.0


def test_layer_error_equals_accumulated_loss_changes_without_dampening(orc):
    """With lambda = 0 the recorded loss changes w_p^2 / (2 [H^-1]_pp) of Sec. 4 add up, over all
    steps of all rows, to the layer objective of eq. (2) evaluated from X."""
    W, X = _problem(71, 12, n=60, R=4)
    H = orc.hessian(X, damp_rel=-1)
    A = orc.invert(H)
    res = orc.prune_rows(A, W, k_steps=7)
    assert np.isclose(orc.layer_error(W, res["W"], X), res["loss"].sum(), rtol=1e-8)
    grids = [orc.minmax_grid(W[i], 3) for i in range(W.shape[0])]
    q = orc.quant_rows(A, W, [g[0] for g in grids], [g[1] for g in grids], grids[0][2])
    assert np.isclose(orc.layer_error(W, q["W"], X), q["loss"].sum(), rtol=1e-8)


# ----------------------------------------------------------------------------- group-OBS recovery
def test_closed_form_recovery_is_least_squares_on_the_support_and_the_replayed_state(orc):
    """Sec. 4 Step 2: the weights for a mask follow from the group-OBS formula at once.  Pinned by
    the least-squares problem on the kept support solved on H itself (never touching H^-1), by the
    state Algorithm 1 reaches after pruning the same weights one by one, and by a two-weight case
    worked out by hand."""
    W, X = _problem(81, 20, n=90, R=3)
    H = orc.hessian(X)
    A = orc.invert(H)
    res = orc.prune_rows(A, W, k_steps=20)
    counts = np.array([0, 7, 20], np.int32)
    mask = orc.mask_from_counts(res["order"], counts, 20)
    got = orc.reconstruct_closed_form(A, W, mask)
    assert np.array_equal(got[0], W[0])                       # nothing pruned: untouched
    for i in range(3):
        P = np.flatnonzero(mask[i])
        ref = _ls_on_support(H, W[i], P, np.zeros(len(P)))
        assert np.allclose(got[i], ref, rtol=1e-7, atol=1e-10)
        assert np.all(got[i][P] == 0.0)
    assert np.allclose(got, orc.reconstruct(A, W, counts), rtol=1e-7, atol=1e-10)
    # a mask that no greedy run produced is handled alike
    rng = np.random.default_rng(82)
    m2 = (rng.random((3, 20)) < 0.4).astype(np.uint8)
    got = orc.reconstruct_closed_form(A, W, m2)
    for i in range(3):
        P = np.flatnonzero(m2[i])
        assert np.allclose(got[i], _ls_on_support(H, W[i], P, np.zeros(len(P))), rtol=1e-7, atol=1e-10)
    # by hand: H^-1 = [[2, 1], [1, 1]], w = (3, 5), prune index 0: w1 - (1/2) * 3 = 3.5
    out = orc.reconstruct_closed_form(np.array([[2.0, 1.0], [1.0, 1.0]]), np.array([[3.0, 5.0]]), np.array([[1, 0]]))
    assert np.array_equal(out, np.array([[0.0, 3.5]]))
