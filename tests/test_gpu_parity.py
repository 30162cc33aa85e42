"""GPU parity: every entry point of libobc.so, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Tolerances are stated in tests/parity.py."""
import numpy as np
import pytest
import torch

import obc_inputs
from tests.parity import RowParity, check_block_row, check_row

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def obc():
    import paper_2208_11580_amd as pkg

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ctx = pkg.Context()
    yield ctx
    ctx.close()


def _np(t):
    return t.detach().cpu().numpy()


def _layer(name, **kw):
    W, X, spec = obc_inputs.make_layer(name, device="cuda", **kw)
    return W, X


def _hinv(obc, X, damp=0.01):
    H = obc.obc_hessian(X, damp_rel=damp)
    obc.obc_invert(H)
    return H


# ------------------------------------------------------------------------------ Hessian
@pytest.mark.parametrize("d,N,pad", [(32, 256, 0), (200, 3001, 3), (131, 777, 0), (576, 20000, 0)])
def test_hessian_matches_oracle(obc, orc, d, N, pad):
    torch.manual_seed(d)
    Xfull = torch.randn(d, N + pad, device="cuda")
    X = Xfull[:, :N]
    H = obc.obc_hessian(X, damp_rel=0.01)
    Href = orc.hessian(_np(X))
    Hg = _np(H).astype(np.float64)
    assert np.array_equal(Hg, Hg.T)
    rel = np.linalg.norm(Hg - Href) / np.linalg.norm(Href)
    assert rel < 2e-6, rel
    assert np.allclose(Hg, Href, rtol=0, atol=3e-6 * np.abs(Href).max())
    # undamped, then accumulated in two batches
    H0 = obc.obc_hessian(X, damp_rel=-1.0)
    h = N // 2
    Hacc = obc.obc_hessian(Xfull[:, :h], damp_rel=-1.0)
    Hacc = obc.obc_hessian(Xfull[:, h:N], damp_rel=-1.0, H=Hacc, accumulate=True)
    ref0 = orc.hessian(_np(X), damp_rel=-1)
    assert np.linalg.norm(_np(H0) - ref0) / np.linalg.norm(ref0) < 2e-6
    assert np.linalg.norm(_np(Hacc) - ref0) / np.linalg.norm(ref0) < 2e-6


def test_hessian_on_correlated_relu_inputs(obc, orc):
    W, X = _layer("conv64x576", n_samples=10000)
    H = obc.obc_hessian(X)
    Href = orc.hessian(_np(X))
    assert np.linalg.norm(_np(H) - Href) / np.linalg.norm(Href) < 2e-6


# ------------------------------------------------------------------------------ inverse
@pytest.mark.parametrize("d", [1, 32, 100, 257, 576])
def test_invert_matches_oracle(obc, orc, d):
    W, X = _layer("conv64x576", d_col=d, d_row=2, n_samples=4 * d + 50)
    H = obc.obc_hessian(X)
    H64 = _np(H).astype(np.float64)
    A = _np(obc.obc_invert(H.clone())).astype(np.float64)
    assert np.array_equal(A, A.T)
    Aref = orc.invert(H64)
    assert np.linalg.norm(A - Aref) / np.linalg.norm(Aref) < 3e-7
    assert np.linalg.norm(A @ H64 - np.eye(d)) / np.sqrt(d) < 1e-4


def test_invert_reports_non_spd(obc):
    import paper_2208_11580_amd as pkg

    H = torch.eye(70, device="cuda")
    H[65, 65] = -1.0
    with pytest.raises(pkg.ObcError) as e:
        obc.obc_invert(H)
    assert e.value.code == pkg.OBC_ERR_NOT_SPD
    obc.obc_check()  # latch is cleared


# ------------------------------------------------------------------------------ sequential re-fit
@pytest.mark.parametrize("d_col,d_row,N,pad", [(32, 16, 256, 0), (200, 77, 3001, 3), (131, 300, 777, 1),
                                               (576, 64, 20000, 0)])
def test_cross_matches_oracle(obc, orc, d_col, d_row, N, pad):
    torch.manual_seed(d_col + d_row)
    Xf = torch.randn(d_col, N + pad, device="cuda")
    Yf = torch.randn(d_row, N + 2 * pad, device="cuda") + 0.3 * Xf[:1, :N].mean()
    X, Y = Xf[:, :N], Yf[:, :N]
    C = obc.obc_cross(X, Y)
    ref = orc.cross(_np(X), _np(Y))
    assert C.shape == (d_row, d_col)
    assert np.linalg.norm(_np(C) - ref) / np.linalg.norm(ref) < 2e-6
    assert np.allclose(_np(C), ref, rtol=0, atol=3e-6 * np.abs(ref).max())
    # accumulated in two batches
    h = N // 2
    Cacc = obc.obc_cross(Xf[:, :h], Yf[:, :h])
    Cacc = obc.obc_cross(Xf[:, h:N], Yf[:, h:N], C=Cacc, accumulate=True)
    assert np.linalg.norm(_np(Cacc) - ref) / np.linalg.norm(ref) < 2e-6


@pytest.mark.parametrize("d_col,d_row", [(32, 16), (203, 70), (576, 64), (257, 1)])
def test_refit_matches_oracle(obc, orc, d_col, d_row):
    # appendix "Sequential Quantization with OBQ": inputs of the compressed model (here the dense
    # inputs plus a perturbation), outputs of the dense layer
    W, X = _layer("conv64x576", d_col=d_col, d_row=d_row, n_samples=4 * d_col + 50)
    torch.manual_seed(3)
    Xc = (X + 0.1 * X.std() * torch.randn_like(X)).contiguous()
    Y = (W.double() @ X.double()).float()
    H = obc.obc_hessian(Xc)
    C = obc.obc_cross(Xc, Y)
    H0 = H.clone()
    Wr = obc.obc_refit(H, C)
    assert torch.equal(H, H0)                     # H is left alone
    ref = orc.refit(_np(H).astype(np.float64), _np(C).astype(np.float64))
    err = np.linalg.norm(_np(Wr) - ref) / np.linalg.norm(ref)
    assert err < 1e-6, err
    # sharing the factorisation: same weights, and H becomes what obc_invert gives
    Wr2 = obc.obc_refit(H, C, invert_in_place=True)
    assert torch.equal(Wr, Wr2)
    assert torch.equal(H, obc.obc_invert(H0.clone()))
    # the re-fitted weights have (up to the fp32 rounding of H, C and W) zero gradient under the
    # new inputs, the gradient being written out from the data in fp64
    Wn, Xn, Yn = _np(Wr).astype(np.float64), _np(Xc).astype(np.float64), _np(Y).astype(np.float64)
    lam = 0.01 * np.mean(2.0 * np.sum(Xn * Xn, axis=1))
    grad = 2.0 * (Wn @ Xn - Yn) @ Xn.T + lam * Wn
    scale = np.linalg.norm(2.0 * Yn @ Xn.T)
    assert np.linalg.norm(grad) < 5e-4 * scale


def test_sequential_obq_flow(obc, orc):
    # re-fit, then OBQ on the re-fitted weights with the same Hessian, as the appendix describes;
    # each stage is compared with the oracle fed the GPU's previous stage
    W, X = _layer("conv64x576", d_col=260, d_row=6, n_samples=3000)
    torch.manual_seed(4)
    Xc = (X + 0.2 * X.std() * torch.randn_like(X)).contiguous()
    Y = (W.double() @ X.double()).float()
    H = obc.obc_hessian(Xc)
    C = obc.obc_cross(Xc, Y)
    Wr = obc.obc_refit(H, C, invert_in_place=True)      # H now holds the inverse
    _check_quant(obc, orc, Wr, H, 3, 0)


# ------------------------------------------------------------------------------ pruning rows
def _check_prune(obc, orc, W, Hinv, k_steps, nm, strategy, rows=None, want_trace=False):
    res = obc.obc_prune_rows(W, Hinv, k_steps=k_steps, nm=nm, strategy=strategy, want_trace=want_trace)
    obc.obc_check()
    A = _np(Hinv)
    Wn = _np(W)
    st = RowParity()
    order, loss, Wo = _np(res["order"]), _np(res["loss"]), _np(res["W"])
    tr = _np(res["trace"]) if want_trace else None
    for i in (range(W.shape[0]) if rows is None else rows):
        check_row(orc, st, "prune", A, Wn[i], order[i], loss[i], Wo[i], order.shape[1], nm=nm,
                  g_trace=None if tr is None else tr[i])
    print(st)
    st.assert_order_rule()
    return res, st


@pytest.mark.parametrize("strategy", [1, 2])
def test_prune_rows_tiny_layer_full_trace(obc, orc, strategy):
    W, X = _layer("lin16x32")
    Hinv = _hinv(obc, X)
    _check_prune(obc, orc, W, Hinv, 32, (0, 0), strategy, want_trace=True)


@pytest.mark.parametrize("strategy", [1, 2])
@pytest.mark.parametrize("d,R,k", [(203, 5, 203), (320, 6, 320), (576, 4, 576), (1100, 3, 300)])
def test_prune_rows_streamed_sizes(obc, orc, strategy, d, R, k):
    W, X = _layer("conv64x576", d_col=d, d_row=R, n_samples=3 * d)
    Hinv = _hinv(obc, X)
    _check_prune(obc, orc, W, Hinv, k, (0, 0), strategy, want_trace=(d <= 320))


@pytest.mark.parametrize("strategy", [1, 2])
@pytest.mark.parametrize("nm", [(2, 4), (4, 8)])
def test_prune_rows_n_m(obc, orc, strategy, nm):
    d = 264
    W, X = _layer("conv64x576", d_col=d, d_row=4, n_samples=2000)
    Hinv = _hinv(obc, X)
    k = d // nm[1] * (nm[1] - nm[0])
    res, _ = _check_prune(obc, orc, W, Hinv, k, nm, strategy)
    zeros = (_np(res["W"]) == 0).reshape(4, -1, nm[1]).sum(axis=2)
    assert np.all(zeros == nm[1] - nm[0])


@pytest.mark.parametrize("strategy", [1, 2])
def test_prune_rows_zero_weights_and_ties(obc, orc, strategy):
    d = 96
    W, X = _layer("conv64x576", d_col=d, d_row=3, n_samples=1000)
    W[0, 5] = 0.0
    W[0, 50] = 0.0
    W[1, :] = 0.0
    Hinv = _hinv(obc, X)
    res, _ = _check_prune(obc, orc, W, Hinv, d, (0, 0), strategy)
    assert _np(res["order"])[0, :2].tolist() == [5, 50]
    assert _np(res["order"])[1].tolist() == list(range(d))  # all scores equal: index order


@pytest.mark.parametrize("strategy", [1, 2])
def test_prune_rows_is_deterministic(obc, strategy):
    W, X = _layer("conv64x576", d_col=300, d_row=8, n_samples=2000)
    Hinv = _hinv(obc, X)
    a = obc.obc_prune_rows(W, Hinv, strategy=strategy)
    b = obc.obc_prune_rows(W, Hinv, strategy=strategy)
    torch.cuda.synchronize()
    for key in ("order", "loss", "W"):
        assert torch.equal(a[key], b[key])


def test_strategies_agree_on_order(obc):
    W, X = _layer("conv64x576", d_col=448, d_row=6, n_samples=3000)
    Hinv = _hinv(obc, X)
    a = obc.obc_prune_rows(W, Hinv, strategy=1)
    b = obc.obc_prune_rows(W, Hinv, strategy=2)
    assert (a["order"] != b["order"]).float().mean().item() < 0.01
    assert torch.allclose(a["loss"], b["loss"], rtol=1e-3, atol=1e-9)


# ------------------------------------------------------------------------------ block pruning
def _check_blocks(obc, orc, W, Hinv, c, k_blocks, strategy, want_trace=False):
    res = obc.obc_prune_blocks(W, Hinv, c, k_blocks=k_blocks, want_trace=want_trace, strategy=strategy)
    obc.obc_check()
    A, Wn = _np(Hinv), _np(W)
    order, loss, Wo = _np(res["order"]), _np(res["loss"]), _np(res["W"])
    swaps = 0
    for i in range(W.shape[0]):
        swaps += check_block_row(orc, A, Wn[i], c, order[i], loss[i], Wo[i], k_blocks,
                                 g_trace=_np(res["trace"])[i] if want_trace else None)
    return res, swaps


@pytest.mark.parametrize("strategy,d,R,c,kb", [
    (1, 32, 16, 4, 8), (1, 32, 16, 2, 16), (1, 200, 4, 8, 20), (1, 576, 4, 4, 100), (1, 260, 3, 4, 65),
    (1, 126, 3, 3, 42),
    (2, 32, 16, 4, 8), (2, 200, 4, 4, 50), (2, 576, 4, 4, 100), (2, 260, 3, 4, 65), (2, 576, 3, 4, 144),
    (2, 768, 2, 4, 192)])
def test_prune_blocks_matches_oracle(obc, orc, strategy, d, R, c, kb):
    name = "lin16x32" if d == 32 else ("attn768x768" if d == 768 else "conv64x576")
    W, X = _layer(name, d_col=d, d_row=R, n_samples=max(256, 3 * d))
    Hinv = _hinv(obc, X)
    _check_blocks(obc, orc, W, Hinv, c, kb, strategy, want_trace=(d <= 200))


def test_block_strategies_agree(obc):
    W, X = _layer("conv64x576", d_col=576, d_row=8, n_samples=3000)
    Hinv = _hinv(obc, X)
    a = obc.obc_prune_blocks(W, Hinv, 4, strategy=1)
    b = obc.obc_prune_blocks(W, Hinv, 4, strategy=2)
    obc.obc_check()
    same = (a["order"] == b["order"]).float().mean().item()
    assert same > 0.98, same
    assert torch.allclose(a["loss"].sum(dim=1), b["loss"].sum(dim=1), rtol=1e-4)
    import paper_2208_11580_amd as pkg
    with pytest.raises(pkg.ObcError):
        obc.obc_prune_blocks(W, Hinv, 2, strategy=2)     # the deferred-update solver does blocks of 4


@pytest.mark.parametrize("strategy", [1])
def test_prune_blocks_of_one_is_prune_rows(obc, strategy):
    W, X = _layer("conv64x576", d_col=260, d_row=4, n_samples=2000)
    Hinv = _hinv(obc, X)
    a = obc.obc_prune_rows(W, Hinv, k_steps=100, strategy=strategy)
    b = obc.obc_prune_blocks(W, Hinv, 1, k_blocks=100, strategy=strategy)
    obc.obc_check()
    assert torch.equal(a["order"], b["order"])
    assert torch.allclose(a["loss"], b["loss"], rtol=1e-6, atol=0)
    assert torch.allclose(a["W"], b["W"], rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("d", [128, 320])
def test_block_traces_feed_the_global_step(obc, orc, d):
    # Alg. 2 on the block loss traces, then the weights of the chosen per-row block counts both by
    # replay (stop_counts) and from the stored trace (d = 128: LDS-resident solver, 320: deferred)
    W, X = _layer("conv64x576", d_col=d, d_row=12, n_samples=1000)
    Hinv = _hinv(obc, X)
    c = 4
    full = obc.obc_prune_blocks(W, Hinv, c, want_trace=True)
    k = (12 * (d // 4)) // 2
    counts, block_mask = obc.obc_global_select(full["loss"], full["order"], k)
    ref = orc.global_select(_np(full["loss"]).astype(np.float64), k)
    assert np.array_equal(_np(counts), ref)
    assert int(block_mask.sum()) == k
    replay = obc.obc_prune_blocks(W, Hinv, c, stop_counts=counts)
    gathered = obc.obc_gather_trace(W, full["trace"], counts)
    obc.obc_check()
    assert torch.equal(replay["W"], gathered)
    zeros = (gathered == 0).sum(dim=1)
    assert torch.equal(zeros.to(torch.int32), counts * c)


# ------------------------------------------------------------------------------ OBQ rows
def _check_quant(obc, orc, W, Hinv, bits, strategy, live=None, rows=None, grid=None, outliers=False):
    if grid is None:
        delta, offset, maxq = obc.obc_minmax_grid(W, bits, live=live)
    else:
        delta, offset, maxq = grid
    res = obc.obc_quant_rows(W, Hinv, delta, offset, maxq, live=live, strategy=strategy, outliers=outliers)
    obc.obc_check()
    A, Wn = _np(Hinv), _np(W)
    dl, of = _np(delta), _np(offset)
    lv = None if live is None else _np(live)
    st = RowParity()
    order, loss, Wo, codes = _np(res["order"]), _np(res["loss"]), _np(res["W"]), _np(res["codes"])
    for i in (range(W.shape[0]) if rows is None else rows):
        wl = Wn[i] if lv is None else Wn[i][lv[i] != 0]
        if grid is None:
            # the grid the GPU computed is the oracle's min-max grid of the same fp32 weights
            g = orc.minmax_grid(wl.astype(np.float64), bits)
            assert np.float32(g[1]) == of[i] and np.isclose(g[0], dl[i], rtol=1e-6)
        k = len(wl)
        check_row(orc, st, "quant", A, Wn[i], order[i], loss[i], Wo[i], k,
                  grid=(float(dl[i]), float(of[i]), maxq), g_codes=codes[i],
                  live=None if lv is None else lv[i], outlier=outliers)
    print(st)
    st.assert_order_rule()
    return res, st


@pytest.mark.parametrize("strategy", [1, 2])
@pytest.mark.parametrize("d,R,bits", [(32, 16, 4), (203, 4, 3), (576, 4, 4), (768, 3, 2)])
def test_quant_rows_matches_oracle(obc, orc, strategy, d, R, bits):
    name = "lin16x32" if d == 32 else ("attn768x768" if d == 768 else "conv64x576")
    W, X = _layer(name, d_col=d, d_row=R, n_samples=max(256, 3 * d))
    Hinv = _hinv(obc, X)
    _check_quant(obc, orc, W, Hinv, bits, strategy)


@pytest.mark.parametrize("strategy", [1, 2])
@pytest.mark.parametrize("d", [64, 320])
def test_quant_rows_at_rounding_boundaries(obc, orc, strategy, d):
    """Weights exactly on a half step of the grid, and one fp32 ulp to either side: the code written
    is the code the candidate was scored with (round half to even), and both equal the oracle's.
    The inverse Hessian is diagonal, so OBQ is plain rounding and every weight keeps its value
    until it is chosen."""
    delta, offset, maxq = 0.25, -1.0, 7          # the grid -1, -0.75, ..., 0.75; exact in fp32
    base = np.float32(offset) + np.float32(delta) * (np.arange(d, dtype=np.float32) % 7 + np.float32(0.5))
    rows = np.stack([base, np.nextafter(base, np.float32(-4), dtype=np.float32),
                     np.nextafter(base, np.float32(4), dtype=np.float32)]).astype(np.float32)
    rng = np.random.default_rng(5)
    diag = rng.uniform(0.5, 2.0, d).astype(np.float32)
    W = torch.tensor(rows, device="cuda")
    Hinv = torch.diag(torch.tensor(diag, device="cuda")).contiguous()
    dl = torch.full((3,), delta, device="cuda")
    of = torch.full((3,), offset, device="cuda")
    q = obc.obc_quant_rows(W, Hinv, dl, of, maxq, strategy=strategy)
    obc.obc_check()
    codes = _np(q["codes"])
    for i in range(3):
        want = np.array([orc.quant_code(float(rows[i, j]), delta, offset, maxq) for j in range(d)])
        assert np.array_equal(codes[i], want), (i, np.flatnonzero(codes[i] != want)[:5])
        ro = orc.quant_row(np.diag(diag.astype(np.float64)), rows[i].astype(np.float64), (delta, offset, maxq))
        assert np.array_equal(codes[i], ro.codes)
        # the recorded loss is the one of the written code
        step_of = np.empty(d, np.int64)
        step_of[_np(q["order"][i])] = np.arange(d)
        err = (offset + delta * codes[i].astype(np.float64)) - rows[i].astype(np.float64)
        assert np.allclose(_np(q["loss"][i])[step_of], err * err / (2.0 * diag.astype(np.float64)), rtol=1e-5, atol=1e-12)
    # exactly on the half step the even code wins: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, ...
    half = (np.arange(d) % 7) + 0.5
    assert np.array_equal(codes[0], np.minimum(np.round(half), maxq).astype(np.int32))
    deq = (of[:, None].double() + dl[:, None].double() * q["codes"].double()).float()
    assert torch.equal(q["W"], deq)


def _narrow_grid(W, bits, shrink):
    """A min-max grid shrunk about its centre: the weights beyond it start as outliers."""
    maxq = (1 << bits) - 1
    lo, hi = W.min(dim=1).values, W.max(dim=1).values
    mid, half = 0.5 * (lo + hi), 0.5 * (hi - lo) * shrink
    return (2.0 * half / maxq).contiguous(), (mid - half).contiguous(), maxq


@pytest.mark.parametrize("strategy", [1, 2])
@pytest.mark.parametrize("d,R,bits,shrink", [(32, 16, 3, 0.5), (203, 4, 3, 0.6), (576, 4, 4, 0.7), (768, 3, 2, 0.5)])
def test_quant_rows_outlier_heuristic_matches_oracle(obc, orc, strategy, d, R, bits, shrink):
    # Sec. 5, outlier heuristic: on a grid narrower than the weight range several weights start
    # beyond half a step from the grid, and compensation pushes more of them out on the way
    name = "lin16x32" if d == 32 else ("attn768x768" if d == 768 else "conv64x576")
    W, X = _layer(name, d_col=d, d_row=R, n_samples=max(256, 3 * d))
    Hinv = _hinv(obc, X)
    grid = _narrow_grid(W, bits, shrink)
    res, st = _check_quant(obc, orc, W, Hinv, bits, strategy, grid=grid, outliers=True)
    # the heuristic changed the outcome (else the case does not test it)
    plain = obc.obc_quant_rows(W, Hinv, *grid, strategy=strategy)
    assert not torch.equal(plain["order"], res["order"])


@pytest.mark.parametrize("strategy", [1, 2])
def test_outlier_heuristic_is_inactive_on_a_covering_grid(obc, strategy):
    # on the min-max grid no weight starts as an outlier; the flag only matters once compensation
    # has pushed a weight out, so with a very wide grid both runs are bit-identical
    W, X = _layer("conv64x576", d_col=260, d_row=4, n_samples=2000)
    Hinv = _hinv(obc, X)
    delta, offset, maxq = obc.obc_minmax_grid(W, 8)
    wide = (delta * 4, offset - delta * 4 * 384, 1023)
    a = obc.obc_quant_rows(W, Hinv, *wide, strategy=strategy)
    b = obc.obc_quant_rows(W, Hinv, *wide, strategy=strategy, outliers=True)
    for k in ("order", "loss", "codes", "W"):
        assert torch.equal(a[k], b[k])


def test_symmetric_grid_matches_oracle(obc, orc):
    W, _ = _layer("conv64x576", d_col=203, d_row=8, n_samples=256)
    W[3] = 0.0                       # empty range
    live = (torch.rand_like(W) > 0.3).to(torch.uint8)
    live[5] = 0                      # no live weight
    for lv in (None, live):
        delta, offset, maxq = obc.obc_minmax_grid(W, 4, live=lv, symmetric=True)
        Wn = _np(W)
        for i in range(W.shape[0]):
            wl = Wn[i] if lv is None else Wn[i][_np(lv)[i] != 0]
            if wl.size == 0:
                assert delta[i].item() == 1.0 and offset[i].item() == 0.0
                continue
            g = orc.symmetric_grid(wl.astype(np.float64), 4)
            assert np.float32(g[1]) == offset[i].item()
            assert np.isclose(g[0], delta[i].item(), rtol=1e-6)
            assert maxq == g[2]


@pytest.mark.parametrize("strategy", [1, 2])
def test_quant_with_single_point_grid_is_pruning(obc, strategy):
    # quant(.) == 0 turns OBQ into ExactOBS (Sec. 5): bit-identical on the GPU too
    W, X = _layer("conv64x576", d_col=260, d_row=4, n_samples=2000)
    Hinv = _hinv(obc, X)
    p = obc.obc_prune_rows(W, Hinv, strategy=strategy)
    delta = torch.ones(4, device="cuda")
    offset = torch.zeros(4, device="cuda")
    q = obc.obc_quant_rows(W, Hinv, delta, offset, 0, strategy=strategy)
    obc.obc_check()
    assert torch.equal(p["order"], q["order"])
    assert torch.equal(p["loss"], q["loss"])
    assert torch.equal(q["W"], torch.zeros_like(q["W"]))
    assert torch.all(q["codes"] == 0)


@pytest.mark.parametrize("strategy", [1, 2])
def test_quant_rows_on_survivors_of_2_4(obc, orc, strategy):
    d = 256
    W, X = _layer("conv64x576", d_col=d, d_row=4, n_samples=2000)
    Hinv = _hinv(obc, X)
    p = obc.obc_prune_rows(W, Hinv, nm=(2, 4), strategy=strategy)
    live = (p["W"] != 0).to(torch.uint8)
    _check_quant(obc, orc, p["W"], Hinv, 4, strategy, live=live)


# ------------------------------------------------------------------------------ global step
def _check_global(obc, orc, loss, order, k):
    counts, mask = obc.obc_global_select(loss, order, k)
    torch.cuda.synchronize()
    ref = orc.global_select(_np(loss).astype(np.float64), k)
    assert np.array_equal(_np(counts), ref)
    assert np.array_equal(_np(mask), orc.mask_from_counts(_np(order), ref, loss.shape[1]))
    return counts, mask


def test_global_select_matches_algorithm_2(obc, orc):
    W, X = _layer("lin16x32")
    Hinv = _hinv(obc, X)
    res = obc.obc_prune_rows(W, Hinv)
    for k in (0, 1, 100, 256, 511, 512):
        _check_global(obc, orc, res["loss"], res["order"], k)
    W, X = _layer("conv64x576", d_col=300, d_row=37, n_samples=2000)
    Hinv = _hinv(obc, X)
    res = obc.obc_prune_rows(W, Hinv)
    for k in (1, 37 * 300 // 2, int(0.6 * 37 * 300), 37 * 300 - 1):
        _check_global(obc, orc, res["loss"], res["order"], k)


def test_global_select_non_monotone_and_tied_traces(obc, orc):
    rng = np.random.default_rng(0)
    R, d = 1100, 24   # more rows than one scan chunk
    L = rng.integers(0, 6, size=(R, d)).astype(np.float32)   # many exact ties, non-monotone rows
    loss = torch.tensor(L, device="cuda")
    order = torch.stack([torch.randperm(d, device="cuda") for _ in range(R)]).to(torch.int32)
    for k in (1, 5, 1234, R * d // 2, R * d):
        _check_global(obc, orc, loss, order, k)


def test_end_to_end_tiny_layer(obc, orc):
    """configs[0]: 16 x 32, prune to 50 % with the global step; whole path GPU vs whole path oracle."""
    W, X = _layer("lin16x32")
    Hinv = _hinv(obc, X)
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    k = obc_inputs.target_count(0.5, 16, 32)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    What = obc.obc_gather_trace(W, res["trace"], counts)
    replay = obc.obc_prune_rows(W, Hinv, stop_counts=counts)
    obc.obc_check()
    assert torch.equal(replay["W"], What)
    Xn, Wn = _np(X), _np(W)
    Ao = orc.invert(orc.hessian(Xn))
    ro = orc.prune_rows(Ao, Wn.astype(np.float64))
    co = orc.global_select(ro["loss"], k)
    Wo = orc.reconstruct(Ao, Wn.astype(np.float64), co)
    assert np.array_equal(_np(counts), co)
    assert np.array_equal(_np(mask), orc.mask_from_counts(ro["order"], co, 32))
    e_gpu = orc.layer_error(Wn, _np(What), Xn)
    e_orc = orc.layer_error(Wn, Wo, Xn)
    assert abs(e_gpu - e_orc) <= 1e-3 * e_orc
    assert np.linalg.norm(_np(What) - Wo) <= 1e-4 * np.linalg.norm(Wo)


@pytest.mark.parametrize("strategy", [1, 2])
def test_prune_rows_on_an_already_sparse_matrix(obc, orc, strategy):
    """Sec. 4 "Implementation Details": an already sparse matrix is pruned further on the dense
    sub-problem of its non-zeros.  The oracle works on that sub-problem directly (inverse of the
    sub-Hessian); the GPU reaches it by eliminating the zeros from H^-1 first."""
    d, k1, k2 = 260, 100, 60
    W, X = _layer("conv64x576", d_col=d, d_row=4, n_samples=2000)
    Hinv = _hinv(obc, X)
    first = obc.obc_prune_rows(W, Hinv, k_steps=k1, strategy=strategy)
    live = (first["W"] != 0).to(torch.uint8)
    assert int(live.sum()) == 4 * (d - k1)
    second = obc.obc_prune_rows(first["W"], Hinv, k_steps=k2, live=live, strategy=strategy, want_trace=True)
    obc.obc_check()
    A, W1 = _np(Hinv), _np(first["W"])
    st = RowParity()
    for i in range(4):
        check_row(orc, st, "prune", A, W1[i], _np(second["order"][i]), _np(second["loss"][i]),
                  _np(second["W"][i]), k2, live=_np(live[i]), g_trace=_np(second["trace"][i]))
    print(st)
    st.assert_order_rule()
    assert int((second["W"] == 0).sum()) == 4 * (k1 + k2)
    # continuing from the reduced inverse is continuing the same greedy run: the one-pass run over
    # k1 + k2 steps takes (up to near ties) the same weights next
    one = obc.obc_prune_rows(W, Hinv, k_steps=k1 + k2, strategy=strategy)
    same = (one["order"][:, k1:] == second["order"]).float().mean().item()
    assert same > 0.9, same
    assert torch.allclose(one["W"], second["W"], rtol=1e-3, atol=1e-5)
    # a row with fewer survivors than k_steps stops when none is left
    live2 = live.clone()
    live2[1, 5:] = 0
    W2 = first["W"] * live2
    few = obc.obc_prune_rows(W2, Hinv, k_steps=k2, live=live2, strategy=strategy)
    obc.obc_check()
    assert torch.all(few["W"][1] == 0)
    n1 = int(live2[1].sum())
    assert torch.all(few["order"][1, n1:] == -1) and torch.all(few["order"][1, :n1] >= 0)
    # not combined with N:M
    import paper_2208_11580_amd as pkg
    with pytest.raises(pkg.ObcError):
        obc.obc_prune_rows(W[:, :256].contiguous(), Hinv[:256, :256].contiguous(), nm=(2, 4),
                           live=live[:, :256].contiguous(), strategy=strategy)


def test_many_sparsity_levels_from_one_trace(obc, orc):
    """The paper's database of sparsity levels s_i = 1 - (1 - delta)^i (Sec. 6) comes from ONE run of
    the row solver: every level is a global step over the same loss traces and a gather from the
    same weight trace.  Each level is checked against the oracle's replay of its own traces."""
    W, X = _layer("conv64x576", d_col=96, d_row=24, n_samples=800)
    Hinv = _hinv(obc, X)
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    obc.obc_check()
    R, d = W.shape
    A, Wn = _np(Hinv).astype(np.float64), _np(W).astype(np.float64)
    ro = orc.prune_rows(A, Wn)
    assert np.array_equal(ro["order"], _np(res["order"]))       # no near ties in this layer
    levels = [1.0 - 0.9 ** i for i in range(1, 31, 3)]
    prev = -1
    for sp in levels:
        k = obc_inputs.target_count(sp, R, d)
        assert k > prev
        prev = k
        counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
        What = obc.obc_gather_trace(W, res["trace"], counts)
        # Alg. 2 on the GPU's own (fp32) traces: the counts are then an exact integer comparison
        co = orc.global_select(_np(res["loss"]).astype(np.float64), k)
        assert np.array_equal(_np(counts), co), sp
        assert int(mask.sum()) == k and int((What == 0).sum()) >= k
        Wo = orc.reconstruct(A, Wn, co)
        assert np.linalg.norm(_np(What) - Wo) <= 1e-4 * np.linalg.norm(Wo), sp


@pytest.mark.parametrize("strategy", [1, 2])
def test_rows_that_do_no_step_keep_their_weights(obc, strategy):
    W, X = _layer("conv64x576", d_col=280, d_row=5, n_samples=1500)
    Hinv = _hinv(obc, X)
    full = obc.obc_prune_rows(W, Hinv, strategy=strategy, want_trace=True)
    counts = torch.tensor([0, 1, 70, 0, 280], dtype=torch.int32, device="cuda")
    rep = obc.obc_prune_rows(W, Hinv, stop_counts=counts, strategy=strategy)
    obc.obc_check()
    assert torch.equal(rep["W"], obc.obc_gather_trace(W, full["trace"], counts))
    assert torch.equal(rep["W"][0], W[0]) and torch.equal(rep["W"][3], W[3])
    none = obc.obc_prune_rows(W, Hinv, k_steps=0, strategy=strategy)
    assert torch.equal(none["W"], W)


@pytest.mark.parametrize("strategy", [1, 2])
def test_trace_beyond_a_rows_last_step_is_zero(obc, strategy):
    """Trace entries of the steps a row does not take (per-row step limits, fewer survivors than
    steps) are zero in both solvers, whatever the buffer held before."""
    W, X = _layer("conv64x576", d_col=264, d_row=4, n_samples=1500)
    Hinv = _hinv(obc, X)
    k = 100
    counts = torch.tensor([0, 7, 100, 64], dtype=torch.int32, device="cuda")
    out = dict(trace=torch.full((4, k, 264), float("nan"), device="cuda"))
    res = obc.obc_prune_rows(W, Hinv, k_steps=k, stop_counts=counts, strategy=strategy, out=out)
    full = obc.obc_prune_rows(W, Hinv, k_steps=k, strategy=strategy, want_trace=True)
    obc.obc_check()
    for i, c in enumerate(counts.tolist()):
        assert torch.equal(res["trace"][i, :c], full["trace"][i, :c])
        assert torch.all(res["trace"][i, c:] == 0)
    # an already sparse row runs out of survivors before k steps
    live = torch.ones(4, 264, dtype=torch.uint8, device="cuda")
    live[1, 40:] = 0                                           # 40 survivors
    out = dict(trace=torch.full((4, k, 264), float("nan"), device="cuda"))
    sp = obc.obc_prune_rows(W * live, Hinv, k_steps=k, live=live, strategy=strategy, out=out)
    obc.obc_check()
    assert torch.isfinite(sp["trace"]).all()
    assert torch.all(sp["trace"][1, 40:] == 0)
    assert torch.all(sp["trace"][1, 39] == 0) and not torch.all(sp["trace"][1, 38] == 0)


def test_membench_kernels_move_what_they_say(obc):
    """The plain copy kernel copies (both store policies); read and write passes return a time."""
    n = 1 << 22
    src = (torch.arange(n, device="cuda", dtype=torch.int32) * 2).view(torch.uint8)    # low bits clear
    dst = torch.zeros_like(src)
    for streaming in (False, True):
        dst.zero_()
        ms = obc.obc_membench(2, src, dst, src.numel(), reps=2, streaming=streaming)
        assert ms > 0 and torch.equal(dst, src)
    assert obc.obc_membench(0, src, None, src.numel(), reps=2) > 0
    assert obc.obc_membench(1, None, dst, dst.numel(), reps=2, streaming=True) > 0
    import paper_2208_11580_amd as pkg
    with pytest.raises(pkg.ObcError):
        obc.obc_membench(2, src, dst, 24, reps=1)              # not a multiple of 16 bytes


def test_mfmabench_stays_below_the_data_sheet(obc):
    """The loop of independent MFMA instructions runs and reports a rate no matrix core can exceed."""
    f32 = obc.obc_mfmabench(0, iters=2000, reps=2)
    f64 = obc.obc_mfmabench(1, iters=2000, reps=2)
    print("fp32 MFMA %.1f TFLOP/s, fp64 MFMA %.1f TFLOP/s" % (f32, f64))
    assert 10.0 < f32 < 157.3 * 1.05
    assert 5.0 < f64 < 78.6 * 1.05
    import paper_2208_11580_amd as pkg
    with pytest.raises(pkg.ObcError):
        obc.obc_mfmabench(2)


def test_trace_of_an_odd_width_is_fully_written(obc, orc):
    # the trace is cleared by a 16-byte-wide fill before the steps scatter into it: a size that is
    # no multiple of four floats, over memory that held NaNs before
    W, X = _layer("conv64x576", d_col=301, d_row=3, n_samples=1500)
    Hinv = _hinv(obc, X)
    poison = torch.full((3 * 301 * 301 + 64,), float("nan"), device="cuda")
    del poison
    res = obc.obc_prune_rows(W, Hinv, strategy=2, want_trace=True)
    obc.obc_check()
    tr = _np(res["trace"])
    assert np.isfinite(tr).all()
    order = _np(res["order"])
    for i in range(3):
        r = orc.prune_row(_np(Hinv).astype(np.float64), _np(W[i]).astype(np.float64), forced=order[i].astype(np.int32),
                          want_trace=True)
        for t in (0, 1, 150, 299, 300):
            assert np.all(tr[i, t, order[i, :t + 1]] == 0.0)
            assert np.linalg.norm(tr[i, t] - r.trace[t]) <= 1e-4 * np.linalg.norm(r.trace[t]) + 1e-30


# ------------------------------------------------------------------------------ closed-form recovery
@pytest.mark.parametrize("d,R,sparsity", [(32, 16, 0.5), (203, 5, 0.4), (576, 4, 0.6), (1100, 3, 0.5)])
def test_reconstruct_rows_matches_oracle_and_the_trace(obc, orc, d, R, sparsity):
    """Sec. 4 Step 2: the weights of the global step's mask by the group-OBS closed form, against the
    oracle's closed form (same fp32 inputs) and against the weights gathered from the pruning trace."""
    name = "lin16x32" if d == 32 else "conv64x576"
    W, X = _layer(name, d_col=d, d_row=R, n_samples=max(256, 3 * d))
    Hinv = _hinv(obc, X)
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    k = obc_inputs.target_count(sparsity, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    from_trace = obc.obc_gather_trace(W, res["trace"], counts)
    got = obc.obc_reconstruct_rows(W, Hinv, mask, max_pruned=int(counts.max()))
    obc.obc_check()
    ref = orc.reconstruct_closed_form(_np(Hinv), _np(W), _np(mask))
    g = _np(got).astype(np.float64)
    for i in range(R):
        assert np.linalg.norm(g[i] - ref[i]) <= 1e-6 * np.linalg.norm(ref[i]) + 1e-30, i
        assert np.linalg.norm(g[i] - _np(from_trace[i])) <= 1e-4 * np.linalg.norm(ref[i]) + 1e-30, i
    assert torch.equal(got == 0, mask.bool())
    # the default workspace bound (any count up to d) gives the same weights
    assert torch.equal(obc.obc_reconstruct_rows(W, Hinv, mask), got)


def test_reconstruct_rows_edge_cases(obc, orc):
    import paper_2208_11580_amd as pkg

    d, R = 200, 6
    W, X = _layer("conv64x576", d_col=d, d_row=R, n_samples=900)
    Hinv = _hinv(obc, X)
    g = torch.Generator(device="cuda")
    g.manual_seed(4)
    mask = (torch.rand(R, d, generator=g, device="cuda") < 0.45).to(torch.uint8)
    mask[0] = 0                                    # nothing pruned
    mask[1] = 1                                    # everything pruned
    mask[2] = 0
    mask[2, 77] = 1                                # a single weight
    mask[3, :65] = 1                               # one more than a block of 64 among others
    got = obc.obc_reconstruct_rows(W, Hinv, mask)
    obc.obc_check()
    ref = orc.reconstruct_closed_form(_np(Hinv), _np(W), _np(mask))
    assert torch.equal(got[0], W[0]) and int(got[1].abs().sum()) == 0
    assert np.linalg.norm(_np(got) - ref) <= 1e-6 * np.linalg.norm(ref)
    assert torch.equal(got == 0, mask.bool())
    # the single-weight row is the OBS update of eq. (3): w - H^-1[:, p] w_p / [H^-1]_pp
    A = _np(Hinv).astype(np.float64)
    w2 = _np(W[2]).astype(np.float64)
    one = w2 - A[:, 77] * w2[77] / A[77, 77]
    one[77] = 0.0
    assert np.allclose(_np(got[2]), one, rtol=1e-6, atol=1e-9)
    # a workspace bound below a row's count: that row comes back unchanged and the call is flagged
    small = obc.obc_reconstruct_rows(W, Hinv, mask, max_pruned=70)
    with pytest.raises(pkg.ObcError) as e:
        obc.obc_check()
    assert e.value.code == pkg.OBC_ERR_WORKSPACE
    many = mask.sum(dim=1) > 70
    assert bool(many.any()) and torch.equal(small[many], W[many])
    assert torch.equal(small[~many], got[~many])
    # argument errors
    with pytest.raises(pkg.ObcError):
        obc.obc_reconstruct_rows(W, Hinv, mask, max_pruned=d + 1)


# ------------------------------------------------------------------------------ boundary errors
def test_argument_errors(obc):
    import paper_2208_11580_amd as pkg

    W = torch.randn(4, 30, device="cuda")
    Hinv = torch.eye(30, device="cuda")
    with pytest.raises(pkg.ObcError) as e:
        obc.obc_prune_rows(W, Hinv, k_steps=31)
    assert e.value.code == pkg.OBC_ERR_BAD_SHAPE
    with pytest.raises(pkg.ObcError) as e:
        obc.obc_prune_rows(W, Hinv, nm=(2, 4), k_steps=10)   # 30 % 4 != 0
    assert e.value.code == pkg.OBC_ERR_BAD_SHAPE
    with pytest.raises(pkg.ObcError) as e:
        obc.obc_global_select(torch.zeros(4, 30, device="cuda"), torch.zeros(4, 30, dtype=torch.int32, device="cuda"), 121)
    assert e.value.code == pkg.OBC_ERR_BAD_SHAPE
    # a non-positive pivot is latched by the kernel and reported by obc_check
    bad = torch.eye(30, device="cuda")
    bad[3, 3] = -1.0
    obc.obc_prune_rows(W, bad)
    with pytest.raises(pkg.ObcError) as e:
        obc.obc_check()
    assert e.value.code == pkg.OBC_ERR_NUMERIC
    obc.obc_check()
    # empty inputs are fine
    out = obc.obc_prune_rows(W[:0], Hinv)
    assert out["order"].shape == (0, 30)


def test_rows_many_more_rows_than_cus(obc, orc):
    """Several times more rows than CUs at a mid-size width: the solver switches to the panel variant
    of which three workgroups share a CU; sampled rows against the oracle, all rows against invariants."""
    R, d = 1030, 420
    W, X = _layer("attn768x768", d_col=d, d_row=R, n_samples=2000)
    Hinv = _hinv(obc, X)
    rows = [0, 515, 1029]
    res, _ = _check_prune(obc, orc, W, Hinv, d, (0, 0), 2, rows=rows)
    srt = torch.sort(res["order"], dim=1).values
    assert torch.equal(srt, torch.arange(d, device="cuda", dtype=torch.int32).expand(R, d))
    assert torch.all(res["W"] == 0)
    _check_quant(obc, orc, W, Hinv, 4, 2, rows=rows)
    # block pruning through the same shared-CU variant
    kb = d // 4
    blk = obc.obc_prune_blocks(W, Hinv, 4, strategy=2)
    obc.obc_check()
    A, Wn = _np(Hinv), _np(W)
    for i in rows:
        check_block_row(orc, A, Wn[i], 4, _np(blk["order"][i]), _np(blk["loss"][i]), _np(blk["W"][i]), kb)
    srt = torch.sort(blk["order"], dim=1).values
    assert torch.equal(srt, torch.arange(kb, device="cuda", dtype=torch.int32).expand(R, kb))
    assert torch.all(blk["W"] == 0)


def test_edge_cases_of_the_widened_entry_points(obc, orc):
    """Smallest shapes and degenerate masks: one sample, one column, one block, rows whose weights are
    all pruned already, every row with enough pruned weights for the bulk elimination."""
    ctx = obc
    torch.manual_seed(0)
    for N in (1, 3, 17):
        X = torch.randn(5, N, device="cuda")
        Y = torch.randn(3, N, device="cuda")
        C = ctx.obc_cross(X, Y)
        assert np.allclose(_np(C), orc.cross(_np(X), _np(Y)), rtol=1e-5, atol=1e-6), N
    X = torch.randn(1, 50, device="cuda")
    Y = torch.randn(2, 50, device="cuda")
    H = ctx.obc_hessian(X)
    C = ctx.obc_cross(X, Y)
    assert np.allclose(_np(ctx.obc_refit(H, C)), orc.refit(_np(H), _np(C)), rtol=1e-5)
    # a row that is one block
    X = torch.randn(4, 64, device="cuda")
    W = torch.randn(3, 4, device="cuda")
    Hinv = _hinv(ctx, X)
    for st in (0, 1, 2):
        r = ctx.obc_prune_blocks(W, Hinv, 4, strategy=st)
        ctx.obc_check()
        assert torch.all(r["W"] == 0) and torch.all(r["order"] == 0)
        ro = orc.block_prune_row(_np(Hinv).astype(np.float64), _np(W[0]).astype(np.float64), 4)
        assert abs(r["loss"][0, 0].item() - ro.loss[0]) <= 1e-4 * ro.loss[0]
    # live masks on both solvers
    d = 260
    X = torch.randn(d, 1000, device="cuda")
    W = torch.randn(3, d, device="cuda") * 0.1
    Hinv = _hinv(ctx, X)
    for st in (1, 2):
        live = torch.ones(3, d, dtype=torch.uint8, device="cuda")
        live[1] = 0                                  # a row with nothing left
        Wl = W * live
        delta, offset, maxq = ctx.obc_minmax_grid(Wl, 4, live=live)
        q = ctx.obc_quant_rows(Wl, Hinv, delta, offset, maxq, live=live, strategy=st)
        ctx.obc_check()
        assert torch.all(q["W"][1] == 0) and torch.all(q["codes"][1] == -1)
        q0 = ctx.obc_quant_rows(W, Hinv, *ctx.obc_minmax_grid(W, 4)[:2], 15, strategy=st)
        assert torch.equal(q["W"][0], q0["W"][0]) and torch.equal(q["order"][2], q0["order"][2])
        p = ctx.obc_prune_rows(Wl, Hinv, k_steps=10, live=live, strategy=st)
        ctx.obc_check()
        assert torch.all(p["W"][1] == 0) and torch.all(p["order"][1] == -1)
        # every row has at least 64 pruned weights (bulk elimination), one row has no survivor
        live2 = torch.ones(3, d, dtype=torch.uint8, device="cuda")
        live2[:, :130] = 0
        live2[2, :] = 0
        W2 = W * live2
        p2 = ctx.obc_prune_rows(W2, Hinv, k_steps=20, live=live2, strategy=st)
        ctx.obc_check()
        Hfull = np.linalg.inv(_np(Hinv).astype(np.float64))
        ref = orc.prune_row(orc.invert(Hfull[130:, 130:]), _np(W2[0, 130:]).astype(np.float64), k_steps=20)
        assert np.array_equal(_np(p2["order"][0]) - 130, ref.order)
        assert np.allclose(_np(p2["W"][0, 130:]), ref.w, rtol=1e-3, atol=1e-6)
        assert torch.all(p2["W"][2] == 0)
    # the outlier flag with a single-point grid: everything is an outlier until it sits at zero
    a = ctx.obc_quant_rows(W, Hinv, torch.ones(3, device="cuda"), torch.zeros(3, device="cuda"), 0, outliers=True)
    ctx.obc_check()
    assert torch.all(a["W"] == 0)
