"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the whole layer
runs on the GPU, the oracle checks sampled rows one by one (tests/parity.py protocol)."""
import numpy as np
import pytest
import torch

import obc_inputs
from tests.parity import RowParity, check_block_row, check_row, check_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def obc():
    import paper_2208_11580_amd as pkg

    ctx = pkg.Context()
    yield ctx
    ctx.close()


def _np(t):
    return t.detach().cpu().numpy()


def test_conv256x2304_obq4_sampled_rows(obc, orc):
    W, X, _ = obc_inputs.make_layer("conv256x2304", device="cuda")
    R, d = W.shape
    H = obc.obc_hessian(X)
    Hd = _np(H).astype(np.float64)
    Hinv = obc.obc_invert(H)
    A = _np(Hinv)
    # inverse quality at full size (conditioning, not entry-wise agreement, is what can be checked)
    resid = np.linalg.norm(A.astype(np.float64) @ Hd - np.eye(d)) / np.sqrt(d)
    assert resid < 1e-3, resid
    delta, offset, maxq = obc.obc_minmax_grid(W, 4)
    res = obc.obc_quant_rows(W, Hinv, delta, offset, maxq)
    obc.obc_check()
    st = RowParity()
    rows = list(range(0, 256, 8))              # 32 rows, two rounds of the oracle's 16 threads
    order, loss, Wo, codes = (_np(res[k][rows]) for k in ("order", "loss", "W", "codes"))
    check_rows(orc, st, "quant", A, _np(W[rows]), order, loss, Wo, d,
               grids=(_np(delta[rows]), _np(offset[rows]), maxq), g_codes=codes)
    print(st)
    st.assert_order_rule()
    assert st.rows == len(rows)
    # properties that hold for every row at any size
    c = res["codes"]
    assert int(c.min()) >= 0 and int(c.max()) <= maxq
    srt = torch.sort(res["order"], dim=1).values
    assert torch.equal(srt, torch.arange(d, device="cuda", dtype=torch.int32).expand(R, d))
    assert torch.all(res["loss"] >= 0)
    deq = (offset[:, None].double() + delta[:, None].double() * c.double()).float()
    assert torch.equal(res["W"], deq)
    # OBQ must beat plain rounding on the layer objective 1/2 (w-w^)^T H (w-w^) for every row
    rtn = offset[:, None] + delta[:, None] * torch.clamp(torch.round((W - offset[:, None]) / delta[:, None]), 0, maxq)
    Hm = torch.tensor(Hd, device="cuda")
    q_obq = (((W - res["W"]).double() @ Hm) * (W - res["W"]).double()).sum(dim=1)
    q_rtn = (((W - rtn).double() @ Hm) * (W - rtn).double()).sum(dim=1)
    assert torch.all(q_obq < q_rtn)
    # the loss trace sums to that quadratic form (loss identity) on every row
    dev = float(((res["loss"].double().sum(dim=1) - 0.5 * q_obq).abs() / (0.5 * q_obq)).max())
    print("loss identity, largest relative deviation over the rows: %.2e" % dev)
    assert dev < 1e-5


def test_ffn768x3072_prune_sampled_row(obc, orc):
    """The second target layer (d_col = 3072): whole layer on the GPU with the HBM trace, global
    step to 50 %, weights gathered from the trace; the oracle replays one sampled row."""
    W, X, _ = obc_inputs.make_layer("ffn768x3072", device="cuda")
    R, d = W.shape
    H = obc.obc_hessian(X)
    Hinv = obc.obc_invert(H)
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    obc.obc_check()
    k = obc_inputs.target_count(0.5, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    What = obc.obc_gather_trace(W, res["trace"], counts)
    torch.cuda.synchronize()
    assert int(counts.sum()) == k and int(mask.sum()) == k
    # the mask is exactly the zero pattern of the gathered weights
    assert torch.equal(What == 0, mask.bool())
    # every row's order is a permutation; cumulative loss is non-decreasing
    srt = torch.sort(res["order"], dim=1).values
    assert torch.equal(srt, torch.arange(d, device="cuda", dtype=torch.int32).expand(R, d))
    assert torch.all(res["loss"] >= 0)
    # Algorithm 2 property: every pruned weight's key (prefix max of its row's losses) is <= every
    # kept weight's key
    keys = torch.cummax(res["loss"], dim=1).values
    idx = torch.arange(d, device="cuda").expand(R, d)
    pruned = idx < counts[:, None]
    assert keys[pruned].max() <= keys[~pruned].min()
    # sampled rows against the oracle; for two of them also the state at the count the global step chose
    rows = [0, 51, 77, 102, 153, 204, 255, 306, 357, 408, 459, 510, 561, 612, 700, 767]
    st = RowParity()
    A = _np(Hinv)
    check_rows(orc, st, "prune", A, _np(W[rows]), _np(res["order"][rows]), _np(res["loss"][rows]),
               _np(res["W"][rows]), d)
    print(st)
    st.assert_order_rule()
    assert st.rows == len(rows)
    for i in (77, 612):
        c = int(counts[i])
        ref = orc.prune_row(A.astype(np.float64), _np(W[i]).astype(np.float64), k_steps=c,
                            forced=_np(res["order"][i]).astype(np.int32)).w
        got = _np(What[i]).astype(np.float64)
        assert np.linalg.norm(got - ref) <= 1e-4 * np.linalg.norm(ref)


def test_conv64x576_end_to_end_layer_error(obc, orc):
    """configs[1] at full size: Hessian, inverse, pruning traces, global step to 60 %, and 2:4, all
    on the GPU; the oracle runs its own whole path from X in fp64.  Graded on the layer error."""
    W, X, _ = obc_inputs.make_layer("conv64x576", device="cuda")
    R, d = W.shape
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    k = obc_inputs.target_count(0.6, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    What = obc.obc_gather_trace(W, res["trace"], counts)
    nm = obc.obc_prune_rows(W, Hinv, nm=(2, 4))
    obc.obc_check()
    Xn, Wn = _np(X), _np(W).astype(np.float64)
    Ho = orc.hessian(Xn)
    Ao = orc.invert(Ho)
    assert np.linalg.norm(_np(Hinv) - Ao) / np.linalg.norm(Ao) < 1e-4
    ro = orc.prune_rows(Ao, Wn, n_threads=16)
    co = orc.global_select(ro["loss"], k)
    Wo = orc.reconstruct(Ao, Wn, co)
    # counts may differ by near-ties between the fp32 and fp64 inverses; the layer error may not
    assert np.abs(_np(counts) - co).sum() <= 0.002 * k
    Hq = Ho - 0.0  # (w-w^)^T H (w-w^) / 2 with the damped H = ||.X||^2 + lambda/2 ||.||^2
    def quad(Wh):
        E = Wn - Wh
        return 0.5 * float(np.sum((E @ Hq) * E))
    e_gpu, e_orc = quad(_np(What).astype(np.float64)), quad(Wo)
    assert abs(e_gpu - e_orc) <= 1e-3 * e_orc, (e_gpu, e_orc)
    no = orc.prune_rows(Ao, Wn, nm=(2, 4), n_threads=16)
    e_gpu, e_orc = quad(_np(nm["W"]).astype(np.float64)), quad(no["W"])
    assert abs(e_gpu - e_orc) <= 1e-3 * e_orc, (e_gpu, e_orc)
    zeros = (_np(nm["W"]) == 0).reshape(R, -1, 4).sum(axis=2)
    assert np.all(zeros == 2)


def test_compound_prune_then_quantize(obc, orc):
    """configs[4]'s recipe at a size the oracle finishes: global pruning to 50 %, then OBQ 4-bit on
    the survivors (dense sub-problem per row), GPU vs oracle row by row."""
    W, X, _ = obc_inputs.make_layer("conv512x4608", device="cuda", d_row=6, d_col=448, n_samples=4000)
    R, d = W.shape
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    k = obc_inputs.target_count(0.5, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    Wp = obc.obc_gather_trace(W, res["trace"], counts)
    live = (1 - mask).contiguous()
    delta, offset, maxq = obc.obc_minmax_grid(Wp, 4, live=live)
    q = obc.obc_quant_rows(Wp, Hinv, delta, offset, maxq, live=live)
    obc.obc_check()
    st = RowParity()
    A = _np(Hinv)
    for i in range(R):
        n_live = int(live[i].sum())
        check_row(orc, st, "quant", A, _np(Wp[i]), _np(q["order"][i]), _np(q["loss"][i]), _np(q["W"][i]),
                  n_live, grid=(float(delta[i]), float(offset[i]), maxq), g_codes=_np(q["codes"][i]),
                  live=_np(live[i]))
    print(st)
    st.assert_order_rule()
    assert torch.all(q["W"][mask.bool()] == 0) and torch.all(q["codes"][mask.bool()] == -1)


def test_rank1_strategy_at_full_width(obc, orc):
    """The literal rank-1 schedule at d_col = 2304 (a few rows): same protocol, same tolerances."""
    import paper_2208_11580_amd as pkg

    W, X, _ = obc_inputs.make_layer("conv256x2304", device="cuda", d_row=4)
    d = W.shape[1]
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    delta, offset, maxq = obc.obc_minmax_grid(W, 4)
    q = obc.obc_quant_rows(W, Hinv, delta, offset, maxq, strategy=pkg.STRATEGY_RANK1)
    p = obc.obc_prune_rows(W, Hinv, strategy=pkg.STRATEGY_RANK1)
    obc.obc_check()
    st = RowParity()
    A = _np(Hinv)
    check_row(orc, st, "quant", A, _np(W[1]), _np(q["order"][1]), _np(q["loss"][1]), _np(q["W"][1]), d,
              grid=(float(delta[1]), float(offset[1]), maxq), g_codes=_np(q["codes"][1]))
    check_row(orc, st, "prune", A, _np(W[2]), _np(p["order"][2]), _np(p["loss"][2]), _np(p["W"][2]), d)
    print(st)
    st.assert_order_rule()
    # the two strategies take the same decisions
    qb = obc.obc_quant_rows(W, Hinv, delta, offset, maxq, strategy=pkg.STRATEGY_BLOCKED)
    assert (q["order"] != qb["order"]).float().mean().item() < 0.002
    assert (q["codes"] != qb["codes"]).float().mean().item() < 0.002


def test_conv256x2304_block4_sampled_rows(obc, orc):
    """Block pruning (blocks of 4) of the whole 256 x 2304 layer in the deferred-update solver; the
    oracle replays sampled rows, the rest is checked through properties."""
    W, X, _ = obc_inputs.make_layer("conv256x2304", device="cuda")
    R, d = W.shape
    c = 4
    H = obc.obc_hessian(X)
    Hd = torch.tensor(_np(H).astype(np.float64), device="cuda")
    Hinv = obc.obc_invert(H)
    kb = d // c // 2                     # half of the blocks of every row
    res = obc.obc_prune_blocks(W, Hinv, c, k_blocks=kb)
    obc.obc_check()
    A = _np(Hinv)
    rows = [3, 130]
    swaps = 0
    for i in rows:
        swaps += check_block_row(orc, A, _np(W[i]), c, _np(res["order"][i]), _np(res["loss"][i]),
                                 _np(res["W"][i]), kb)
    print("rows with near-tie swaps:", swaps)
    # every row: zeros exactly on the chosen aligned blocks, nowhere else
    zero = (res["W"] == 0)
    blk_zero = zero.view(R, d // c, c)
    assert torch.all(blk_zero.all(dim=2) == blk_zero.any(dim=2))
    chosen = torch.zeros(R, d // c, dtype=torch.bool, device="cuda")
    chosen.scatter_(1, res["order"].long(), True)
    assert torch.equal(chosen, blk_zero.all(dim=2))
    assert torch.all(res["loss"] >= 0)
    # loss identity on every row: the block losses add up to 1/2 (w - w^)^T H (w - w^)
    dW = (W - res["W"]).double()
    q = 0.5 * ((dW @ Hd) * dW).sum(dim=1)
    dev = float(((res["loss"].double().sum(dim=1) - q).abs() / q).max())
    print("loss identity, largest relative deviation over the rows: %.2e" % dev)
    assert dev < 1e-5


def test_conv256x2304_sequential_obq_with_outlier_heuristic(obc, orc):
    """The sequential variant at full size: inputs of a perturbed model, re-fit sharing the
    factorisation with the inverse, then 3-bit OBQ on a symmetric grid shrunk by 20 % with the
    outlier heuristic; sampled rows against the oracle."""
    W, X, _ = obc_inputs.make_layer("conv256x2304", device="cuda")
    R, d = W.shape
    torch.manual_seed(8)
    Y = (W @ X).contiguous()
    Xc = (X + 0.1 * X.std() * torch.randn_like(X)).contiguous()
    del X
    H = obc.obc_hessian(Xc)
    C = obc.obc_cross(Xc, Y)
    H0 = H.clone()
    Wr = obc.obc_refit(H, C, invert_in_place=True)
    # the re-fit against the oracle, fed the GPU's H and C (sampled rows; the solve is per row)
    rows = [5, 250]
    ref = orc.refit(_np(H0).astype(np.float64), _np(C[rows]).astype(np.float64))
    assert np.linalg.norm(_np(Wr[rows]) - ref) <= 1e-6 * np.linalg.norm(ref)
    delta, offset, maxq = obc.obc_minmax_grid(Wr, 3, symmetric=True)
    delta = (delta * 0.8).contiguous()
    offset = (offset * 0.8).contiguous()
    res = obc.obc_quant_rows(Wr, H, delta, offset, maxq, outliers=True)
    plain = obc.obc_quant_rows(Wr, H, delta, offset, maxq)
    obc.obc_check()
    assert not torch.equal(res["order"], plain["order"])      # the heuristic is active
    A = _np(H)
    st = RowParity()
    for i in rows:
        check_row(orc, st, "quant", A, _np(Wr[i]), _np(res["order"][i]), _np(res["loss"][i]), _np(res["W"][i]), d,
                  grid=(float(delta[i]), float(offset[i]), maxq), g_codes=_np(res["codes"][i]), outlier=True)
    print(st)
    st.assert_order_rule()


def test_width_4608_first_blocks(obc, orc):
    """The widest layer of the workloads (d_col = 4608) uses the panel variant with nine owned
    indices per thread and blocks of 24; the oracle replays the first 240 steps of one row."""
    W, X, _ = obc_inputs.make_layer("conv512x4608", device="cuda", d_row=3, n_samples=12000)
    R, d = W.shape
    assert d == 4608
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    k = 240
    res = obc.obc_prune_rows(W, Hinv, k_steps=k)
    obc.obc_check()
    st = RowParity()
    check_row(orc, st, "prune", _np(Hinv), _np(W[1]), _np(res["order"][1]), _np(res["loss"][1]),
              _np(res["W"][1]), k)
    print(st)
    st.assert_order_rule()
    assert int((res["W"] == 0).sum()) == R * k
    # OBQ over the same width: every weight ends on its grid value, the trace of loss changes sums
    # to the quadratic form (checked in fp64 against H itself)
    delta, offset, maxq = obc.obc_minmax_grid(W, 4)
    q = obc.obc_quant_rows(W, Hinv, delta, offset, maxq)
    obc.obc_check()
    deq = (offset[:, None].double() + delta[:, None].double() * q["codes"].double()).float()
    assert torch.equal(q["W"], deq)
    H = torch.linalg.inv(Hinv.double())
    dW = (W - q["W"]).double()
    quad = 0.5 * ((dW @ H) * dW).sum(dim=1)
    rel = ((q["loss"].double().sum(dim=1) - quad).abs() / quad).max().item()
    print("loss identity at d_col = 4608, worst row: rel %.2e" % rel)
    assert rel <= 1e-3


def test_width_4608_quantize_survivors(obc, orc):
    """Prune-then-quantize at d_col = 4608: half of every row is pruned, the survivors are quantized
    on the dense sub-problem.  The GPU removes the pruned indices from H^-1 in blocks of 64 (block
    form of Lemma 1) and the rest one by one; the oracle inverts the survivors' sub-Hessian."""
    W, X, _ = obc_inputs.make_layer("conv512x4608", device="cuda", d_row=3, n_samples=12000)
    R, d = W.shape
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    counts = torch.tensor([d // 2, d // 2 - 37, d // 2 + 101], dtype=torch.int32, device="cuda")
    p = obc.obc_prune_rows(W, Hinv, k_steps=d // 2 + 101, stop_counts=counts)
    live = (p["W"] != 0).to(torch.uint8)
    assert torch.equal((1 - live).sum(dim=1).to(torch.int32), counts)
    delta, offset, maxq = obc.obc_minmax_grid(p["W"], 4, live=live)
    q = obc.obc_quant_rows(p["W"], Hinv, delta, offset, maxq, live=live)
    obc.obc_check()
    i = 1
    st = RowParity()
    k = int(live[i].sum())
    check_row(orc, st, "quant", _np(Hinv), _np(p["W"][i]), _np(q["order"][i]), _np(q["loss"][i]), _np(q["W"][i]), k,
              grid=(float(delta[i]), float(offset[i]), maxq), g_codes=_np(q["codes"][i]), live=_np(live[i]))
    print(st)
    st.assert_order_rule()
    # every row: pruned weights stay zero with code -1, survivors sit on their grid
    assert torch.all(q["W"][live == 0] == 0) and torch.all(q["codes"][live == 0] == -1)
    c = q["codes"]
    assert int(c[live != 0].min()) >= 0 and int(c[live != 0].max()) <= maxq


@pytest.mark.parametrize("d_col,kb", [(2400, 30), (3200, 14), (4200, 12)])
def test_wide_block_pruning_first_blocks(obc, orc, d_col, kb):
    """Block pruning (blocks of 4) above 2304 columns runs on the panel variants with six, eight and
    nine owned indices per thread (blocks of 40, 28 and 24 steps); the oracle replays the first
    block steps (two to three such blocks of steps) of one row."""
    W, X, _ = obc_inputs.make_layer("ffn768x3072", device="cuda", d_row=2, d_col=d_col, n_samples=8000)
    R, d = W.shape
    assert d == d_col
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    res = obc.obc_prune_blocks(W, Hinv, 4, k_blocks=kb)
    obc.obc_check()
    check_block_row(orc, _np(Hinv), _np(W[1]), 4, _np(res["order"][1]), _np(res["loss"][1]), _np(res["W"][1]), kb)
    assert int((res["W"] == 0).sum()) == R * kb * 4


def test_width_3200_first_steps(obc, orc):
    """Live sizes 3073..4096 run on the panel variant with eight owned indices per thread and blocks of
    28 steps; the oracle replays the first 60 steps (two blocks and a flush each, then a part) of one
    row."""
    W, X, _ = obc_inputs.make_layer("ffn768x3072", device="cuda", d_row=2, d_col=3200, n_samples=8000)
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    k = 60
    res = obc.obc_prune_rows(W, Hinv, k_steps=k)
    obc.obc_check()
    st = RowParity()
    check_row(orc, st, "prune", _np(Hinv), _np(W[0]), _np(res["order"][0]), _np(res["loss"][0]),
              _np(res["W"][0]), k)
    print(st)
    st.assert_order_rule()
    assert int((res["W"] == 0).sum()) == 2 * k


@pytest.mark.parametrize("name", ["attn768x768", "ffn3072x768"])
def test_transformer_layers_on_768_features_full_size(obc, orc, name):
    """The two transformer layers on 768 input features at their real row counts and N = 49 152
    (the 3072-row layer is the workload that runs three rows per compute unit): pruning with full
    traces and the global step to 50 %, and OBQ 4-bit; sampled rows against the oracle, the rest
    through properties."""
    W, X, _ = obc_inputs.make_layer(name, device="cuda")
    R, d = W.shape
    assert X.shape == (768, 49152)
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    del X
    A = _np(Hinv)
    rows = [int(r) for r in np.linspace(0, R - 1, 16).round()]
    # ---- pruning, global step, weights from the trace
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    obc.obc_check()
    k = obc_inputs.target_count(0.5, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    What = obc.obc_gather_trace(W, res["trace"], counts)
    assert int(counts.sum()) == k and int(mask.sum()) == k
    assert torch.equal(What == 0, mask.bool())
    srt = torch.sort(res["order"], dim=1).values
    assert torch.equal(srt, torch.arange(d, device="cuda", dtype=torch.int32).expand(R, d))
    assert torch.all(res["loss"] >= 0)
    st = RowParity()
    ro = check_rows(orc, st, "prune", A, _np(W[rows]), _np(res["order"][rows]), _np(res["loss"][rows]),
                    _np(res["W"][rows]), d)
    print(name, "prune", st)
    st.assert_order_rule()
    # Algorithm 2 on the GPU's traces equals the oracle's Algorithm 2 on the same traces
    co = orc.global_select(_np(res["loss"]).astype(np.float64), k)
    assert np.array_equal(_np(counts), co)
    # the gathered weights of the sampled rows are the oracle's state after counts[i] steps
    for n, i in enumerate(rows[:6]):
        c = int(counts[i])
        ref = orc.prune_row(A.astype(np.float64), _np(W[i]).astype(np.float64), k_steps=c,
                            forced=_np(res["order"][i]).astype(np.int32)).w
        got = _np(What[i]).astype(np.float64)
        assert np.linalg.norm(got - ref) <= 1e-4 * np.linalg.norm(ref)
    del res, What
    # ---- OBQ 4-bit
    delta, offset, maxq = obc.obc_minmax_grid(W, 4)
    q = obc.obc_quant_rows(W, Hinv, delta, offset, maxq)
    obc.obc_check()
    st = RowParity()
    check_rows(orc, st, "quant", A, _np(W[rows]), _np(q["order"][rows]), _np(q["loss"][rows]), _np(q["W"][rows]), d,
               grids=(_np(delta[rows]), _np(offset[rows]), maxq), g_codes=_np(q["codes"][rows]))
    print(name, "obq4", st)
    st.assert_order_rule()
    c = q["codes"]
    assert int(c.min()) >= 0 and int(c.max()) <= maxq
    deq = (offset[:, None].double() + delta[:, None].double() * c.double()).float()
    assert torch.equal(q["W"], deq)
    srt = torch.sort(q["order"], dim=1).values
    assert torch.equal(srt, torch.arange(d, device="cuda", dtype=torch.int32).expand(R, d))


def test_conv512x4608_every_panel_variant_and_compound(obc, orc):
    """The widest workload (d_col = 4608, N = 100 000) on 64 rows: one row is followed by the oracle
    through all 4608 pruning steps, which crosses every panel variant and every flush block size;
    then the global step to 50 % and OBQ 4-bit on the survivors, four rows against the oracle (which
    inverts each row's sub-Hessian of survivors directly)."""
    from concurrent.futures import ThreadPoolExecutor

    W, X, _ = obc_inputs.make_layer("conv512x4608", device="cuda", d_row=64)
    R, d = W.shape
    assert d == 4608 and X.shape[1] == 100000
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    del X
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    obc.obc_check()
    k = obc_inputs.target_count(0.5, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    Wp = obc.obc_gather_trace(W, res["trace"], counts)
    live = (1 - mask).contiguous()
    delta, offset, maxq = obc.obc_minmax_grid(Wp, 4, live=live)
    q = obc.obc_quant_rows(Wp, Hinv, delta, offset, maxq, live=live)
    obc.obc_check()
    assert int(counts.sum()) == k
    assert torch.equal(Wp == 0, mask.bool())
    assert torch.all(q["W"][mask.bool()] == 0) and torch.all(q["codes"][mask.bool()] == -1)
    c = q["codes"]
    assert int(c[live != 0].min()) >= 0 and int(c[live != 0].max()) <= maxq
    srt = torch.sort(res["order"], dim=1).values
    assert torch.equal(srt, torch.arange(d, device="cuda", dtype=torch.int32).expand(R, d))

    A = _np(Hinv)
    st_p, st_q = RowParity(), RowParity()
    full_row = 33
    jobs = [lambda: check_row(orc, st_p, "prune", A, _np(W[full_row]), _np(res["order"][full_row]),
                              _np(res["loss"][full_row]), _np(res["W"][full_row]), d)]
    for i in (0, 21, 42, 63):
        n_live = int(live[i].sum())
        jobs.append(lambda i=i, n_live=n_live: check_row(
            orc, st_q, "quant", A, _np(Wp[i]), _np(q["order"][i]), _np(q["loss"][i]), _np(q["W"][i]), n_live,
            grid=(float(delta[i]), float(offset[i]), maxq), g_codes=_np(q["codes"][i]), live=_np(live[i])))
    # the oracle's rows are independent and its C code runs outside the interpreter lock
    with ThreadPoolExecutor(max_workers=len(jobs)) as pool:
        futs = [pool.submit(j) for j in jobs]
        for f in futs:
            f.result()
    print("4608 full row:", st_p)
    print("4608 compound rows:", st_q)
    st_p.assert_order_rule()
    st_q.assert_order_rule()
    assert st_p.rows == 1 and st_q.rows == 4


def test_conv256x2304_closed_form_recovery(obc, orc):
    """The group-OBS closed form at full size: the 256 x 2304 layer pruned to 50 % by the global step;
    every row's recovered weights against the weights gathered from the trace, sampled rows against
    the oracle's closed form."""
    W, X, _ = obc_inputs.make_layer("conv256x2304", device="cuda")
    R, d = W.shape
    Hinv = obc.obc_invert(obc.obc_hessian(X))
    del X
    res = obc.obc_prune_rows(W, Hinv, want_trace=True)
    k = obc_inputs.target_count(0.5, R, d)
    counts, mask = obc.obc_global_select(res["loss"], res["order"], k)
    from_trace = obc.obc_gather_trace(W, res["trace"], counts)
    del res
    got = obc.obc_reconstruct_rows(W, Hinv, mask, max_pruned=int(counts.max()))
    obc.obc_check()
    assert torch.equal(got == 0, mask.bool())
    num = (got.double() - from_trace.double()).norm(dim=1)
    den = from_trace.double().norm(dim=1)
    print("closed form vs trace, worst row: rel %.2e" % float((num / den).max()))
    assert torch.all(num <= 1e-4 * den)
    rows = [0, 100, 255]
    ref = orc.reconstruct_closed_form(_np(Hinv), _np(W[rows]), _np(mask[rows]))
    g = _np(got[rows]).astype(np.float64)
    for n in range(len(rows)):
        assert np.linalg.norm(g[n] - ref[n]) <= 1e-6 * np.linalg.norm(ref[n])
