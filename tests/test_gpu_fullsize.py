"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: the whole layer
runs on the GPU, the oracle checks sampled rows one by one (tests/parity.py protocol)."""
import numpy as np
import pytest
import torch

import obc_inputs
from tests.parity import RowParity, check_row

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
    rows = [0, 101, 255]
    order, loss, Wo, codes = (_np(res[k][rows]) for k in ("order", "loss", "W", "codes"))
    Wn, dl, of = _np(W[rows]), _np(delta[rows]), _np(offset[rows])
    for n, i in enumerate(rows):
        check_row(orc, st, "quant", A, Wn[n], order[n], loss[n], Wo[n], d,
                  grid=(float(dl[n]), float(of[n]), maxq), g_codes=codes[n])
    print(st)
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
    assert torch.allclose(res["loss"].double().sum(dim=1), 0.5 * q_obq, rtol=2e-3)
