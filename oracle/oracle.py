"""ExactOBS / OBQ oracle (CPU, fp64) -- Python face of ``obc_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's cpu-baseline leg.  It shares no code with the HIP library and never
imports it.

What each function follows in the paper (arxiv 2208.11580):

* ``hessian``         Sec. 4: H = 2 X X^T, plus the diagonal dampening of "Implementation Details"
* ``invert``          Sec. 4 Step 1: the inverse every row starts from
* ``prune_row(s)``    Algorithm 1 (+ the N:M rule of Sec. 4 "N:M Sparsity")
* ``minmax_grid``     asymmetric per-channel min-max grid (Sec. 6 uses asymmetric per-channel grids)
* ``quant_row(s)``    Sec. 5 eq. (7) / Appendix Algorithm 3
* ``global_select``   Appendix Algorithm 2
* ``reconstruct``     Sec. 4 Step 2: a row's weights depend only on how many of its weights were pruned
* ``reconstruct_closed_form``  Sec. 4 Step 2: the group-OBS formula for all pruned weights of a row at once
* ``compound_row``    Sec. 6 "Experimental Setup": prune first, then quantize the remaining weights,
                      on the dense sub-problem of the non-zeros (Sec. 4 "Implementation Details")
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_int, c_int32, c_int64, c_uint8

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "obc_oracle.c")
_LIB = os.path.join(_HERE, "libobc_oracle.so")

ORC_OK, ORC_BAD_ARG, ORC_NOT_SPD, ORC_NUMERIC = 0, -1, -3, -5


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp, ip, bp = POINTER(c_double), POINTER(c_int32), POINTER(c_uint8)
        lib.orc_spd_inverse.argtypes = [dp, c_int]
        lib.orc_spd_inverse.restype = c_int
        lib.orc_quant_code.argtypes = [c_double, c_double, c_double, c_int]
        lib.orc_quant_code.restype = c_int
        lib.orc_row_solve.argtypes = [
            c_int, dp, c_int, dp, c_int, c_int, c_int, c_int, c_double, c_double, c_int,
            ip, ip, dp, ip, dp, dp, dp, dp, dp, dp, bp,
        ]
        lib.orc_row_solve.restype = c_int
        lib.orc_rows_solve.argtypes = [
            c_int, dp, c_int, c_int, dp, c_int, c_int, c_int, c_int, dp, dp, c_int,
            ip, dp, ip, dp, dp, c_int, POINTER(c_int),
        ]
        lib.orc_rows_solve.restype = c_int
        lib.orc_block_row_solve.argtypes = [dp, c_int, dp, c_int, c_int, ip, ip, dp, dp, dp, dp, dp, dp, bp]
        lib.orc_block_row_solve.restype = c_int
        lib.orc_block_rows_solve.argtypes = [dp, c_int, c_int, dp, c_int, c_int, ip, dp, dp, c_int,
                                             POINTER(c_int)]
        lib.orc_block_rows_solve.restype = c_int
        lib.orc_global_select.argtypes = [dp, c_int, c_int, c_int64, ip]
        lib.orc_global_select.restype = c_int
        _lib = lib
    return _lib


def _d(a):
    return a.ctypes.data_as(POINTER(c_double)) if a is not None else None


def _i(a):
    return a.ctypes.data_as(POINTER(c_int32)) if a is not None else None


def _b(a):
    return a.ctypes.data_as(POINTER(c_uint8)) if a is not None else None


class OracleError(RuntimeError):
    def __init__(self, code, where):
        super().__init__("oracle %s failed with status %d" % (where, code))
        self.code = code


# --------------------------------------------------------------------------- Hessian / inverse
def hessian(X, damp_rel: float = 0.01):
    """H = 2 X X^T + damp_rel * mean(diag(2 X X^T)) * I in fp64 (X is d_col x N).

    The sum over samples is not divided by N.  ``damp_rel < 0`` leaves H undamped.
    """
    X = np.asarray(X, dtype=np.float64)
    H = 2.0 * (X @ X.T)
    if damp_rel is not None and damp_rel >= 0:
        lam = damp_rel * np.mean(np.diag(H))
        H = H + lam * np.eye(H.shape[0])
    return H


def invert(H):
    """Inverse of the SPD matrix H through its Cholesky factor (plain C loops)."""
    A = np.array(H, dtype=np.float64, order="C", copy=True)
    if A.ndim != 2 or A.shape[0] != A.shape[1]:
        raise ValueError("H must be square")
    rc = _load().orc_spd_inverse(_d(A), A.shape[0])
    if rc != ORC_OK:
        raise OracleError(rc, "orc_spd_inverse")
    return A


def cross(X, Y):
    """C = 2 Y X^T in fp64 (X is d_col x N, Y is d_row x N): the second moment that the sequential
    variant accumulates beside the Hessian (appendix "Sequential Quantization with OBQ")."""
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    return 2.0 * (Y @ X.T)


def refit(H, C):
    """Dense weights re-optimised for new inputs (appendix "Sequential Quantization with OBQ").

    The closed form of linear regression, W^T = (X X^T)^-1 X Y^T, written with the quantities the
    method already holds: H = 2 X X^T and C = 2 Y X^T give W^T = H^-1 C^T.  With a dampened H this is
    the minimiser of the quadratic whose Hessian the row solver assumes (gradient W H - C = 0).
    The linear system is solved by the library routine; H^-1 is not formed.
    """
    H = np.asarray(H, dtype=np.float64)
    C = np.asarray(C, dtype=np.float64)
    return np.linalg.solve(H, C.T).T


# --------------------------------------------------------------------------- one row
class RowResult:
    """Outputs of one greedy row run (arrays are fp64 / int32 numpy)."""

    __slots__ = ("order", "loss", "codes", "w", "trace", "min_score", "pick_score",
                 "pre_round", "A", "live")


def _row_solve(mode, Hinv, w, k_steps, nm=(0, 0), grid=(1.0, 0.0, 0), forced=None,
               want_trace=False, outlier=False):
    Hinv = np.ascontiguousarray(Hinv, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    d = w.shape[0]
    assert Hinv.shape == (d, d)
    r = RowResult()
    r.order = np.zeros(k_steps, np.int32)
    r.loss = np.zeros(k_steps, np.float64)
    r.codes = np.full(d, -1, np.int32) if mode == 1 else None
    r.w = np.zeros(d, np.float64)
    r.trace = np.zeros((k_steps, d), np.float64) if want_trace else None
    r.min_score = np.zeros(k_steps, np.float64)
    r.pick_score = np.zeros(k_steps, np.float64)
    r.pre_round = np.zeros(k_steps, np.float64) if mode == 1 else None
    r.A = np.zeros((d, d), np.float64)
    r.live = np.zeros(d, np.uint8)
    f = None if forced is None else np.ascontiguousarray(forced, dtype=np.int32)
    if f is not None:
        assert f.shape[0] >= k_steps
    rc = _load().orc_row_solve(
        mode, _d(Hinv), d, _d(w), k_steps, int(nm[0]), int(nm[1]), int(bool(outlier)),
        float(grid[0]), float(grid[1]), int(grid[2]), _i(f), _i(r.order), _d(r.loss),
        _i(r.codes), _d(r.w), _d(r.trace), _d(r.min_score), _d(r.pick_score),
        _d(r.pre_round), _d(r.A), _b(r.live),
    )
    if rc != ORC_OK:
        raise OracleError(rc, "orc_row_solve")
    return r


def prune_row(Hinv, w, k_steps=None, nm=(0, 0), forced=None, want_trace=False):
    """Algorithm 1 on one row; ``nm=(N, M)`` switches on the N:M eligibility rule."""
    d = len(w)
    if k_steps is None:
        k_steps = d if nm[1] == 0 else (d // nm[1]) * (nm[1] - nm[0])
    return _row_solve(0, Hinv, w, k_steps, nm=nm, forced=forced, want_trace=want_trace)


def block_prune_row(Hinv, w, c, k_blocks=None, forced=None, want_trace=False):
    """Block-pruning variant (Sec. 4 "Block-Sparsity", eq. (5)) on one row, blocks of ``c``.

    ``order`` holds block indices, ``loss`` the halved block scores.
    """
    Hinv = np.ascontiguousarray(Hinv, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    d = w.shape[0]
    assert Hinv.shape == (d, d)
    if k_blocks is None:
        k_blocks = d // c
    r = RowResult()
    r.order = np.zeros(k_blocks, np.int32)
    r.loss = np.zeros(k_blocks, np.float64)
    r.codes = None
    r.pre_round = None
    r.w = np.zeros(d, np.float64)
    r.trace = np.zeros((k_blocks, d), np.float64) if want_trace else None
    r.min_score = np.zeros(k_blocks, np.float64)
    r.pick_score = np.zeros(k_blocks, np.float64)
    r.A = np.zeros((d, d), np.float64)
    r.live = np.zeros(d, np.uint8)
    f = None if forced is None else np.ascontiguousarray(forced, dtype=np.int32)
    if f is not None:
        assert f.shape[0] >= k_blocks
    rc = _load().orc_block_row_solve(_d(Hinv), d, _d(w), int(c), int(k_blocks), _i(f), _i(r.order),
                                     _d(r.loss), _d(r.w), _d(r.trace), _d(r.min_score),
                                     _d(r.pick_score), _d(r.A), _b(r.live))
    if rc != ORC_OK:
        raise OracleError(rc, "orc_block_row_solve")
    return r


def block_prune_rows(Hinv, W, c, k_blocks=None, n_threads=0):
    Hinv = np.ascontiguousarray(Hinv, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.float64)
    R, d = W.shape
    if k_blocks is None:
        k_blocks = d // c
    order = np.zeros((R, k_blocks), np.int32)
    loss = np.zeros((R, k_blocks), np.float64)
    W_out = np.zeros((R, d), np.float64)
    used = c_int(0)
    rc = _load().orc_block_rows_solve(_d(Hinv), R, d, _d(W), int(c), int(k_blocks), _i(order),
                                      _d(loss), _d(W_out), int(n_threads), ctypes.byref(used))
    if rc != ORC_OK:
        raise OracleError(rc, "orc_block_rows_solve")
    return dict(order=order, loss=loss, W=W_out, threads=used.value)


def minmax_grid(w_live, bits: int):
    """Asymmetric min-max grid of one row: (delta, offset, maxq).

    delta = (max - min) / maxq, offset = min; a constant row gets delta = 1.
    """
    maxq = (1 << bits) - 1
    lo = float(np.min(w_live))
    hi = float(np.max(w_live))
    delta = (hi - lo) / maxq if (hi > lo and maxq > 0) else 1.0
    return delta, lo, maxq


def quant_code(w, delta, offset, maxq):
    return _load().orc_quant_code(float(w), float(delta), float(offset), int(maxq))


def symmetric_grid(w_live, bits: int):
    """Grid symmetric about zero spanning [-max|w|, +max|w|]: (delta, offset, maxq).

    The paper uses symmetric per-channel grids in some experiments (Sec. 6) without giving the
    formula; this is the plain reading (range symmetric, 2^bits levels).
    """
    maxq = (1 << bits) - 1
    m = float(np.max(np.abs(w_live)))
    delta = 2.0 * m / maxq if (m > 0 and maxq > 0) else 1.0
    return delta, -m, maxq


def quant_row(Hinv, w, grid, k_steps=None, forced=None, want_trace=False, outlier=False):
    """Appendix Algorithm 3 on one row; ``grid = (delta, offset, maxq)``.

    ``outlier=True`` switches on the outlier heuristic of Sec. 5 (see obc_oracle.c for the reading).
    """
    d = len(w)
    if k_steps is None:
        k_steps = d
    return _row_solve(1, Hinv, w, k_steps, grid=grid, forced=forced, want_trace=want_trace,
                      outlier=outlier)


# --------------------------------------------------------------------------- many rows
def _rows_solve(mode, Hinv, W, k_steps, nm, delta, offset, maxq, want_trace, n_threads, outlier=False):
    Hinv = np.ascontiguousarray(Hinv, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.float64)
    R, d = W.shape
    order = np.zeros((R, k_steps), np.int32)
    loss = np.zeros((R, k_steps), np.float64)
    codes = np.full((R, d), -1, np.int32) if mode == 1 else None
    W_out = np.zeros((R, d), np.float64)
    trace = np.zeros((R, k_steps, d), np.float64) if want_trace else None
    dl = np.ascontiguousarray(delta, dtype=np.float64) if delta is not None else None
    of = np.ascontiguousarray(offset, dtype=np.float64) if offset is not None else None
    used = c_int(0)
    rc = _load().orc_rows_solve(
        mode, _d(Hinv), R, d, _d(W), k_steps, int(nm[0]), int(nm[1]), int(bool(outlier)), _d(dl), _d(of),
        int(maxq), _i(order), _d(loss), _i(codes), _d(W_out), _d(trace), int(n_threads),
        ctypes.byref(used),
    )
    if rc != ORC_OK:
        raise OracleError(rc, "orc_rows_solve")
    return dict(order=order, loss=loss, codes=codes, W=W_out, trace=trace, threads=used.value)


def prune_rows(Hinv, W, k_steps=None, nm=(0, 0), want_trace=False, n_threads=0):
    d = W.shape[1]
    if k_steps is None:
        k_steps = d if nm[1] == 0 else (d // nm[1]) * (nm[1] - nm[0])
    return _rows_solve(0, Hinv, W, k_steps, nm, None, None, 0, want_trace, n_threads)


def quant_rows(Hinv, W, delta, offset, maxq, n_threads=0, outlier=False):
    return _rows_solve(1, Hinv, W, W.shape[1], (0, 0), delta, offset, maxq, False, n_threads, outlier)


# --------------------------------------------------------------------------- global step
def global_select(loss, k: int):
    """Appendix Algorithm 2: per-row pruned counts for k pruned weights in the layer."""
    L = np.ascontiguousarray(loss, dtype=np.float64)
    R, d = L.shape
    counts = np.zeros(R, np.int32)
    rc = _load().orc_global_select(_d(L), R, d, int(k), _i(counts))
    if rc != ORC_OK:
        raise OracleError(rc, "orc_global_select")
    return counts


def mask_from_counts(order, counts, d):
    """mask[i, j] = 1 iff weight j of row i is among the first counts[i] pruned in row i."""
    R = order.shape[0]
    mask = np.zeros((R, d), np.uint8)
    for i in range(R):
        mask[i, order[i, : counts[i]]] = 1
    return mask


def reconstruct(Hinv, W, counts):
    """Weights of every row after exactly counts[i] steps of Algorithm 1 (replay)."""
    W = np.asarray(W, dtype=np.float64)
    out = np.zeros_like(W)
    for i in range(W.shape[0]):
        out[i] = prune_row(Hinv, W[i], k_steps=int(counts[i])).w
    return out


def reconstruct_closed_form(Hinv, W, mask):
    """Weights of every row for a given mask by the group-OBS formula of Sec. 4 Step 2 (its sign as in
    eq. (5)): with P the pruned indices of the row,

        w_hat = w - H^-1[:, P] ((H^-1)[P, P])^-1 w_P,      w_hat[P] = 0 exactly,

    from the original weights and the original inverse Hessian.  The linear system is solved by the
    library routine.  ``mask`` is R x d, non-zero = pruned.
    """
    A = np.asarray(Hinv, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    out = W.copy()
    for i in range(W.shape[0]):
        P = np.flatnonzero(np.asarray(mask[i]) != 0)
        if P.size == 0:
            continue
        z = np.linalg.solve(A[np.ix_(P, P)], W[i, P])
        out[i] = W[i] - A[:, P] @ z
        out[i, P] = 0.0
    return out


# --------------------------------------------------------------------------- compound
def compound_row(H, w_pruned, live, bits: int):
    """OBQ over the surviving weights of an already pruned row.

    ``w_pruned`` is the row after pruning and ``live`` flags its survivors (non-zero
    = kept).  The inverse of the sub-Hessian H[S, S] is formed directly; the grid is
    the min-max grid of the survivors.  Returns (w_out, codes, row result) at full
    width, with code -1 and weight 0 at pruned positions.
    """
    w_pruned = np.asarray(w_pruned, dtype=np.float64)
    d = w_pruned.shape[0]
    S = np.flatnonzero(np.asarray(live) != 0)
    w_out = np.zeros(d, np.float64)
    codes = np.full(d, -1, np.int32)
    if S.size == 0:
        return w_out, codes, None
    A = invert(np.asarray(H, dtype=np.float64)[np.ix_(S, S)])
    grid = minmax_grid(w_pruned[S], bits)
    r = quant_row(A, w_pruned[S], grid)
    w_out[S] = r.w
    codes[S] = r.codes
    return w_out, codes, r


def layer_error(W, W_hat, X):
    """||W X - W_hat X||_F^2 in fp64 (Sec. 3 eq. (2))."""
    D = (np.asarray(W, np.float64) - np.asarray(W_hat, np.float64)) @ np.asarray(X, np.float64)
    return float(np.sum(D * D))
