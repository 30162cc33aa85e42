"""Thin ctypes binding of libobc.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/obc.h) and takes torch
tensors that already live on the GPU; torch is used for device memory and the current stream,
nothing else.  All arithmetic of the method runs inside the library's HIP kernels.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int, c_int64, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libobc.so")

OBC_OK = 0
OBC_ERR_BAD_ARG, OBC_ERR_BAD_SHAPE, OBC_ERR_NOT_SPD = -1, -2, -3
OBC_ERR_WORKSPACE, OBC_ERR_NUMERIC, OBC_ERR_HIP = -4, -5, -6
STRATEGY_AUTO, STRATEGY_RANK1, STRATEGY_BLOCKED = 0, 1, 2
QUANT_OUTLIERS = 1
SELECT_STATIC_MAX_WEIGHTS, SELECT_STATIC_MAX_ROWS = 2359296, 8192   # limits of obc_global_select_static

EXPORTS = [
    "obc_create", "obc_destroy", "obc_last_error", "obc_version", "obc_check",
    "obc_profile_begin", "obc_profile_end", "obc_membench", "obc_mfmabench",
    "obc_hessian_workspace_bytes", "obc_hessian",
    "obc_invert_workspace_bytes", "obc_invert",
    "obc_cross_workspace_bytes", "obc_cross", "obc_refit_workspace_bytes", "obc_refit",
    "obc_rows_workspace_bytes", "obc_prune_rows", "obc_blocks_workspace_bytes", "obc_prune_blocks", "obc_quant_rows", "obc_minmax_grid",
    "obc_global_select_workspace_bytes", "obc_global_select", "obc_global_select_static", "obc_gather_trace",
    "obc_reconstruct_workspace_bytes", "obc_reconstruct_rows",
]


KERNEL_CLASSES = ("panel", "flush", "rank1")


class KernelStat(ctypes.Structure):
    _fields_ = [("launches", c_int), ("ms", ctypes.c_double), ("bytes", ctypes.c_double),
                ("flops", ctypes.c_double)]


class ObcError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libobc error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load_library():
    """dlopen libobc.so and declare the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2208_11580_amd.build` "
            "(there is no fallback path)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, sp = c_void_p, POINTER(c_size_t)
    lib.obc_create.argtypes = [POINTER(vp), vp]
    lib.obc_destroy.argtypes = [vp]
    lib.obc_last_error.argtypes = [vp]
    lib.obc_last_error.restype = c_char_p
    lib.obc_version.argtypes = []
    lib.obc_version.restype = c_char_p
    lib.obc_check.argtypes = [vp]
    lib.obc_profile_begin.argtypes = [vp]
    lib.obc_profile_end.argtypes = [vp, POINTER(KernelStat)]
    lib.obc_membench.argtypes = [vp, c_int, c_int, vp, vp, c_size_t, c_int, POINTER(ctypes.c_double)]
    lib.obc_mfmabench.argtypes = [vp, c_int, c_int, c_int, POINTER(ctypes.c_double), POINTER(ctypes.c_double)]
    lib.obc_hessian_workspace_bytes.argtypes = [c_int, c_int64, sp]
    lib.obc_hessian.argtypes = [vp, vp, c_int, c_int64, c_int64, c_float, c_int, vp, vp, c_size_t]
    lib.obc_invert_workspace_bytes.argtypes = [c_int, sp]
    lib.obc_invert.argtypes = [vp, vp, c_int, vp, c_size_t]
    lib.obc_rows_workspace_bytes.argtypes = [c_int, c_int, c_int, sp]
    lib.obc_prune_rows.argtypes = [vp, vp, vp, c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, vp,
                                   c_int, vp, c_size_t]
    lib.obc_blocks_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, sp]
    lib.obc_prune_blocks.argtypes = [vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, c_int, vp, c_size_t]
    lib.obc_quant_rows.argtypes = [vp, vp, vp, c_int, c_int, vp, vp, c_int, vp, c_int, vp, vp, vp, vp, c_int,
                                   vp, c_size_t]
    lib.obc_minmax_grid.argtypes = [vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp]
    lib.obc_cross_workspace_bytes.argtypes = [c_int, c_int, c_int64, sp]
    lib.obc_cross.argtypes = [vp, vp, vp, c_int, c_int, c_int64, c_int64, c_int64, c_int, vp, vp, c_size_t]
    lib.obc_refit_workspace_bytes.argtypes = [c_int, c_int, sp]
    lib.obc_refit.argtypes = [vp, vp, c_int, vp, c_int, vp, c_int, vp, c_size_t]
    lib.obc_global_select_workspace_bytes.argtypes = [c_int, c_int, sp]
    lib.obc_global_select.argtypes = [vp, vp, vp, c_int, c_int, c_int64, vp, vp, vp, c_size_t]
    lib.obc_global_select_static.argtypes = [vp, vp, vp, c_int, c_int, c_int64, vp, vp]
    lib.obc_gather_trace.argtypes = [vp, vp, vp, vp, c_int, c_int, c_int, vp]
    lib.obc_reconstruct_workspace_bytes.argtypes = [c_int, c_int, c_int, sp]
    lib.obc_reconstruct_rows.argtypes = [vp, vp, vp, vp, c_int, c_int, c_int, vp, vp, c_size_t]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("obc_last_error", "obc_version"):
            fn.restype = c_int
    _lib = lib
    return lib


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libobc takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libobc takes contiguous tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected %s, got %s" % (dtype, t.dtype))
    return c_void_p(t.data_ptr())


class Context:
    """An obc_ctx bound to a torch stream (default: the current one)."""

    def __init__(self, stream: torch.cuda.Stream | None = None):
        self.lib = load_library()
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = c_void_p()
        rc = self.lib.obc_create(byref(h), c_void_p(self.stream.cuda_stream))
        if rc != OBC_OK:
            raise ObcError(rc, "obc_create failed")
        self.h = h
        self._ws = None

    def close(self):
        if getattr(self, "h", None):
            self.lib.obc_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc):
        if rc != OBC_OK:
            raise ObcError(rc, self.lib.obc_last_error(self.h).decode())

    def workspace(self, nbytes: int) -> torch.Tensor:
        """A cached device byte buffer of at least nbytes (device memory is torch's job)."""
        nbytes = max(int(nbytes), 256)
        if self._ws is None or self._ws.numel() < nbytes:
            if self._ws is not None:
                # earlier calls queued on the context's stream may still use the old buffer: the
                # allocator must not hand it out again before that stream has passed this point
                self._ws.record_stream(self.stream)
            self._ws = None
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device=torch.device("cuda", torch.cuda.current_device()))
        return self._ws

    def release_workspace(self):
        if self._ws is not None:
            self._ws.record_stream(self.stream)
        self._ws = None

    # ------------------------------------------------------------------ entry points
    def obc_check(self):
        self._ck(self.lib.obc_check(self.h))

    def obc_profile_begin(self):
        self._ck(self.lib.obc_profile_begin(self.h))

    def obc_profile_end(self):
        arr = (KernelStat * len(KERNEL_CLASSES))()
        self._ck(self.lib.obc_profile_end(self.h, arr))
        return {name: dict(launches=arr[i].launches, ms=arr[i].ms, bytes=arr[i].bytes, flops=arr[i].flops)
                for i, name in enumerate(KERNEL_CLASSES)}

    def obc_mfmabench(self, kind, iters=20000, reps=3):
        """TFLOP/s of a loop of independent fp32 (kind 0) / fp64 (kind 1) MFMA instructions."""
        ms, fl = ctypes.c_double(), ctypes.c_double()
        self._ck(self.lib.obc_mfmabench(self.h, int(kind), int(iters), int(reps), byref(ms), byref(fl)))
        return fl.value / (ms.value * 1e-3) / 1e12

    def obc_membench(self, kind, src, dst, nbytes, reps=5, streaming=False):
        """Mean milliseconds per pass of the plain read (0) / write (1) / copy (2) kernel."""
        ms = ctypes.c_double()
        self._ck(self.lib.obc_membench(self.h, int(kind), int(bool(streaming)), _ptr(src), _ptr(dst), int(nbytes),
                                       int(reps), byref(ms)))
        return ms.value

    def obc_hessian(self, X, damp_rel=0.01, H=None, accumulate=False):
        d, N = X.shape
        if H is None:
            H = torch.empty(d, d, dtype=torch.float32, device=X.device)
        need = c_size_t()
        self.lib.obc_hessian_workspace_bytes(d, N, byref(need))
        ws = self.workspace(need.value)
        ldx = X.stride(0)
        if X.stride(1) != 1:
            raise ValueError("X must have unit stride along the sample axis")
        self._ck(self.lib.obc_hessian(self.h, c_void_p(X.data_ptr()), d, N, ldx, float(damp_rel),
                                      int(bool(accumulate)), _ptr(H, torch.float32),
                                      c_void_p(ws.data_ptr()), ws.numel()))
        return H

    def obc_invert(self, H):
        d = H.shape[0]
        need = c_size_t()
        self.lib.obc_invert_workspace_bytes(d, byref(need))
        ws = self.workspace(need.value)
        self._ck(self.lib.obc_invert(self.h, _ptr(H, torch.float32), d, c_void_p(ws.data_ptr()), ws.numel()))
        return H

    def obc_cross(self, X, Y, C=None, accumulate=False):
        d_col, N = X.shape
        d_row, Ny = Y.shape
        if Ny != N:
            raise ValueError("X and Y must hold the same number of samples")
        if X.stride(1) != 1 or Y.stride(1) != 1:
            raise ValueError("X and Y must have unit stride along the sample axis")
        if C is None:
            C = torch.empty(d_row, d_col, dtype=torch.float32, device=X.device)
        need = c_size_t()
        self.lib.obc_cross_workspace_bytes(d_row, d_col, N, byref(need))
        ws = self.workspace(need.value)
        self._ck(self.lib.obc_cross(self.h, c_void_p(X.data_ptr()), c_void_p(Y.data_ptr()), d_col, d_row, N,
                                    X.stride(0), Y.stride(0), int(bool(accumulate)), _ptr(C, torch.float32),
                                    c_void_p(ws.data_ptr()), ws.numel()))
        return C

    def obc_refit(self, H, C, invert_in_place=False, W_out=None):
        d_col = H.shape[0]
        d_row = C.shape[0]
        if C.shape[1] != d_col:
            raise ValueError("C must be d_row x d_col")
        if W_out is None:
            W_out = torch.empty(d_row, d_col, dtype=torch.float32, device=H.device)
        need = c_size_t()
        self.lib.obc_refit_workspace_bytes(d_col, d_row, byref(need))
        ws = self.workspace(need.value)
        self._ck(self.lib.obc_refit(self.h, _ptr(H, torch.float32), d_col, _ptr(C, torch.float32), d_row,
                                    _ptr(W_out, torch.float32), int(bool(invert_in_place)),
                                    c_void_p(ws.data_ptr()), ws.numel()))
        return W_out

    def rows_workspace_bytes(self, R, d, strategy=STRATEGY_AUTO):
        need = c_size_t()
        rc = self.lib.obc_rows_workspace_bytes(R, d, strategy, byref(need))
        if rc != OBC_OK:
            raise ObcError(rc, "obc_rows_workspace_bytes")
        return need.value

    def obc_prune_rows(self, W, Hinv, k_steps=None, nm=(0, 0), stop_counts=None, want_trace=False,
                       strategy=STRATEGY_AUTO, out=None, live=None):
        R, d = W.shape
        if k_steps is None:
            k_steps = d if nm[1] == 0 else (d // nm[1]) * (nm[1] - nm[0])
        dev = W.device
        if out is None:
            out = {}
        order = out.get("order")
        if order is None:
            order = torch.full((R, k_steps), -1, dtype=torch.int32, device=dev)
        loss = out.get("loss")
        if loss is None:
            loss = torch.zeros((R, k_steps), dtype=torch.float32, device=dev)
        W_out = out.get("W")
        if W_out is None:
            W_out = torch.empty((R, d), dtype=torch.float32, device=dev)
        trace = out.get("trace")
        if trace is None and want_trace:
            trace = torch.empty((R, k_steps, d), dtype=torch.float32, device=dev)
        ws = self.workspace(self.rows_workspace_bytes(R, d, strategy))
        self._ck(self.lib.obc_prune_rows(
            self.h, _ptr(W, torch.float32), _ptr(Hinv, torch.float32), R, d, int(k_steps), int(nm[0]),
            int(nm[1]), _ptr(stop_counts, torch.int32), _ptr(live, torch.uint8), _ptr(order), _ptr(loss),
            _ptr(W_out), _ptr(trace),
            int(strategy), c_void_p(ws.data_ptr()), ws.numel()))
        return dict(order=order, loss=loss, W=W_out, trace=trace)

    def obc_prune_blocks(self, W, Hinv, c, k_blocks=None, stop_counts=None, want_trace=False,
                         strategy=STRATEGY_AUTO):
        R, d = W.shape
        if k_blocks is None:
            k_blocks = d // c
        dev = W.device
        order = torch.empty(R, k_blocks, dtype=torch.int32, device=dev)
        loss = torch.empty(R, k_blocks, dtype=torch.float32, device=dev)
        W_out = torch.empty(R, d, dtype=torch.float32, device=dev)
        trace = torch.empty(R, k_blocks, d, dtype=torch.float32, device=dev) if want_trace else None
        need = c_size_t()
        rc = self.lib.obc_blocks_workspace_bytes(R, d, int(c), int(strategy), byref(need))
        if rc != OBC_OK:
            raise ObcError(rc, "obc_blocks_workspace_bytes")
        ws = self.workspace(need.value)
        self._ck(self.lib.obc_prune_blocks(
            self.h, _ptr(W, torch.float32), _ptr(Hinv, torch.float32), R, d, int(c), int(k_blocks),
            _ptr(stop_counts, torch.int32), _ptr(order), _ptr(loss), _ptr(W_out), _ptr(trace),
            int(strategy), c_void_p(ws.data_ptr()), ws.numel()))
        return dict(order=order, loss=loss, W=W_out, trace=trace)

    def obc_minmax_grid(self, W, bits, live=None, symmetric=False):
        R, d = W.shape
        maxq = (1 << bits) - 1
        delta = torch.empty(R, dtype=torch.float32, device=W.device)
        offset = torch.empty(R, dtype=torch.float32, device=W.device)
        self._ck(self.lib.obc_minmax_grid(self.h, _ptr(W, torch.float32), _ptr(live, torch.uint8), R, d,
                                          maxq, int(bool(symmetric)), _ptr(delta), _ptr(offset)))
        return delta, offset, maxq

    def obc_quant_rows(self, W, Hinv, delta, offset, maxq, live=None, strategy=STRATEGY_AUTO, out=None,
                       outliers=False):
        R, d = W.shape
        dev = W.device
        if out is None:
            out = {}
        order = out.get("order")
        if order is None:
            order = torch.full((R, d), -1, dtype=torch.int32, device=dev)
        loss = out.get("loss")
        if loss is None:
            loss = torch.zeros((R, d), dtype=torch.float32, device=dev)
        codes = out.get("codes")
        if codes is None:
            codes = torch.empty((R, d), dtype=torch.int32, device=dev)
        W_out = out.get("W")
        if W_out is None:
            W_out = torch.empty((R, d), dtype=torch.float32, device=dev)
        ws = self.workspace(self.rows_workspace_bytes(R, d, strategy))
        self._ck(self.lib.obc_quant_rows(
            self.h, _ptr(W, torch.float32), _ptr(Hinv, torch.float32), R, d, _ptr(delta, torch.float32),
            _ptr(offset, torch.float32), int(maxq), _ptr(live, torch.uint8), QUANT_OUTLIERS if outliers else 0,
            _ptr(order), _ptr(loss),
            _ptr(codes), _ptr(W_out), int(strategy), c_void_p(ws.data_ptr()), ws.numel()))
        return dict(order=order, loss=loss, codes=codes, W=W_out)

    def obc_global_select(self, loss, order, k):
        R, d = loss.shape
        counts = torch.empty(R, dtype=torch.int32, device=loss.device)
        mask = torch.empty((R, d), dtype=torch.uint8, device=loss.device)
        need = c_size_t()
        self.lib.obc_global_select_workspace_bytes(R, d, byref(need))
        ws = self.workspace(need.value)
        self._ck(self.lib.obc_global_select(self.h, _ptr(loss, torch.float32), _ptr(order, torch.int32), R, d,
                                            int(k), _ptr(counts), _ptr(mask), c_void_p(ws.data_ptr()),
                                            ws.numel()))
        return counts, mask

    def obc_global_select_static(self, loss, order, k, counts, mask):
        """The global step on the library's built-in scratch; every buffer is the caller's."""
        R, d = loss.shape
        self._ck(self.lib.obc_global_select_static(self.h, _ptr(loss, torch.float32), _ptr(order, torch.int32), R, d,
                                                   int(k), _ptr(counts, torch.int32), _ptr(mask, torch.uint8)))
        return counts, mask

    def obc_gather_trace(self, W, trace, counts):
        R, k_steps, d = trace.shape
        W_out = torch.empty((R, d), dtype=torch.float32, device=W.device)
        self._ck(self.lib.obc_gather_trace(self.h, _ptr(W, torch.float32), _ptr(trace, torch.float32),
                                           _ptr(counts, torch.int32), R, d, k_steps, _ptr(W_out)))
        return W_out

    def obc_reconstruct_rows(self, W, Hinv, mask, max_pruned=None, W_out=None):
        """Weights of a mask by the closed form; max_pruned bounds any row's pruned count (default: d)."""
        R, d = W.shape
        if max_pruned is None:
            max_pruned = d
        if W_out is None:
            W_out = torch.empty((R, d), dtype=torch.float32, device=W.device)
        need = c_size_t()
        rc = self.lib.obc_reconstruct_workspace_bytes(R, d, int(max_pruned), byref(need))
        if rc != OBC_OK:
            raise ObcError(rc, "obc_reconstruct_workspace_bytes")
        ws = self.workspace(need.value)
        self._ck(self.lib.obc_reconstruct_rows(self.h, _ptr(W, torch.float32), _ptr(Hinv, torch.float32),
                                               _ptr(mask, torch.uint8), R, d, int(max_pruned), _ptr(W_out),
                                               c_void_p(ws.data_ptr()), ws.numel()))
        return W_out
