"""Seeded synthetic layers shaped like the workloads of arxiv 2208.11580.

The paper measures on trained ResNet / YOLOv5 / BERT layers with ImageNet, COCO and
SQuAD calibration data (Sec. 6, "Objectives, Models & Datasets").  None of that is
available here, so these generators stand in for it: they reproduce the layer shapes
(3x3 convolutions with 64 / 256 / 512 channels unfold to d_col = 576 / 2304 / 4608;
BERT-base widths 768 / 3072; 128 sequences of 384 tokens) and the value structure
(correlated post-ReLU activations; LayerNorm-like activations with a few heavy
channels).

This module holds no arithmetic of the compression method itself: it is the one piece
both the oracle's tests and the HIP path's tests / benchmark may import.

Seeds: ``1000 * cfg + {0: W, 1: mixing matrix, 2: Z, 3: heavy-channel choice}``.
Tensors are generated with torch on the requested device; a given (device type, seed)
pair always yields the same values.
"""
from __future__ import annotations

import functools
import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class LayerSpec:
    name: str
    cfg: int          # seed family
    d_row: int
    d_col: int
    n_samples: int
    w_std: float
    kind: str         # "mix" | "relu_mix" | "layernorm_heavy"
    note: str = ""


SPECS = {
    # BASELINE configs[0]: tiny linear layer, parity / LDS-resident path
    "lin16x32": LayerSpec("lin16x32", 1, 16, 32, 256, 0.1, "mix"),
    # configs[1]: 3x3x64 conv unfolded
    "conv64x576": LayerSpec("conv64x576", 2, 64, 576, 50_000, 0.05, "relu_mix"),
    # configs[2]: 3x3x256 conv unfolded (OBQ 4 bit)
    "conv256x2304": LayerSpec("conv256x2304", 3, 256, 2304, 50_000, 0.03, "relu_mix"),
    # configs[3]: transformer linears on 768 input features
    "attn768x768": LayerSpec("attn768x768", 4, 768, 768, 49_152, 0.02, "layernorm_heavy"),
    "ffn3072x768": LayerSpec("ffn3072x768", 4, 3072, 768, 49_152, 0.02, "layernorm_heavy"),
    # the 768 x 3072 layer (d_col = 3072) named by the performance target
    "ffn768x3072": LayerSpec("ffn768x3072", 6, 768, 3072, 49_152, 0.02, "layernorm_heavy"),
    # configs[4]: 3x3x512 conv unfolded
    "conv512x4608": LayerSpec("conv512x4608", 5, 512, 4608, 100_000, 0.02, "relu_mix"),
}


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


@functools.lru_cache(maxsize=4)
def mixing_matrix(d: int, seed: int, cond: float = 1e3) -> torch.Tensor:
    """A = U diag(s) V^T with orthogonal U, V (QR of Gaussians) and s log-spaced 1 .. 1/cond.

    Built on the CPU in fp64 so that the same matrix is used whatever device the rest of the
    layer is generated on; returned as fp32 (cached: callers must not modify it).
    """
    g = _gen("cpu", seed)
    G1 = torch.randn(d, d, generator=g, dtype=torch.float64)
    G2 = torch.randn(d, d, generator=g, dtype=torch.float64)
    U, _ = torch.linalg.qr(G1)
    V, _ = torch.linalg.qr(G2)
    s = torch.logspace(0.0, -math.log10(cond), d, dtype=torch.float64)
    return ((U * s) @ V.T).to(torch.float32)


def make_layer(name: str, device="cpu", d_row=None, d_col=None, n_samples=None):
    """Return (W, X, spec): W is d_row x d_col fp32, X is d_col x N fp32, both on ``device``.

    ``d_row`` / ``d_col`` / ``n_samples`` shrink (or grow) the layer while keeping its recipe;
    tests use that to get sizes the oracle finishes in seconds.
    """
    spec = SPECS[name]
    R = spec.d_row if d_row is None else int(d_row)
    d = spec.d_col if d_col is None else int(d_col)
    N = spec.n_samples if n_samples is None else int(n_samples)
    dev = torch.device(device)
    base = 1000 * spec.cfg
    W = torch.randn(R, d, generator=_gen(dev, base + 0), device=dev, dtype=torch.float32) * spec.w_std
    Z = torch.randn(d, N, generator=_gen(dev, base + 2), device=dev, dtype=torch.float32)
    if spec.kind in ("mix", "relu_mix"):
        A = mixing_matrix(d, base + 1).to(dev)
        X = A @ Z
        if spec.kind == "relu_mix":
            X = torch.clamp_min(X, 0.0)
    elif spec.kind == "layernorm_heavy":
        # every token (column) standardised over the features, then ~1 % heavy channels x10
        X = (Z - Z.mean(dim=0, keepdim=True)) / Z.std(dim=0, unbiased=False, keepdim=True)
        n_heavy = max(1, round(0.01 * d))
        perm = torch.randperm(d, generator=_gen("cpu", base + 3))[:n_heavy].to(dev)
        X[perm, :] *= 10.0
    else:
        raise ValueError(spec.kind)
    return W.contiguous(), X.contiguous(), spec


def target_count(sparsity: float, d_row: int, d_col: int) -> int:
    """Number of weights to prune for a layer sparsity fraction (floor)."""
    return int(math.floor(sparsity * d_row * d_col + 1e-9))
