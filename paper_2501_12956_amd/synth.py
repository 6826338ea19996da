"""Seeded synthetic layer inputs (weights W and calibration activations X).

Stand-ins for LLaMA-shaped linear layers and for the calibration activations
(128 sequences x 2048 tokens) that the paper draws from a text corpus
(Section 4.1 Setup); neither is available here.  This module holds random
draws and scalings only - none of the solver's arithmetic - and is the one
module that both the CPU oracle's tests and the GPU path's tests use, so
that the two sides consume exactly the same stored values.

Each tensor has its own generator, seeded with ``seed`` plus a fixed
per-tensor offset, and is rounded to its storage dtype once.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    m: int            # output channels (rows of W)
    n: int            # input channels (columns of W, rows of X)
    p: int            # calibration tokens (columns of X)
    nbits: int
    iters: int
    w_dtype: torch.dtype
    x_dtype: torch.dtype
    w_kind: str       # "gauss_outlier" | "student_t"
    w_nu: int         # degrees of freedom for student_t
    x_kind: str       # "gauss" | "heavy"
    x_outlier_frac: float   # fraction of feature rows that are scaled (or count if >= 1)
    x_outlier_scale: float


CONFIGS = {
    # Tiny layer: the case the oracle finishes in seconds.
    "c1": LayerConfig("c1", 256, 512, 4096, 4, 10, torch.float32, torch.float32,
                      "gauss_outlier", 0, "gauss", 4, 20.0),
    # LLaMA-7B q_proj shape, 3-bit and 4-bit.
    "c2": LayerConfig("c2", 4096, 4096, 262144, 3, 10, torch.float16, torch.float16,
                      "student_t", 5, "gauss", 0.01, 20.0),
    "c3": LayerConfig("c3", 4096, 4096, 262144, 4, 10, torch.float16, torch.float16,
                      "student_t", 5, "gauss", 0.01, 20.0),
    # LLaMA-7B MLP pair.
    "c4a": LayerConfig("c4a", 11008, 4096, 262144, 4, 10, torch.float16, torch.float16,
                       "student_t", 5, "gauss", 0.01, 20.0),
    "c4b": LayerConfig("c4b", 4096, 11008, 262144, 4, 10, torch.float16, torch.float16,
                       "student_t", 5, "heavy", 0.005, 30.0),
    # Llama-3-70B down_proj shape, 4-bit and 3-bit (same W and X).
    "c5": LayerConfig("c5", 8192, 28672, 131072, 4, 10, torch.float16, torch.float16,
                      "student_t", 4, "heavy", 0.005, 30.0),
    "c5_3": LayerConfig("c5_3", 8192, 28672, 131072, 3, 10, torch.float16, torch.float16,
                        "student_t", 4, "heavy", 0.005, 30.0),
}

_W_OFFSET = 1
_WSCALE_OFFSET = 2
_WMASK_OFFSET = 3
_X_OFFSET = 4
_XROWS_OFFSET = 5


def _gen(seed, offset, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + offset)
    return g


def scaled_config(cfg: LayerConfig, m=None, n=None, p=None, nbits=None, iters=None) -> LayerConfig:
    """Same recipe at another size (used for parity cases that span a few
    tiles and a ragged tail)."""
    return LayerConfig(cfg.name + "_scaled", m or cfg.m, n or cfg.n, p or cfg.p,
                       nbits or cfg.nbits, iters or cfg.iters, cfg.w_dtype, cfg.x_dtype,
                       cfg.w_kind, cfg.w_nu, cfg.x_kind, cfg.x_outlier_frac, cfg.x_outlier_scale)


def make_weight(cfg: LayerConfig, seed=0, device="cpu", rows=None) -> torch.Tensor:
    """W (m, n) in cfg.w_dtype.

    gauss_outlier : N(0, 0.02^2), a Bernoulli(0.005) subset of entries x10.
    student_t     : per-row scale ~ LogNormal(-4, 0.3) times a Student-t
                    draw (nu degrees of freedom), generated as
                    z / sqrt(chi2_nu / nu).
    """
    m, n = cfg.m, cfg.n
    g = _gen(seed, _W_OFFSET, device)
    if cfg.w_kind == "gauss_outlier":
        W = torch.randn(m, n, generator=g, device=device, dtype=torch.float32) * 0.02
        gm = _gen(seed, _WMASK_OFFSET, device)
        mask = torch.rand(m, n, generator=gm, device=device) < 0.005
        W = torch.where(mask, W * 10.0, W)
    elif cfg.w_kind == "student_t":
        gs = _gen(seed, _WSCALE_OFFSET, device)
        scale = torch.exp(-4.0 + 0.3 * torch.randn(m, 1, generator=gs, device=device,
                                                   dtype=torch.float32))
        W = torch.empty(m, n, device=device, dtype=torch.float32)
        step = max(1, (1 << 24) // n)
        for r0 in range(0, m, step):
            r1 = min(m, r0 + step)
            z = torch.randn(r1 - r0, n, generator=g, device=device, dtype=torch.float32)
            chi = torch.zeros_like(z)
            for _ in range(cfg.w_nu):
                chi += torch.randn(r1 - r0, n, generator=g, device=device,
                                   dtype=torch.float32) ** 2
            W[r0:r1] = z / torch.sqrt(chi / cfg.w_nu)
        W *= scale
    else:
        raise ValueError(cfg.w_kind)
    W = W.to(cfg.w_dtype)
    if rows is not None:
        W = W[rows]
    return W.contiguous()


def outlier_feature_rows(cfg: LayerConfig, seed=0) -> torch.Tensor:
    """Indices of the feature rows of X that are scaled up."""
    k = int(cfg.x_outlier_frac) if cfg.x_outlier_frac >= 1 else int(round(cfg.x_outlier_frac * cfg.n))
    g = _gen(seed, _XROWS_OFFSET, "cpu")
    return torch.randperm(cfg.n, generator=g)[:k]


def make_activations(cfg: LayerConfig, seed=0, device="cpu", chunk_tokens=16384) -> torch.Tensor:
    """X (n, p) in cfg.x_dtype, features x tokens.

    gauss : N(0, 1).
    heavy : sign * |N(0,1)|^1.5 (post-activation-like heavy tails).
    A seeded subset of feature rows is multiplied by cfg.x_outlier_scale.
    Generated in token chunks so the float32 staging stays small.
    """
    n, p = cfg.n, cfg.p
    g = _gen(seed, _X_OFFSET, device)
    X = torch.empty(n, p, device=device, dtype=cfg.x_dtype)
    rows = outlier_feature_rows(cfg, seed).to(device)
    mult = torch.ones(n, 1, device=device, dtype=torch.float32)
    mult[rows] = cfg.x_outlier_scale
    for t0 in range(0, p, chunk_tokens):
        t1 = min(p, t0 + chunk_tokens)
        z = torch.randn(n, t1 - t0, generator=g, device=device, dtype=torch.float32)
        if cfg.x_kind == "heavy":
            z = torch.sign(z) * torch.abs(z) ** 1.5
        elif cfg.x_kind != "gauss":
            raise ValueError(cfg.x_kind)
        X[:, t0:t1] = (z * mult).to(cfg.x_dtype)
    return X


def make_layer(cfg: LayerConfig, seed=0, device="cpu"):
    """(W, X) for one configuration."""
    return make_weight(cfg, seed, device), make_activations(cfg, seed, device)
