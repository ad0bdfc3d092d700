"""Seeded synthetic layers and calibration activations (input generator only).

This module holds none of the method's arithmetic.  It produces weights and
activations with the shapes and value structure of the workloads: Gaussian
weights, Gaussian activations with a few outlier channels of much larger
magnitude and, for the LLM-shaped cases, a log-normal per-token scale.  Both
the GPU path and the CPU oracle are fed the SAME tensors (generated once, then
copied), never regenerated on the other side.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class LayerConfig:
    name: str
    d_out: int
    d_in: int
    n_tokens: int
    dtype: torch.dtype
    bits: int
    group_size: int
    damp: float
    act_order: bool
    n_outlier: int          # number of outlier channels
    outlier_factor: float
    token_sigma: float      # sigma of the log-normal per-token scale (0 = none)
    seed: int = 0


def _n_out(d_in: int, frac: float = 0.005) -> int:
    return int(round(frac * d_in))


CONFIGS = {
    # small fp32 layer, 4 outlier channels x20
    "c1": LayerConfig("c1", 256, 512, 1024, torch.float32, 4, 128, 0.01, False, 4, 20.0, 0.0),
    # Llama-style attention projection
    "c2": LayerConfig("c2", 4096, 4096, 128 * 2048, torch.bfloat16, 4, 128, 0.01, False, _n_out(4096), 30.0, 0.5),
    # Llama-style MLP up / gate and down projections
    "c3a": LayerConfig("c3a", 14336, 4096, 262144, torch.bfloat16, 4, 128, 0.01, False, _n_out(4096), 30.0, 0.5),
    "c3b": LayerConfig("c3b", 4096, 14336, 262144, torch.bfloat16, 4, 128, 0.01, False, _n_out(14336), 30.0, 0.5),
    # low-bit, group 64, activation ordering
    "c4_3bit": LayerConfig("c4_3bit", 4096, 14336, 262144, torch.bfloat16, 3, 64, 0.01, True, _n_out(14336), 30.0, 0.5),
    "c4_2bit": LayerConfig("c4_2bit", 4096, 14336, 262144, torch.bfloat16, 2, 64, 0.01, True, _n_out(14336), 30.0, 0.5),
    # 70B-class shapes
    "c5a": LayerConfig("c5a", 28672, 8192, 131072, torch.bfloat16, 3, 128, 0.01, False, _n_out(8192), 50.0, 0.5),
    "c5b": LayerConfig("c5b", 8192, 28672, 131072, torch.bfloat16, 3, 128, 0.01, False, _n_out(28672), 50.0, 0.5),
}


def c5_allocation(seed: int = 0):
    """The mixed-precision stand-in of the 70B-class configuration: six layer instances, three of each shape
    (28672 x 8192 and 8192 x 28672), whose bit-widths are a seeded shuffle of [2, 3, 4, 2, 3, 4] (3 bits on
    average).  The paper plans bit-widths with an integer program over real models (Sec. 4.1); this seeded
    allocation only reproduces the mix of widths such a plan hands to the layer-wise quantizer.
    Returns a list of LayerConfig, each instance with its own seed (distinct weights and activations)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 1000003 + 55)
    bits = [2, 3, 4, 2, 3, 4]
    order = torch.randperm(6, generator=g).tolist()
    shapes = ["c5a", "c5a", "c5a", "c5b", "c5b", "c5b"]
    out = []
    for i, name in enumerate(shapes):
        b = bits[order[i]]
        out.append(scaled(CONFIGS[name], name=f"{name}#{i % 3}_b{b}", bits=b, seed=seed + i))
    return out


def scaled(cfg: LayerConfig, d_out=None, d_in=None, n_tokens=None, **kw) -> LayerConfig:
    """A copy of cfg at other sizes (outlier count follows d_in unless given)."""
    d_in_new = d_in if d_in is not None else cfg.d_in
    fields = dict(cfg.__dict__)
    fields.update(d_out=d_out if d_out is not None else cfg.d_out, d_in=d_in_new,
                  n_tokens=n_tokens if n_tokens is not None else cfg.n_tokens)
    if d_in is not None and "n_outlier" not in kw:
        fields["n_outlier"] = max(1, _n_out(d_in_new)) if cfg.n_outlier > 0 else 0
    fields.update(kw)
    return LayerConfig(**fields)


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + stream)
    return g


def make_weight(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """W [d_out, d_in] ~ N(0, 0.02^2), rounded to cfg.dtype."""
    g = _gen(cfg.seed, 1, device)
    W = torch.empty((cfg.d_out, cfg.d_in), dtype=cfg.dtype, device=device)
    rows = max(1, (1 << 26) // cfg.d_in)
    for r0 in range(0, cfg.d_out, rows):
        r1 = min(cfg.d_out, r0 + rows)
        W[r0:r1] = (torch.randn((r1 - r0, cfg.d_in), generator=g, device=device, dtype=torch.float32) * 0.02).to(cfg.dtype)
    return W


def channel_scale(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """Per-channel multiplier: outlier_factor on a seeded random subset of n_outlier channels, else 1."""
    g = _gen(cfg.seed, 2, "cpu")
    ch = torch.ones(cfg.d_in, dtype=torch.float32)
    if cfg.n_outlier > 0:
        idx = torch.randperm(cfg.d_in, generator=g)[: cfg.n_outlier]
        ch[idx] = cfg.outlier_factor
    return ch.to(device)


def make_activations(cfg: LayerConfig, device="cpu", n_tokens=None) -> torch.Tensor:
    """X [n_tokens, d_in] = token_scale[:, None] * channel_scale[None, :] * N(0, 1), rounded to cfg.dtype."""
    n = cfg.n_tokens if n_tokens is None else n_tokens
    g = _gen(cfg.seed, 3, device)
    gt = _gen(cfg.seed, 4, device)
    ch = channel_scale(cfg, device)
    X = torch.empty((n, cfg.d_in), dtype=cfg.dtype, device=device)
    rows = max(1, (1 << 26) // cfg.d_in)
    for t0 in range(0, n, rows):
        t1 = min(n, t0 + rows)
        blk = torch.randn((t1 - t0, cfg.d_in), generator=g, device=device, dtype=torch.float32)
        if cfg.token_sigma > 0:
            tok = torch.exp(cfg.token_sigma * torch.randn((t1 - t0, 1), generator=gt, device=device, dtype=torch.float32))
            blk = blk * tok
        X[t0:t1] = (blk * ch[None, :]).to(cfg.dtype)
    return X


def make_perturbed_activations(cfg: LayerConfig, X: torch.Tensor, rel_noise: float = 0.05) -> torch.Tensor:
    """X_hat = X * (1 + rel_noise * N(0, 1)), rounded to cfg.dtype: a stand-in for the activations that reach a layer
    once the layers before it have been quantized (same shape and outlier structure as X, a few percent off)."""
    g = _gen(cfg.seed, 5, X.device)
    Xh = torch.empty_like(X)
    rows = max(1, (1 << 26) // cfg.d_in)
    for t0 in range(0, X.shape[0], rows):
        t1 = min(X.shape[0], t0 + rows)
        z = torch.randn((t1 - t0, cfg.d_in), generator=g, device=X.device, dtype=torch.float32)
        Xh[t0:t1] = (X[t0:t1].to(torch.float32) * (1.0 + rel_noise * z)).to(cfg.dtype)
    return Xh
