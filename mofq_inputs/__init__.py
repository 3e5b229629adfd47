"""Seeded synthetic inputs for the MoFQ quantize-and-score path.

This module holds input recipes only: random tensors with the shapes and value
distributions of LLaMA linear layers, the clip-ratio tables handed to the
scale search, and the list of linear shapes of a decoder block.  It contains
none of the method's arithmetic (no scale, codec, error or select code), so
both the CPU oracle's tests and the HIP path's tests may draw from it.

The real LLaMA weights and calibration activations the paper samples
(Section 3.2, Section 5) are not available; these tensors stand in for them.
"""
from __future__ import annotations

import hashlib
import zlib
from typing import List, Tuple

import numpy as np
import torch

# Linear layers of one decoder block, [out_features, in_features]
# (the seven linears that Table 2's FP% counts: 32*7 = 224 for the 7B shape).
LLAMA_SHAPES = {
    "7b": dict(hidden=4096, ffn=11008, blocks=32),
    "65b": dict(hidden=8192, ffn=22016, blocks=80),
}
LINEAR_NAMES = ("q", "k", "v", "o", "gate", "up", "down")


def block_linear_shapes(model: str) -> List[Tuple[str, int, int]]:
    cfg = LLAMA_SHAPES[model]
    h, f = cfg["hidden"], cfg["ffn"]
    return [("q", h, h), ("k", h, h), ("v", h, h), ("o", h, h),
            ("gate", f, h), ("up", f, h), ("down", h, f)]


def model_linear_shapes(model: str) -> List[Tuple[int, str, int, int]]:
    out = []
    for b in range(LLAMA_SHAPES[model]["blocks"]):
        for name, o, i in block_linear_shapes(model):
            out.append((b, name, o, i))
    return out


def tensor_seed(config_id: int, block: int, linear: int, salt: int = 0) -> int:
    """Deterministic 31-bit seed from (config, block, linear)."""
    key = f"mofq:{config_id}:{block}:{linear}:{salt}".encode()
    return zlib.crc32(key) & 0x7FFFFFFF


def clip_ratios(n_clip: int, lo: float = 0.5, hi: float = 1.0) -> np.ndarray:
    """Clip-ratio table r_k = hi - (hi-lo)*k/(K-1), k = 0..K-1, descending from
    hi (least clipping first), both ends included; K = 1 gives {hi}.  Computed
    in double and rounded once to fp32.  The table is an input of the scale
    search: the caller hands the same array to the oracle and to the library."""
    if n_clip < 1:
        raise ValueError("n_clip must be >= 1")
    if n_clip == 1:
        return np.array([hi], dtype=np.float32)
    k = np.arange(n_clip, dtype=np.float64)
    return (hi - (hi - lo) * k / (n_clip - 1)).astype(np.float32)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def config0_weight(seed: int = 0, rows: int = 1024, cols: int = 1024,
                   device="cpu") -> torch.Tensor:
    """fp32 weight: entries N(0, 0.02^2); a Bernoulli(1e-3) subset multiplied
    by 10 as outliers."""
    g = _gen(seed, device)
    w = torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32) * 0.02
    mask = torch.rand(rows, cols, generator=g, device=device) < 1e-3
    return torch.where(mask, w * 10.0, w).contiguous()


def llama_like_weight(rows: int, cols: int, seed: int, dtype=torch.float16,
                      device="cpu", outlier_frac: float = 5e-4,
                      kappa: float = 4.0) -> torch.Tensor:
    """LLaMA-shaped weight: row sigma ~ U(0.01, 0.04); entries N(0, sigma^2);
    a Bernoulli(outlier_frac) subset replaced by sigma*kappa*T with
    T ~ Student-t(nu=3).  Drawn in fp32, rounded once to `dtype`."""
    g = _gen(seed, device)
    sigma = 0.01 + 0.03 * torch.rand(rows, 1, generator=g, device=device)
    w = torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32) * sigma
    mask = torch.rand(rows, cols, generator=g, device=device) < outlier_frac
    n_out = int(mask.sum().item())
    if n_out:
        z = torch.randn(4, n_out, generator=g, device=device, dtype=torch.float32)
        t3 = z[0] / torch.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0)
        rows_idx = mask.nonzero(as_tuple=True)[0]
        w[mask] = sigma[rows_idx, 0] * kappa * t3
    return w.to(dtype).contiguous()


def layer_outlier_frac(config_id: int, block: int, linear: int) -> float:
    """Share of heavy-tail entries of one layer in the tail-spread variant of a model-shaped set:
    log-uniform over [1.3e-5, 5e-3], fixed by (config, block, linear).  Layers then differ in how
    heavy their tails are; with this spread about one layer in eight is close enough to Gaussian
    for the integer format to win the 4-bit select, the others prefer the floating-point format."""
    digest = hashlib.sha256(f"mofq-tail:{config_id}:{block}:{linear}".encode()).digest()
    u = int.from_bytes(digest[:6], "little") / float(1 << 48)
    return float(1.3e-5 * (5e-3 / 1.3e-5) ** u)


def model_weight(config_id: int, block: int, linear: int, rows: int, cols: int,
                 dtype=torch.float16, device="cpu", tail_spread: bool = False) -> torch.Tensor:
    """The weight of linear `linear` of block `block` in the model-shaped set of a config:
    llama_like_weight with the layer's seed.  By default every layer has the same share of
    heavy-tail entries (0.05 %); with `tail_spread` the share differs per layer
    (layer_outlier_frac), which makes both outcomes of the 4-bit select occur in one set."""
    frac = layer_outlier_frac(config_id, block, linear) if tail_spread else 5e-4
    return llama_like_weight(rows, cols, seed=tensor_seed(config_id, block, linear), dtype=dtype,
                             device=device, outlier_frac=frac)


def outlier_channels(in_features: int, n: int = 6, seed: int = 1234) -> np.ndarray:
    """The fixed outlier columns of the activations: drawn once per
    in_features, reused for every layer and token."""
    rng = np.random.default_rng(seed + in_features)
    return np.sort(rng.choice(in_features, size=n, replace=False)).astype(np.int64)


def activations(tokens: int, in_features: int, seed: int, dtype=torch.bfloat16,
                device="cpu", n_outlier: int = 6, outlier_scale: float = 60.0
                ) -> torch.Tensor:
    """X [tokens, in_features]: N(0,1) with `n_outlier` fixed columns
    multiplied by `outlier_scale`, then rounded once to `dtype`."""
    g = _gen(seed, device)
    x = torch.randn(tokens, in_features, generator=g, device=device, dtype=torch.float32)
    cols = torch.as_tensor(outlier_channels(in_features, n_outlier), device=device)
    x[:, cols] *= outlier_scale
    return x.to(dtype).contiguous()


def to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an fp32/fp16/bf16 tensor to a host fp32 array."""
    return t.detach().to("cpu").to(torch.float32).contiguous().numpy()


def activation_batches(n_batches: int, tokens: int, in_features: int, seed: int,
                       dtype=torch.bfloat16, device="cpu", spread: float = 0.35) -> List[torch.Tensor]:
    """Batches of one layer's input for static calibration: activations() with a
    per-batch gain drawn log-normally (sigma = `spread`), so the largest magnitude
    differs from batch to batch and the calibrated scale is larger than most batches
    need."""
    g = _gen(seed, "cpu")
    gains = torch.exp(torch.randn(n_batches, generator=g) * spread)
    out = []
    for b in range(n_batches):
        x = activations(tokens, in_features, seed=seed * 1000 + b + 1, dtype=torch.float32, device=device)
        out.append((x * float(gains[b])).to(dtype).contiguous())
    return out

