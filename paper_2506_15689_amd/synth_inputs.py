"""Seeded synthetic inputs for the W4A4 rotated linear layer.

This module only draws random numbers and shapes them like the activations and
weights of LLaMA-style linears; it contains none of the method's arithmetic
(no rotation, no quantiser, no bias calibration).  Both the CPU oracle's tests
and the HIP path's tests/benchmark take their tensors from here, so the two
sides always see identical bits.

Activation model (paper Sec. 3.1, Eq. 1 and Sec. 3.2): a Gaussian bulk whose
channels have different means, plus a few outlier channels of much larger
amplitude.  The real model activations the paper measures on are not available;
these tensors stand in for them.

All tensors are generated on the CPU in fp32 from ``torch.Generator`` with a
fixed seed and then rounded to bf16, which is the storage type the layer sees.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 20250615


@dataclass(frozen=True)
class LayerConfig:
    """Shape and distribution parameters of one synthetic layer."""

    name: str
    index: int            # seed offset
    M: int                # tokens
    K: int                # input channels (= rotation size n)
    N: int                # output channels
    n_outlier: int        # number of outlier channels
    outlier_scale: float  # whole-channel multiplier of an outlier channel
    clip: float           # clip ratio applied to both range ends
    w_std: float          # std of the (already rotated) weights
    act: str = "gauss"    # "gauss": mu_c + N(0,1); "swiglu": silu(g)*u + mu_c
    mean_std: float = 0.5  # std of the per-channel mean offsets
    calib_tokens: int = 0  # >0: draw a separate calibration batch of this many tokens
    description: str = ""

    @property
    def rot_size(self) -> int:
        return self.K


CONFIGS: Dict[str, LayerConfig] = {
    c.name: c
    for c in [
        LayerConfig("C1", 1, 64, 1024, 1024, 8, 20.0, 0.9, 0.02,
                    description="small single linear (oracle finishes in seconds)"),
        LayerConfig("C2", 2, 2048, 4096, 12288, 16, 20.0, 0.9, 0.02,
                    description="LLaMA-2-7B-shaped fused QKV prefill"),
        LayerConfig("C3_M1", 3, 1, 4096, 4096, 16, 20.0, 0.9, 0.02, calib_tokens=2048,
                    description="decode, 1 token"),
        LayerConfig("C3_M4", 3, 4, 4096, 4096, 16, 20.0, 0.9, 0.02, calib_tokens=2048,
                    description="decode, 4 tokens"),
        LayerConfig("C3_M16", 3, 16, 4096, 4096, 16, 20.0, 0.9, 0.02, calib_tokens=2048,
                    description="decode, 16 tokens"),
        LayerConfig("C4", 4, 2048, 14336, 4096, 32, 30.0, 0.85, 0.02, act="swiglu",
                    description="LLaMA-3-8B-shaped MLP down projection (H_28 x H_512 rotation)"),
        LayerConfig("C5", 5, 4096, 8192, 28672, 32, 20.0, 0.9, 0.015,
                    description="LLaMA-2-70B-shaped gate/up prefill"),
    ]
}


@dataclass
class LayerInputs:
    """Tensors of one synthetic layer (all on the CPU)."""

    cfg: LayerConfig
    X: torch.Tensor                   # bf16 [M, K] activations, original basis
    X_calib: torch.Tensor             # bf16 [Mc, K] tokens the channel bias is calibrated on
    W_rot: torch.Tensor               # bf16 [N, K] weights, already in the rotated basis
    layer_bias: Optional[torch.Tensor] = None  # fp32 [N] or None
    outlier_channels: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))


def _draw_activations(cfg: LayerConfig, tokens: int, mu: torch.Tensor, chan_scale: torch.Tensor,
                      gen: torch.Generator) -> torch.Tensor:
    if cfg.act == "gauss":
        x = torch.randn(tokens, cfg.K, generator=gen, dtype=torch.float32)
    elif cfg.act == "swiglu":
        g = torch.randn(tokens, cfg.K, generator=gen, dtype=torch.float32)
        u = torch.randn(tokens, cfg.K, generator=gen, dtype=torch.float32)
        x = torch.nn.functional.silu(g) * u
    else:  # pragma: no cover - config table is static
        raise ValueError(f"unknown activation model {cfg.act!r}")
    x = (x + mu) * chan_scale        # outlier channels scale the whole channel, mean included
    return x.to(torch.bfloat16)


def make_layer(cfg: LayerConfig, *, M: Optional[int] = None, N: Optional[int] = None,
               seed: Optional[int] = None, with_layer_bias: bool = False) -> LayerInputs:
    """Draw the tensors of ``cfg``.  ``M``/``N`` override the token/output counts
    (used for sampled parity cases and sweeps); the draw order keeps X identical
    for a given seed whatever ``N`` is."""
    M = cfg.M if M is None else M
    N = cfg.N if N is None else N
    gen = torch.Generator(device="cpu")
    gen.manual_seed(BASE_SEED + cfg.index if seed is None else seed)

    mu = torch.randn(cfg.K, generator=gen, dtype=torch.float32) * cfg.mean_std
    perm = torch.randperm(cfg.K, generator=gen)
    outliers = perm[: cfg.n_outlier].sort().values
    chan_scale = torch.ones(cfg.K, dtype=torch.float32)
    chan_scale[outliers] = cfg.outlier_scale

    X = _draw_activations(cfg, M, mu, chan_scale, gen)
    if cfg.calib_tokens > 0:
        X_calib = _draw_activations(cfg, cfg.calib_tokens, mu, chan_scale, gen)
    else:
        X_calib = X
    W = (torch.randn(N, cfg.K, generator=gen, dtype=torch.float32) * cfg.w_std).to(torch.bfloat16)
    lb = None
    if with_layer_bias:
        lb = torch.randn(N, generator=gen, dtype=torch.float32) * 0.1
    return LayerInputs(cfg, X, X_calib, W, lb, outliers.numpy())


def make_tiny(M: int, K: int, N: int, *, seed: int = 0, n_outlier: int = 2, outlier_scale: float = 20.0,
              clip: float = 0.9, w_std: float = 0.02, act: str = "gauss") -> LayerInputs:
    """A small layer of arbitrary shape with the same recipe (for unit tests)."""
    cfg = LayerConfig(f"tiny_{M}x{K}x{N}", 0, M, K, N, min(n_outlier, K), outlier_scale, clip, w_std, act=act)
    return make_layer(cfg, seed=BASE_SEED + 1000 + seed)


# ---- storage-format helpers (bit reinterpretation only) ---------------------------------------

def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 torch tensor -> numpy uint16 array holding the same bits."""
    assert t.dtype == torch.bfloat16
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray) -> torch.Tensor:
    """numpy uint16 bit patterns -> bf16 torch tensor."""
    assert a.dtype == np.uint16
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)
