"""Seeded synthetic inputs for the ConvLinear4bit forward path.

This module only *draws numbers*: it holds none of the method's arithmetic (no
rotation, no quantiser, no GEMM).  Both the CPU oracle's tests and the GPU
tests / benchmark import it so that the two sides see the same bf16 bit
patterns.  Everything is numpy; tensors are returned as ``uint16`` arrays that
hold bf16 bit patterns (row-major, C-contiguous).

The value distributions stand in for FLUX.1-dev activations and weights, which
the paper measures on (Sec. 5.1 "Models", supplement Sec. B for the layer
shapes: 4608 tokens = 4096 image + 512 text, widths 3072 / 12288 / 15360) and
describes as carrying both column-wise (channel) and row-wise (token)
outliers (Sec. 1, Fig. 3-2 caption).  None of the paper's data is used.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

__all__ = [
    "f32_to_bf16_bits", "bf16_bits_to_f32", "LayerSpec", "make_activation",
    "make_weight", "make_bias", "make_layer", "CONFIGS", "NEXT_CONFIGS", "layers_of_config",
]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class LayerSpec:
    """One linear layer of a benchmark configuration: Y[M,N] = X[M,K] W[N,K]^T."""
    name: str
    M: int
    K: int
    N: int
    group: int = 16
    # activation recipe
    x_kind: str = "normal"            # "normal" or "halfnormal" (|N(0,1)|, GELU-like)
    x_col_frac: float = 0.01          # fraction of channels that are outliers
    x_col_range: Tuple[float, float] = (20.0, 100.0)   # log-uniform scale range
    x_row_frac: float = 0.005         # fraction of tokens that are outliers
    x_row_range: Tuple[float, float] = (10.0, 40.0)
    x_col_count: Optional[int] = None  # fixed count overrides the fraction
    x_row_count: Optional[int] = None
    # weight recipe
    w_std: float = 0.02
    w_col_count: int = 0              # outlier *input* channels of W
    w_col_scale: float = 20.0
    seed: int = 0


def _rng(seed: int, stream: str) -> np.random.Generator:
    # counter-based generator; one independent sub-stream per (seed, tensor name)
    key = np.frombuffer(stream.encode("utf8").ljust(16, b"\0")[:16], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed) ^ key[0], key[1]]))


def _log_uniform(rng: np.random.Generator, lo: float, hi: float, n: int) -> np.ndarray:
    if lo == hi:
        return np.full(n, lo, dtype=np.float32)
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n)).astype(np.float32)


def make_activation(spec: LayerSpec, rows: Optional[int] = None) -> np.ndarray:
    """X as bf16 bits, shape [M, K].  Base draw, channel scaling, token scaling, RNE to bf16."""
    M = spec.M if rows is None else rows
    rng = _rng(spec.seed, "X:" + spec.name)
    x = rng.standard_normal(size=(M, spec.K), dtype=np.float32)
    if spec.x_kind == "halfnormal":
        np.abs(x, out=x)
    ncol = spec.x_col_count if spec.x_col_count is not None else int(round(spec.x_col_frac * spec.K))
    nrow = spec.x_row_count if spec.x_row_count is not None else int(round(spec.x_row_frac * M))
    orng = _rng(spec.seed, "XO:" + spec.name)
    if ncol > 0:
        cols = orng.choice(spec.K, size=ncol, replace=False)
        x[:, cols] *= _log_uniform(orng, *spec.x_col_range, ncol)[None, :]
    if nrow > 0 and M > 0:
        rws = orng.choice(M, size=min(nrow, M), replace=False)
        x[rws, :] *= _log_uniform(orng, *spec.x_row_range, len(rws))[:, None]
    return f32_to_bf16_bits(x)


def make_weight(spec: LayerSpec, rows: Optional[int] = None) -> np.ndarray:
    """W as bf16 bits, shape [N, K]: N(0, w_std) with optional outlier input channels."""
    N = spec.N if rows is None else rows
    rng = _rng(spec.seed, "W:" + spec.name)
    w = rng.standard_normal(size=(N, spec.K), dtype=np.float32) * np.float32(spec.w_std)
    if spec.w_col_count > 0:
        orng = _rng(spec.seed, "WO:" + spec.name)
        cols = orng.choice(spec.K, size=spec.w_col_count, replace=False)
        w[:, cols] *= np.float32(spec.w_col_scale)
    return f32_to_bf16_bits(w)


def make_bias(spec: LayerSpec) -> np.ndarray:
    """Bias as bf16 bits, shape [N]: N(0, 0.1).  (The paper's Eq. 10 has no bias; the linear layers it replaces do.)"""
    rng = _rng(spec.seed, "B:" + spec.name)
    return f32_to_bf16_bits(rng.standard_normal(size=(spec.N,), dtype=np.float32) * np.float32(0.1))


def make_layer(spec: LayerSpec) -> Tuple[np.ndarray, np.ndarray]:
    return make_activation(spec), make_weight(spec)


def _flux(name, M, K, N, group=16, **kw) -> LayerSpec:
    return LayerSpec(name=name, M=M, K=K, N=N, group=group, **kw)


# The five benchmark configurations.  Config 1 is the small case; config 3's
# up-projection is the shape the headline metric is quoted on.
CONFIGS: Dict[str, Tuple[LayerSpec, ...]] = {
    "cfg1_tiny": (
        LayerSpec("tiny", M=256, K=1024, N=1024, group=16,
                  x_col_count=4, x_col_range=(50.0, 50.0),
                  x_row_count=2, x_row_range=(30.0, 30.0),
                  w_col_count=2, w_col_scale=20.0, seed=0),
    ),
    "cfg2_qkv": (_flux("qkv", 4608, 3072, 9216),),
    "cfg3_mlp": (
        _flux("mlp_up", 4608, 3072, 12288),
        _flux("mlp_down", 4608, 12288, 3072, x_kind="halfnormal"),
    ),
    "cfg4_group_sweep": tuple(
        _flux(f"square_g{g}", 4608, 3072, 3072, group=g) for g in (4, 16, 64, 256)
    ),
    "cfg5_hires": (
        _flux("hires_up", 16896, 3072, 12288),
        _flux("hires_down", 16896, 12288, 3072, x_kind="halfnormal"),
    ),
}

HEADLINE = CONFIGS["cfg3_mlp"][0]

# Shapes beyond the five configurations: the fused-width layer the paper itself profiles (supplement
# Sec. B: X [1 x 4608 x 15360], W [3072 x 15360]), run with a bias.
NEXT_CONFIGS: Dict[str, Tuple[LayerSpec, ...]] = {
    "n1_fused_width": (_flux("fused_out", 4608, 15360, 3072, x_kind="halfnormal"),),
    # the same layer at the group size the paper uses for its high-outlier layers (Sec. 5.2: N_0 = 1024)
    "n3_group_1024": (_flux("fused_out_g1024", 4608, 15360, 3072, group=1024, x_kind="halfnormal"),),
}


def layers_of_config(name: str) -> Tuple[LayerSpec, ...]:
    return CONFIGS[name]
