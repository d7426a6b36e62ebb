"""Seeded synthetic inputs shaped like the paper's LM-training workload.

Shared by the CPU oracle's tests and the GPU tests/benchmark so that both
sides see bit-identical inputs.  This module contains none of the method's
arithmetic: it only draws random tensors with the distributions the
benchmark configurations prescribe and rounds them to the I/O dtype.

Recipe (per configuration, seed = 20250516 + index): NumPy PCG64 stream,
draw order q, k, v, g, z, dO, all float32 in [B,H,L,d] / [B,H,L] order;
q, k, v, dO ~ N(0,1); w = g / ||g||_2 with g ~ N(0, I_d) per token and head;
beta = 2 * sigmoid(z), z ~ N(beta_mean, 1).  Each tensor is then rounded once
to the I/O dtype (bf16: round-to-nearest-even) and returned as float32 holding
exactly the rounded values.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20250516

# The five benchmark configurations (index = position in the list).
CONFIGS = [
    dict(name="cfg0_tiny_fp32", B=1, H=2, L=256, d=64, dtype="fp32", beta_mean=0.0),
    dict(name="cfg1_fwd_bf16_L2048_d64", B=8, H=16, L=2048, d=64, dtype="bf16", beta_mean=0.0),
    dict(name="cfg2_headline_L8192_d128", B=4, H=16, L=8192, d=128, dtype="bf16", beta_mean=0.0),
    dict(name="cfg3_bwd_bf16_L4096_d64", B=8, H=16, L=4096, d=64, dtype="bf16", beta_mean=0.0),
    dict(name="cfg4_long_L32768_d128", B=1, H=32, L=32768, d=128, dtype="bf16", beta_mean=2.0),
]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_inputs(B, H, L, d, dtype="bf16", seed=BASE_SEED, beta_mean=0.0, with_do=False):
    """Returns dict of float32 arrays q,k,v,w [B,H,L,d], beta [B,H,L] (+ dO)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    shp = (B, H, L, d)
    out = {}
    for name in ("q", "k", "v"):
        out[name] = rng.standard_normal(shp, dtype=np.float32)
    g = rng.standard_normal(shp, dtype=np.float32)
    nrm = np.sqrt((g.astype(np.float64) ** 2).sum(-1, keepdims=True))
    out["w"] = (g / np.maximum(nrm, 1e-30)).astype(np.float32)
    z = rng.standard_normal((B, H, L), dtype=np.float32) + np.float32(beta_mean)
    out["beta"] = (2.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)
    if with_do:
        out["dO"] = rng.standard_normal(shp, dtype=np.float32)
    if dtype == "bf16":
        out = {n: round_to_bf16(a) for n, a in out.items()}
    elif dtype != "fp32":
        raise ValueError(f"unknown dtype {dtype!r}")
    return out


def make_config(index: int, with_do: bool | None = None, **override):
    """Inputs of benchmark configuration ``index`` (optionally with B/H/L overridden)."""
    c = dict(CONFIGS[index])
    c.update(override)
    if with_do is None:
        with_do = index == 3
    return make_inputs(c["B"], c["H"], c["L"], c["d"], c["dtype"], BASE_SEED + index,
                       c["beta_mean"], with_do), c
