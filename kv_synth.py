"""Seeded synthetic KV-cache tensors.

Used by the tests, the smoke check and the benchmark to feed the SAME bytes to
the CPU oracle and to the GPU library.  This module holds no codec arithmetic:
it only draws random numbers and rounds them to BF16 / FP8-E5M2 with torch.

The tensors stand in for the real BF16 KV activations the paper measures on
(section 4.1 "Datasets and workloads"), which are not available here.  The
law is chosen so that the exponent statistics land in the regime of the paper's
Table 1: top-16 exponent coverage about 99.8 %, exponent entropy a little over
3 bits.

    x[t, h, d] = N(0, 1) * s[h, d],   s ~ LogNormal(0, 1) per channel (h, d)

Layout is [tokens, kv_heads, head_dim], contiguous, returned flattened as the
raw words (uint16 view for BF16 as a torch.int16 tensor, uint8 for E5M2).
"""
from __future__ import annotations

import torch

KV_HEADS = 8
HEAD_DIM = 128


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + int(stream)) & 0x7FFF_FFFF_FFFF_FFFF)
    return g


def channel_scales(seed: int, layer: int, kind: str, device="cpu") -> torch.Tensor:
    """LogNormal(0,1) scale per channel; V scales are half the K law."""
    g = _gen(seed, 2 * layer + (1 if kind == "V" else 0), device)
    z = torch.randn(KV_HEADS * HEAD_DIM, generator=g, device=device, dtype=torch.float32)
    s = torch.exp(z)
    if kind == "V":
        s = s * 0.5
    return s


def kv_values(tokens: int, seed: int, layer: int = 0, kind: str = "K", device="cpu") -> torch.Tensor:
    """fp32 values [tokens, KV_HEADS*HEAD_DIM] of the Gaussian-times-channel-scale law."""
    s = channel_scales(seed, layer, kind, device)
    g = _gen(seed, 1000 + 2 * layer + (1 if kind == "V" else 0), device)
    x = torch.randn(tokens, KV_HEADS * HEAD_DIM, generator=g, device=device, dtype=torch.float32)
    return x * s


def kv_bf16(tokens: int, seed: int, layer: int = 0, kind: str = "K", device="cpu") -> torch.Tensor:
    """BF16 KV tensor as flat int16 words (round to nearest even)."""
    return kv_values(tokens, seed, layer, kind, device).to(torch.bfloat16).view(torch.int16).reshape(-1)


def kv_e5m2(tokens: int, seed: int, layer: int = 0, kind: str = "K", device="cpu") -> torch.Tensor:
    """FP8 E5M2 KV tensor as flat uint8 words (round to nearest even of the same law)."""
    return kv_values(tokens, seed, layer, kind, device).to(torch.float8_e5m2).view(torch.uint8).reshape(-1)


def kv_e4m3(tokens: int, seed: int, layer: int = 0, kind: str = "K", device="cpu") -> torch.Tensor:
    """FP8 E4M3 KV tensor as flat uint8 words (round to nearest even of the same law; E4M3 has no
    infinities and the law stays far below its largest finite value, 448)."""
    return kv_values(tokens, seed, layer, kind, device).to(torch.float8_e4m3fn).view(torch.uint8).reshape(-1)


def kv_bf16_outliers(tokens: int, seed: int, layer: int = 0, device="cpu",
                     p_outlier: float = 0.005, p_zero: float = 0.001) -> torch.Tensor:
    """Escape-stress tensor: the base law, with a fraction p_outlier of the
    elements multiplied by 2^U{6..14} with a random sign, and a fraction p_zero
    replaced by exact zeros or BF16 subnormals."""
    x = kv_values(tokens, seed, layer, "K", device)
    g = _gen(seed, 5000 + layer, device)
    u = torch.rand(x.shape, generator=g, device=device)
    k = torch.randint(6, 15, x.shape, generator=g, device=device)
    sign = torch.randint(0, 2, x.shape, generator=g, device=device) * 2 - 1
    x = torch.where(u < p_outlier, x.abs() * torch.exp2(k.float()) * sign, x)
    w = x.to(torch.bfloat16).view(torch.int16)
    # zeros / subnormals: exponent field 0, random sign and mantissa (mantissa 0 half the time)
    u2 = torch.rand(x.shape, generator=g, device=device)
    mant = torch.randint(0, 128, x.shape, generator=g, device=device, dtype=torch.int16)
    mant = torch.where(torch.rand(x.shape, generator=g, device=device) < 0.5, torch.zeros_like(mant), mant)
    sgn = (torch.randint(0, 2, x.shape, generator=g, device=device, dtype=torch.int16) * -32768).to(torch.int16)
    w = torch.where(u2 < p_zero, sgn | mant, w)
    return w.reshape(-1)


def to_numpy_words(t: torch.Tensor):
    """Flat numpy view of the raw words (uint16 for int16 tensors, uint8 otherwise)."""
    import numpy as np

    a = t.detach().cpu().contiguous().numpy()
    if a.dtype == np.int16:
        a = a.view(np.uint16)
    return a.reshape(-1)
