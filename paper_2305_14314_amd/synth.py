"""Seeded synthetic inputs for the QLoRA linear-layer path.

This module only draws random tensors of the shapes and distributions of the
workloads (LLaMA-shaped linears, zero-centred normal weights, N(0,1) activations).
It contains none of the method's arithmetic: no codebook, no quantisation, no
matrix product.  Both the parity tests' oracle side and the HIP side consume the
same host arrays produced here.

Recipe: every tensor has its own 64-bit seed, splitmix64-mixed from a base seed
and the (config, layer, role) triple; values come from numpy's counter-based
Philox generator as fp32 standard normals scaled by sigma in fp32; 16-bit tensors
are then rounded to bf16 by torch's CPU cast.  Tensors too large to be worth
drawing on the host can be drawn on the device by torch's seeded generator
(`normal_f32_device`); a parity test then copies them back for the oracle.
"""
from __future__ import annotations

import numpy as np
import torch

BASE_SEED = 230514314
_MASK = (1 << 64) - 1

ROLES = {"W": 1, "L1": 2, "L2": 3, "X": 4, "dY": 5}


def _splitmix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def tensor_seed(config: int, layer: int, role: str, base: int = BASE_SEED) -> int:
    s = _splitmix64(base)
    for v in (config, layer, ROLES[role]):
        s = _splitmix64(s ^ (v & _MASK))
    return s


def normal_f32(shape, sigma: float, seed: int) -> np.ndarray:
    """fp32 array ~ N(0, sigma^2) (sigma is a standard deviation)."""
    rng = np.random.Generator(np.random.Philox(key=seed))
    out = rng.standard_normal(int(np.prod(shape)), dtype=np.float32)
    out *= np.float32(sigma)
    return out.reshape(shape)


def normal_f32_device(shape, sigma: float, seed: int, device="cuda") -> "torch.Tensor":
    """fp32 device tensor ~ N(0, sigma^2) from torch's seeded device generator."""
    g = torch.Generator(device=device)
    g.manual_seed(seed & ((1 << 63) - 1))
    out = torch.empty(shape, dtype=torch.float32, device=device)
    out.normal_(0.0, sigma, generator=g)
    return out


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> bf16 bit patterns (uint16), round to nearest even (torch CPU cast)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal_bf16(shape, sigma: float, seed: int) -> np.ndarray:
    return to_bf16_bits(normal_f32(shape, sigma, seed))


# (h, o) of the linears of one decoder block, in order q, k, v, o, gate, up, down.
def block_linears(d: int, ffn: int):
    return [(d, d)] * 4 + [(d, ffn)] * 2 + [(ffn, d)]


# The five workloads: index = position in the benchmark's config list.
CONFIGS = {
    0: dict(name="single-1024", linears=[(1024, 1024)], M=256, r=16, alpha=16, sigma_l=0.01),
    1: dict(name="llama7b-block", linears=block_linears(4096, 11008), M=8192, r=64, alpha=16, sigma_l=0.01),
    2: dict(name="llama13b-block", linears=block_linears(5120, 13824), M=8192, r=64, alpha=16, sigma_l=0.01),
    3: dict(name="llama65b-block", linears=block_linears(8192, 22016), M=4096, r=64, alpha=16, sigma_l=0.01),
    4: dict(name="llama65b-fewtoken", linears=block_linears(8192, 22016), M=(1, 4, 16), r=64, alpha=16,
            sigma_l=0.01),
}
SIGMA_W = 0.02


def make_layer(config: int, layer: int, M: int | None = None, h: int | None = None, o: int | None = None,
               r: int | None = None):
    """Host tensors of one linear: W fp32 (h, o); L1, L2, X, dY as bf16 bits; scalar s = alpha / r."""
    cfg = CONFIGS[config]
    hh, oo = cfg["linears"][layer]
    h = hh if h is None else h
    o = oo if o is None else o
    r = cfg["r"] if r is None else r
    if M is None:
        M = cfg["M"] if isinstance(cfg["M"], int) else cfg["M"][-1]
    out = dict(h=h, o=o, M=M, r=r, s=cfg["alpha"] / r)
    out["W"] = normal_f32((h, o), SIGMA_W, tensor_seed(config, layer, "W"))
    out["L1"] = normal_bf16((h, r), cfg["sigma_l"], tensor_seed(config, layer, "L1"))
    out["L2"] = normal_bf16((r, o), cfg["sigma_l"], tensor_seed(config, layer, "L2"))
    out["X"] = normal_bf16((M, h), 1.0, tensor_seed(config, layer, "X"))
    out["dY"] = normal_bf16((M, o), 1.0, tensor_seed(config, layer, "dY"))
    return out
