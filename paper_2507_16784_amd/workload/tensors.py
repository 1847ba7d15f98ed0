"""Seeded random Q/K/V inputs (bf16), as the configurations describe them:
iid N(0, 1) entries times a stated scale.  Each block of rows is drawn from its
own torch CPU generator keyed by (seed, stream ids), so any slice can be
regenerated on its own.  A rotation of an iid Gaussian pair is again an iid
Gaussian pair, so stored keys are drawn directly rather than drawn and rotated.
"""
import numpy as np
import torch

from .rng import mix64


def _gen(seed: int, *ids: int) -> torch.Generator:
    s = mix64(seed)
    for i in ids:
        s = mix64(s ^ mix64(i + 0x51ED))
    g = torch.Generator(device="cpu")
    g.manual_seed(s & ((1 << 63) - 1))
    return g


def normal_bf16(seed: int, ids, shape, scale: float = 1.0) -> torch.Tensor:
    """bf16 tensor of N(0,1)*scale, generator keyed by (seed, *ids)."""
    x = torch.randn(shape, generator=_gen(seed, *ids), dtype=torch.float32)
    return (x * scale).to(torch.bfloat16)


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns (numpy, same shape)."""
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def from_bits(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> bf16 tensor."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)
