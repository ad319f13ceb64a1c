"""Seeded random fills (torch, any device).  No arithmetic of the method."""
from __future__ import annotations

import torch

_CHUNK = 1 << 26  # elements per Student-t chunk: bounds the scratch to ~1 GiB


def seed_for(base_seed: int, buffer_id: int, step: int = 0) -> int:
    """One 63-bit seed per (run seed, buffer, outer step), by integer mixing."""
    x = (base_seed * 0x9E3779B97F4A7C15 + buffer_id * 0xBF58476D1CE4E5B9
         + step * 0x94D049BB133111EB + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def _gen(t: torch.Tensor, seed: int) -> torch.Generator:
    g = torch.Generator(device=t.device)
    g.manual_seed(seed)
    return g


def fill_normal_(t: torch.Tensor, std: float, seed: int, mean: float = 0.0) -> torch.Tensor:
    """t ~ N(mean, std^2), in place."""
    return t.normal_(mean, std, generator=_gen(t, seed))


def fill_student_t_(t: torch.Tensor, scale: float, nu: int, seed: int) -> torch.Tensor:
    """t ~ scale * Student-t(nu), in place: z0 / sqrt(mean(z_1..z_nu ^2))."""
    g = _gen(t, seed)
    flat = t.view(-1)
    for lo in range(0, flat.numel(), _CHUNK):
        hi = min(lo + _CHUNK, flat.numel())
        z = torch.randn(nu + 1, hi - lo, generator=g, device=t.device, dtype=torch.float32)
        chi = z[1:].square().mean(dim=0).sqrt_()
        flat[lo:hi] = z[0].div_(chi).mul_(scale)
        del z, chi
    return t


def fill_bf16_normal_(t: torch.Tensor, std: float, seed: int) -> torch.Tensor:
    """bf16 gradients ~ N(0, std^2), in place (t has dtype bfloat16)."""
    assert t.dtype == torch.bfloat16
    g = _gen(t, seed)
    flat = t.view(-1)
    for lo in range(0, flat.numel(), _CHUNK):
        hi = min(lo + _CHUNK, flat.numel())
        flat[lo:hi] = torch.randn(hi - lo, generator=g, device=t.device,
                                  dtype=torch.float32).mul_(std).to(torch.bfloat16)
    return t
