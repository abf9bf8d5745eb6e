"""Seeded random value generators for the synthetic gradient / replica tensors.

Values are drawn with torch generators on the requested device; whichever side draws them,
the identical bits are copied to the other side, so that the CPU oracle and the GPU library
always consume the same inputs.
"""
import math

import torch

SEED_BASE = 2107014990000
SHARED = 99  # "worker" id for draws shared by all workers (per-layer sigmas, the common base replica)


def seed_for(cfg, iteration=0, worker=0):
    return SEED_BASE + cfg * 10000 + iteration * 100 + worker


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def draw(dist, n, seed, device="cpu", scale=1.0, out=None):
    """n fp32 values of `dist` in {"normal", "student_t3", "laplace"} with the given scale.

    normal: N(0, scale^2); student_t3: scale * t(nu=3); laplace: Laplace(0, b=scale).
    """
    g = _gen(seed, device)
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=device)
    if dist == "normal":
        out.normal_(0.0, 1.0, generator=g)
        out.mul_(scale)
    elif dist == "student_t3":
        out.normal_(0.0, 1.0, generator=g)
        chi = torch.zeros_like(out)
        tmp = torch.empty_like(out)
        for _ in range(3):
            tmp.normal_(0.0, 1.0, generator=g)
            chi.addcmul_(tmp, tmp)
        chi.div_(3.0).sqrt_().clamp_(min=1e-20)
        out.div_(chi).mul_(scale)
        out.nan_to_num_(nan=0.0, posinf=1e30 * scale, neginf=-1e30 * scale)
    elif dist == "laplace":
        out.uniform_(-0.5, 0.5, generator=g)
        sign = torch.sign(out)
        mag = torch.log1p(-2.0 * out.abs().clamp_(max=0.5 - 1e-7))
        out.copy_(-scale * sign * mag)
    else:
        raise ValueError(dist)
    return out


def layer_sigmas(num_layers, seed, lo=-5.0, hi=-2.0):
    """Per-tensor standard deviations 10^U(lo,hi), drawn once on the CPU."""
    g = _gen(seed, "cpu")
    u = torch.rand(num_layers, generator=g, dtype=torch.float64)
    return [float(math.pow(10.0, lo + (hi - lo) * x)) for x in u]
