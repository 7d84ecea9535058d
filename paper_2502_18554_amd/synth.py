"""Seeded synthetic inputs with the shape of the paper's workloads.

The paper measures on application datasets (Section 4.1, dataset table: RTM, NYX 512^3,
CESM-ATM, Hurricane).  They are not available here, so smooth synthetic fields of the same
shapes stand in for them.  This module only makes inputs; it contains none of the codec's
arithmetic.  Everything is float32 on the requested torch device, generated from a seed.
"""
import math

import torch


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def sinusoids(n=1 << 20, seed=0, device="cpu", noise=1e-3):
    """Sum of three unit sinusoids (periods 1e3, 1e4, 1e5 elements) plus Gaussian noise."""
    i = torch.arange(n, dtype=torch.float64, device=device)
    x = torch.zeros(n, dtype=torch.float64, device=device)
    for period in (1e3, 1e4, 1e5):
        x += torch.sin(2.0 * math.pi * i / period)
    x += noise * torch.randn(n, dtype=torch.float64, device=device, generator=_gen(seed, device))
    return x.to(torch.float32)


def power_law_field(shape=(512, 512, 512), seed=0, device="cpu", slope=3.0):
    """Gaussian random field with isotropic spectrum P(k) ~ k^-slope, mapped to [-1, 1].

    White noise -> real FFT -> amplitude * k^(-slope/2), mean removed -> inverse FFT ->
    affine map of [min, max] onto [-1, 1]; returned flattened in C order.
    """
    shape = tuple(int(s) for s in shape)
    w = torch.randn(shape, dtype=torch.float32, device=device, generator=_gen(seed, device))
    f = torch.fft.rfftn(w)
    del w
    k2 = None
    for ax, m in enumerate(shape):
        last = ax == len(shape) - 1
        k = (torch.fft.rfftfreq(m, device=device) if last else torch.fft.fftfreq(m, device=device)) * m
        view = [1] * len(shape)
        view[ax] = k.numel()
        k = (k.to(torch.float32) ** 2).reshape(view)
        k2 = k if k2 is None else k2 + k
    amp = torch.where(k2 > 0, k2.clamp_min(1e-30) ** (-slope / 4.0), torch.zeros_like(k2))
    del k2
    f *= amp
    del amp
    x = torch.fft.irfftn(f, s=shape)
    del f
    lo, hi = x.min(), x.max()
    x = (x - lo) * (2.0 / (hi - lo)) - 1.0
    return x.clamp_(-1.0, 1.0).reshape(-1).contiguous()


def hard_mix(n=1 << 28, seed=0, device="cpu"):
    """Stress input: smooth base + a step every 4096 values, 10 % exactly constant 32-blocks,
    and 1 % of the remaining values replaced by uniform spikes in [-1e3, 1e3]."""
    g = _gen(seed, device)
    i = torch.arange(n, dtype=torch.float64, device=device)
    x = torch.zeros(n, dtype=torch.float64, device=device)
    for period in (1e3, 1e4, 1e5):
        x += torch.sin(2.0 * math.pi * i / period)
    del i
    x = x.to(torch.float32)
    nseg = (n + 4095) // 4096
    steps = torch.rand(nseg, device=device, generator=g, dtype=torch.float32) * 2.0 - 1.0
    x += steps.repeat_interleave(4096)[:n]
    nb = (n + 31) // 32
    const_blk = torch.rand(nb, device=device, generator=g) < 0.10
    pad = nb * 32 - n
    xb = torch.nn.functional.pad(x, (0, pad)).reshape(nb, 32)
    xb = torch.where(const_blk[:, None], xb[:, :1].expand(-1, 32), xb)
    spike = (torch.rand(nb, 32, device=device, generator=g) < 0.01) & ~const_blk[:, None]
    vals = (torch.rand(nb, 32, device=device, generator=g, dtype=torch.float32) * 2.0 - 1.0) * 1e3
    xb = torch.where(spike, vals, xb)
    return xb.reshape(-1)[:n].contiguous()


def abs_bound(x, rel):
    """Absolute error bound for a value-range-relative bound: rel * (max - min), as float32."""
    return float(torch.tensor(rel * float(x.max() - x.min()), dtype=torch.float32))
