"""Seeded synthetic inputs shared by the tests, the oracle timing and the benchmark.

This module holds no arithmetic of the compression method: it only draws the
fp32 messages (numpy Generator(PCG64(seed)), float64 math, cast to fp32) that
stand in for the paper's evaluation payloads (Sec. V-A "Datasets": SDRBench
fields, ResNet gradients and nccl-tests buffers, none of which ship here), and
turns a range-relative bound (the paper's REL, Sec. V-B) into an absolute one.
"""
import numpy as np


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def laplace(rng, n, b):
    """Laplace(0, b) by inverse CDF, float64."""
    u = rng.random(n) - 0.5
    return -b * np.sign(u) * np.log1p(-2.0 * np.abs(u))


def smooth_field(shape=(256, 64, 64), seed=1, noise=1e-3):
    """Sum of 4 random-phase sinusoids (amplitude 1, integer wavenumbers 1..8 per axis) + Gaussian noise."""
    rng = _rng(seed)
    grids = np.meshgrid(*[np.arange(s, dtype=np.float64) / s for s in shape], indexing="ij")
    f = np.zeros(shape, np.float64)
    for _ in range(4):
        k = rng.integers(1, 9, size=len(shape))
        phi = rng.random() * 2.0 * np.pi
        arg = sum(kk * g for kk, g in zip(k, grids))
        f += np.sin(2.0 * np.pi * arg + phi)
    f += rng.normal(0.0, noise, size=shape)
    return f.astype(np.float32).ravel()


def gradient_like(n, seed=2, b=1e-3, outlier_frac=0.01, outlier_b=1e-1, block=1 << 24):
    """Laplace(0,b) with a Bernoulli(outlier_frac) mask replaced by Laplace(0,outlier_b); generated in blocks."""
    rng = _rng(seed)
    out = np.empty(n, np.float32)
    for i0 in range(0, n, block):
        m = min(block, n - i0)
        x = laplace(rng, m, b)
        if outlier_frac > 0:
            mask = rng.random(m) < outlier_frac
            x[mask] = laplace(rng, int(mask.sum()), outlier_b)
        out[i0:i0 + m] = x.astype(np.float32)
    return out


def gaussian_random_field(N=512, seed=3, slope=-3.0):
    """Isotropic Gaussian random field N^3 with P(k) ~ k^slope, zero mean, unit variance."""
    rng = _rng(seed)
    white = rng.standard_normal((N, N, N)).astype(np.float32)
    F = np.fft.rfftn(white)
    del white
    kx = np.fft.fftfreq(N)[:, None, None] * N
    ky = np.fft.fftfreq(N)[None, :, None] * N
    kz = np.fft.rfftfreq(N)[None, None, :] * N
    k = np.sqrt(kx * kx + ky * ky + kz * kz)
    k[0, 0, 0] = 1.0
    amp = k ** (slope / 2.0)
    amp[0, 0, 0] = 0.0
    F *= amp
    f = np.fft.irfftn(F, s=(N, N, N), axes=(0, 1, 2))
    del F
    f -= f.mean()
    f /= f.std()
    return f.astype(np.float32).ravel()


def peer_messages(n, peers=8, seed0=40, b=1e-3):
    """Independent Laplace(0,b) gradient messages, one per simulated peer."""
    return [gradient_like(n, seed=seed0 + p, b=b, outlier_frac=0.0) for p in range(peers)]


def sweep_payload(kind, n, seed):
    """1-D payloads of the message-size sweep: 'uniform' in [-1,1], 'laplace'(0,1e-3), 'sinusoid'."""
    rng = _rng(seed)
    if kind == "uniform":
        return (rng.random(n) * 2.0 - 1.0).astype(np.float32)
    if kind == "laplace":
        return laplace(rng, n, 1e-3).astype(np.float32)
    if kind == "sinusoid":
        t = np.arange(n, dtype=np.float64) / n
        f = np.zeros(n, np.float64)
        for _ in range(4):
            k = rng.integers(1, 9)
            f += np.sin(2.0 * np.pi * k * t + rng.random() * 2.0 * np.pi)
        f += rng.normal(0.0, 1e-3, size=n)
        return f.astype(np.float32)
    raise ValueError(kind)


def abs_bound_from_rel(x, rel):
    """Range-relative bound -> absolute fp32 bound: rel * (max - min) over the whole message."""
    lo = float(np.min(x))
    hi = float(np.max(x))
    return float(np.float32(rel * (hi - lo)))
