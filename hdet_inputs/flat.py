"""Flat-buffer case: N replicas x P fp32 parameters, synthetic per-replica gradients."""
from __future__ import annotations

import numpy as np


def flat_theta0(n: int, p: int, seed: int, std: float = 0.02) -> np.ndarray:
    """Initial parameters ~N(0, std^2), identical across replicas (data-parallel start)."""
    rng = np.random.Generator(np.random.Philox(seed))
    one = rng.standard_normal(p, dtype=np.float32) * np.float32(std)
    return np.broadcast_to(one, (n, p)).copy()


def flat_grads(n: int, p: int, seed: int, step: int, std: float = 1e-3) -> np.ndarray:
    """Per-replica gradients ~N(0, std^2); a pure function of (seed, step)."""
    rng = np.random.Generator(np.random.Philox(key=[seed, step]))
    return (rng.standard_normal((n, p), dtype=np.float32) * np.float32(std)).astype(np.float32)


def flat_losses(n: int, step: int, seed: int = 0) -> np.ndarray:
    """Injected per-replica losses for the flat case: 1 + 0.01*r, rotated over the replicas
    from step to step so that the controller sees a changing ranking."""
    base = 1.0 + 0.01 * np.arange(n, dtype=np.float64)
    rng = np.random.Generator(np.random.Philox(key=[seed, step]))
    jitter = 0.002 * rng.standard_normal(n)
    return np.roll(base, step % n) + jitter


def device_normal_(tensor, seed: int, std: float, mean: float = 0.0):
    """Fill a device tensor in place with N(mean, std^2) from torch's seeded generator.
    Used where the buffers (up to 8e9 elements) cannot be produced on the host."""
    import torch
    gen = torch.Generator(device=tensor.device)
    gen.manual_seed(seed)
    flat = tensor.view(-1)
    chunk = 1 << 28
    for start in range(0, flat.numel(), chunk):
        flat[start:start + chunk].normal_(mean, std, generator=gen)
    return tensor
