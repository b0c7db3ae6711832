"""MLP case: parameters, Gaussian batches and labels from a fixed random teacher MLP."""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def mlp_param_count(widths: Sequence[int]) -> int:
    return sum(widths[i + 1] * widths[i] + widths[i + 1] for i in range(len(widths) - 1))


def _init_one(widths: Sequence[int], seed: int) -> np.ndarray:
    """Flat parameter vector [W_1 (d_out x d_in, row-major), b_1, W_2, b_2, ...] with every
    entry ~U(-1/sqrt(fan_in), 1/sqrt(fan_in))."""
    rng = np.random.Generator(np.random.Philox(seed))
    parts: List[np.ndarray] = []
    for i in range(len(widths) - 1):
        fan_in, fan_out = widths[i], widths[i + 1]
        bound = 1.0 / np.sqrt(fan_in)
        parts.append(rng.uniform(-bound, bound, size=fan_out * fan_in).astype(np.float32))
        parts.append(rng.uniform(-bound, bound, size=fan_out).astype(np.float32))
    return np.concatenate(parts)


def mlp_init(n: int, widths: Sequence[int], seed: int) -> np.ndarray:
    """[N, P] initial parameters, identical across replicas."""
    one = _init_one(widths, seed)
    return np.broadcast_to(one, (n, one.size)).copy()


def _teacher_forward(x: np.ndarray, widths: Sequence[int], flat: np.ndarray) -> np.ndarray:
    h = x.astype(np.float64)
    off = 0
    n_layers = len(widths) - 1
    for i in range(n_layers):
        fan_in, fan_out = widths[i], widths[i + 1]
        w = flat[off:off + fan_out * fan_in].reshape(fan_out, fan_in).astype(np.float64)
        off += fan_out * fan_in
        b = flat[off:off + fan_out].astype(np.float64)
        off += fan_out
        h = h @ w.T + b
        if i + 1 < n_layers:
            h = np.maximum(h, 0.0)
    return h


def mlp_teacher_labels(x: np.ndarray, teacher_widths: Sequence[int], seed: int,
                       gain: float = 4.0) -> np.ndarray:
    """labels = argmax of a fixed seeded random teacher MLP applied to x ([..., d_in]).
    The teacher's weights are scaled by `gain` so that its classes are reasonably balanced
    and separable."""
    flat = _init_one(teacher_widths, seed) * np.float32(gain)
    lead = x.shape[:-1]
    logits = _teacher_forward(x.reshape(-1, x.shape[-1]), teacher_widths, flat)
    return np.argmax(logits, axis=-1).astype(np.int32).reshape(lead)


def mlp_batch(n: int, batch: int, d_in: int, seed: int, step: int,
              teacher_widths: Sequence[int], teacher_seed: int,
              identical: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """x [N, B, d_in] ~N(0,1) fresh per (step, replica) -- or one batch repeated for all
    replicas if `identical` -- and teacher labels [N, B] int32."""
    rng = np.random.Generator(np.random.Philox(key=[seed, step]))
    if identical:
        one = rng.standard_normal((batch, d_in), dtype=np.float32)
        x = np.broadcast_to(one, (n, batch, d_in)).copy()
    else:
        x = rng.standard_normal((n, batch, d_in), dtype=np.float32)
    y = mlp_teacher_labels(x, teacher_widths, teacher_seed)
    return x, y
