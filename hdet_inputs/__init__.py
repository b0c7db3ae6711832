"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package holds input generation only -- initial parameters, batches, teacher labels,
synthetic gradients and losses.  It contains none of the method's arithmetic (no update,
converge, schedule or controller code) and imports neither the oracle nor the library.

The paper's workload is a proprietary news-feed dataset; every input here is synthetic
and merely has the shapes and value distributions the benchmark configurations name.
"""
from .flat import flat_theta0, flat_grads, flat_losses, device_normal_  # noqa: F401
from .mlp import mlp_param_count, mlp_init, mlp_teacher_labels, mlp_batch  # noqa: F401
from .transformer import transformer_shapes, transformer_param_count, transformer_init, zipf_tokens  # noqa: F401

SEED_DATA = 1234
SEED_TEACHER = 4321
SEED_INIT = 2024
SEED_PERM = 7
SEED_GRADS = 99
