"""HDET (Hyperparameter-Divergent Ensemble Training) step for one MI355X: hand-written HIP
kernels behind a C ABI (include/hdet.h, libhdet.so) and this thin ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import load_library, make_config, HdetError  # noqa: F401
