"""ctypes binding of libhdet.so: the same names and arguments as include/hdet.h.

Argument marshalling only -- every step of the path runs in the library's HIP kernels.
PyTorch tensors are accepted where the C ABI takes device pointers (their data_ptr() is
passed); PyTorch is used for device memory and streams, nothing else.  There is no CPU
fallback: loading fails loudly if libhdet.so has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HDET_MAX_REPLICAS = 64
HDET_MAX_CH = 8
HDET_MAX_GROUPS = 4
HDET_MAX_LAYERS = 16

HDET_OK, HDET_EINVAL, HDET_ESTATE, HDET_EHIP, HDET_ENONFINITE = 0, -1, -2, -3, -4
HDET_SGDM, HDET_ADAMW = 0, 1
HDET_GRAD_SHARED, HDET_GRAD_PER_REPLICA = 0, 1
HDET_FP32, HDET_BF16_GEMM_FP32_MASTER = 0, 1
HDET_FLAT, HDET_MLP, HDET_TRANSFORMER = 0, 1, 2
HDET_CH_LR, HDET_CH_DROPOUT, HDET_CH_WD, HDET_CH_LABEL_SMOOTH, HDET_CH_ATTN_TEMP = 0, 1, 2, 3, 4
HDET_FUSE_CONVERGE = 1

EXPORTS = [
    "hdet_workspace_bytes", "hdet_create", "hdet_warm_init", "hdet_warm_init_noalloc", "hdet_forward_backward", "hdet_fanout_step", "hdet_train_step",
    "hdet_converge", "hdet_autolr_update", "hdet_get_state", "hdet_set_state",
    "hdet_set_launch_shape", "hdet_last_error", "hdet_destroy",
]


class hdet_channel(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("base", C.c_double),
                ("alpha", C.c_double), ("lambda_", C.c_double), ("lo", C.c_double),
                ("hi", C.c_double)]


class hdet_model_dims(C.Structure):
    _fields_ = [("n_params", C.c_int64), ("n_layers", C.c_int32),
                ("widths", C.c_int32 * (HDET_MAX_LAYERS + 1)), ("batch", C.c_int32),
                ("n_blocks", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ff", C.c_int32), ("seq_len", C.c_int32), ("vocab", C.c_int32)]


class hdet_config(C.Structure):
    _fields_ = [
        ("n_replicas", C.c_int32), ("sync_interval", C.c_int32),
        ("total_steps", C.c_int64), ("warm_steps", C.c_int64),
        ("lr_max", C.c_double), ("f_div", C.c_double), ("f_final", C.c_double),
        ("pct_start", C.c_double),
        ("constant_lr", C.c_int32), ("autolr_enabled", C.c_int32),
        ("alpha", C.c_double), ("beta", C.c_double), ("sigma", C.c_double),
        ("lambda_", C.c_double), ("gamma_override", C.c_double),
        ("optimizer", C.c_int32), ("grad_mode", C.c_int32),
        ("shared_opt_state", C.c_int32), ("reshuffle_every_sync", C.c_int32),
        ("momentum", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
        ("eps", C.c_double), ("weight_decay", C.c_double),
        ("precision", C.c_int32), ("model_kind", C.c_int32),
        ("dims", hdet_model_dims),
        ("n_extra_channels", C.c_int32), ("n_groups", C.c_int32),
        ("group_end", C.c_int64 * HDET_MAX_GROUPS),
        ("extra", hdet_channel * (HDET_MAX_CH - 1)),
        ("seed", C.c_uint64), ("stream", C.c_void_p),
    ]


class hdet_buffers(C.Structure):
    _fields_ = [("params_dev", C.c_void_p), ("grads_dev", C.c_void_p), ("opt_m_dev", C.c_void_p),
                ("opt_v_dev", C.c_void_p), ("params_bf16_dev", C.c_void_p),
                ("workspace_dev", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("plane_stride", C.c_int64)]


class hdet_state(C.Structure):
    _fields_ = [
        ("t", C.c_int64), ("k", C.c_int64), ("controller_active", C.c_int32),
        ("nonfinite", C.c_int32), ("n_replicas", C.c_int32), ("n_channels", C.c_int32),
        ("autolr_done", C.c_int32), ("reserved", C.c_int32),
        ("gamma", C.c_double),
        ("base", C.c_double * HDET_MAX_CH), ("vel", C.c_double * HDET_MAX_CH),
        ("delta", C.c_double * HDET_MAX_CH),
        ("w", C.c_double * HDET_MAX_REPLICAS), ("l_acc", C.c_double * HDET_MAX_REPLICAS),
        ("l_last", C.c_double * HDET_MAX_REPLICAS), ("l_step", C.c_float * HDET_MAX_REPLICAS),
        ("lr", C.c_float * HDET_MAX_REPLICAS),
        ("rho", (C.c_double * HDET_MAX_REPLICAS) * HDET_MAX_CH),
        ("perm", (C.c_int32 * HDET_MAX_REPLICAS) * HDET_MAX_CH),
    ]


LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhdet.so")
_lib = None


class HdetError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"hdet error {code}: {message}")
        self.code = code


def load_library(path: Optional[str] = None):
    """Loads libhdet.so (built by paper_2604_24708_amd.build) and declares the prototypes."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(f"{p} is missing: build it with `python -m paper_2604_24708_amd.build` "
                           "(there is no CPU fallback)")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 and must be the one that
    # libhdet.so binds to, or the library and the tensors it is handed would live in two
    # runtimes (the second one finds no device).  Importing torch first loads that copy.
    import torch  # noqa: F401
    lib = C.CDLL(p)
    vp = C.c_void_p
    lib.hdet_workspace_bytes.argtypes = [C.POINTER(hdet_config), C.c_int64, C.POINTER(C.c_size_t),
                                         C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.hdet_create.argtypes = [C.POINTER(hdet_config), C.POINTER(hdet_buffers), C.POINTER(vp)]
    lib.hdet_warm_init.argtypes = [vp, vp, C.c_double, C.c_uint64]
    lib.hdet_warm_init_noalloc.argtypes = [vp, vp, vp, C.c_int64, C.c_int64, C.c_int32, C.c_double, C.c_uint64, vp]
    lib.hdet_forward_backward.argtypes = [vp, vp, vp, C.POINTER(C.c_float)]
    lib.hdet_fanout_step.argtypes = [vp, vp, C.c_uint32]
    lib.hdet_train_step.argtypes = [vp, vp, vp, C.c_uint32, C.POINTER(C.c_float)]
    lib.hdet_converge.argtypes = [vp]
    lib.hdet_autolr_update.argtypes = [vp, C.POINTER(C.c_double)]
    lib.hdet_get_state.argtypes = [vp, C.POINTER(hdet_state)]
    lib.hdet_set_state.argtypes = [vp, C.POINTER(hdet_state)]
    lib.hdet_set_launch_shape.argtypes = [vp, C.c_int32, C.c_int32]
    lib.hdet_last_error.argtypes = [vp]
    lib.hdet_last_error.restype = C.c_char_p
    lib.hdet_destroy.argtypes = [vp]
    for name in EXPORTS:
        if name != "hdet_last_error":
            getattr(lib, name).restype = C.c_int
    if path is None:
        _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    """Device pointer of a torch tensor (or an int / None passed through)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _check(rc: int, handle=None):
    if rc != HDET_OK:
        msg = load_library().hdet_last_error(handle)
        raise HdetError(rc, msg.decode() if msg else "")


def make_config(**kw) -> hdet_config:
    """hdet_config with the paper's controller constants (beta 0.9, sigma 0.1, lambda 0.5)
    and the usual one-cycle factors as defaults; keyword names are the C field names
    (`lambda_` for lambda; `widths` and `extra` as Python sequences)."""
    cfg = hdet_config()
    cfg.f_div, cfg.f_final, cfg.pct_start = 25.0, 1e4, 0.3
    cfg.beta, cfg.sigma, cfg.lambda_ = 0.9, 0.1, 0.5
    cfg.gamma_override = -1.0
    cfg.momentum, cfg.beta1, cfg.beta2, cfg.eps = 0.9, 0.9, 0.999, 1e-8
    cfg.optimizer, cfg.grad_mode = HDET_ADAMW, HDET_GRAD_PER_REPLICA
    cfg.seed = 7
    widths = kw.pop("widths", None)
    extra = kw.pop("extra", None)
    group_end = kw.pop("group_end", None)
    for key in ("n_params", "batch", "n_blocks", "d_model", "n_heads", "d_ff", "seq_len", "vocab"):
        if key in kw:
            setattr(cfg.dims, key, kw.pop(key))
    if widths is not None:
        cfg.dims.n_layers = len(widths) - 1
        for i, wd in enumerate(widths):
            cfg.dims.widths[i] = wd
    if group_end is not None:
        cfg.n_groups = len(group_end)
        for g, end in enumerate(group_end):
            cfg.group_end[g] = end
    if extra is not None:
        cfg.n_extra_channels = len(extra)
        for j, ch in enumerate(extra):
            kind, base, alpha, lam, lo, hi = ch
            cfg.extra[j].kind, cfg.extra[j].base, cfg.extra[j].alpha = kind, base, alpha
            cfg.extra[j].lambda_, cfg.extra[j].lo, cfg.extra[j].hi = lam, lo, hi
    for key, val in kw.items():
        if not hasattr(cfg, key):
            raise TypeError(f"unknown hdet_config field {key}")
        setattr(cfg, key, val)
    return cfg


def hdet_workspace_bytes(cfg: hdet_config, plane_stride: int):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(load_library().hdet_workspace_bytes(C.byref(cfg), plane_stride, C.byref(a), C.byref(b),
                                               C.byref(c)))
    return a.value, b.value, c.value


def hdet_create(cfg: hdet_config, params, opt_m, opt_v=None, grads=None, params_bf16=None,
                workspace=None, plane_stride: Optional[int] = None):
    """Returns an opaque handle.  Tensors are [N, plane_stride] device tensors kept alive by
    the caller for the lifetime of the handle."""
    buf = hdet_buffers()
    buf.params_dev, buf.grads_dev = _ptr(params), _ptr(grads)
    buf.opt_m_dev, buf.opt_v_dev = _ptr(opt_m), _ptr(opt_v)
    buf.params_bf16_dev = _ptr(params_bf16)
    buf.workspace_dev = _ptr(workspace)
    buf.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    buf.plane_stride = plane_stride if plane_stride is not None else params.stride(0)
    h = C.c_void_p()
    _check(load_library().hdet_create(C.byref(cfg), C.byref(buf), C.byref(h)))
    return h


def hdet_warm_init(h, theta0, nu: float, seed: int):
    _check(load_library().hdet_warm_init(h, _ptr(theta0), nu, seed), h)


def hdet_warm_init_noalloc(theta0, params, params_bf16, n_params: int, plane_stride: int, n_replicas: int,
                           nu: float, seed: int, stream: Optional[int] = None):
    _check(load_library().hdet_warm_init_noalloc(_ptr(theta0), _ptr(params), _ptr(params_bf16), n_params, plane_stride,
                                                 n_replicas, nu, seed, stream))


def hdet_forward_backward(h, x, y, want_losses: bool = False):
    n = HDET_MAX_REPLICAS
    out = (C.c_float * n)() if want_losses else None
    _check(load_library().hdet_forward_backward(h, _ptr(x), _ptr(y), out), h)
    return out


def hdet_fanout_step(h, grads=None, flags: int = 0):
    _check(load_library().hdet_fanout_step(h, _ptr(grads), flags), h)


def hdet_train_step(h, x, y, flags: int = 0, want_losses: bool = False):
    out = (C.c_float * HDET_MAX_REPLICAS)() if want_losses else None
    _check(load_library().hdet_train_step(h, _ptr(x), _ptr(y), flags, out), h)
    return out


def hdet_converge(h):
    _check(load_library().hdet_converge(h), h)


def hdet_autolr_update(h, interval_losses: Optional[Sequence[float]] = None, n_replicas: Optional[int] = None):
    """`interval_losses`: None (the device-accumulated losses) or exactly N values; the C call reads
    N doubles, so the length is checked here against `n_replicas` or, if that is not given, against
    the handle's own count (one state query)."""
    arr = None
    if interval_losses is not None:
        n = n_replicas if n_replicas is not None else hdet_get_state(h).n_replicas
        if len(interval_losses) != n:
            raise ValueError(f"interval_losses has {len(interval_losses)} values, the handle has {n} replicas")
        arr = (C.c_double * n)(*[float(x) for x in interval_losses])
    _check(load_library().hdet_autolr_update(h, arr), h)


def hdet_get_state(h) -> hdet_state:
    st = hdet_state()
    _check(load_library().hdet_get_state(h, C.byref(st)), h)
    return st


def hdet_set_state(h, st: hdet_state):
    _check(load_library().hdet_set_state(h, C.byref(st)), h)


def hdet_set_launch_shape(h, variant: int = 0, blocks: int = 0):
    _check(load_library().hdet_set_launch_shape(h, variant, blocks), h)


def hdet_last_error(h=None) -> str:
    msg = load_library().hdet_last_error(h)
    return msg.decode() if msg else ""


def hdet_destroy(h):
    _check(load_library().hdet_destroy(h))
