"""Drives the HIP library (through the C ABI binding) and the CPU oracle from one
description of a run, so that the parity tests feed both the same seeded inputs."""
from __future__ import annotations

import numpy as np

from oracle import hdet_oracle as O


def rel_err(a: np.ndarray, b: np.ndarray) -> float:
    """max_i |a_i - b_i| / max(|b_i|, rms(b)/32): a relative error with a floor.

    A pure ratio is meaningless for entries that cross zero.  The floor follows from the
    arithmetic: an update forms each entry from about four fp32 operations on operands of
    the tensor's scale (rms), so a correct fp32 kernel is off by up to 4 * 2^-24 * rms in
    absolute terms however small the result is after cancellation; that equals the 1e-5
    per-step bound exactly for an entry of size rms/42, so entries below rms/32 are
    measured against rms/32."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(b * b)))
    floor = max(rms / 32.0, 1e-30)
    return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), floor)))


def rel_err_detail(a: np.ndarray, b: np.ndarray, tol: float):
    """rel_err together with the indices of the entries that pass only thanks to the floor: those whose
    plain relative error |a_i - b_i| / |b_i| exceeds `tol` while the floored one does not."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.size == 0:
        return 0.0, np.zeros((0, a.ndim), dtype=np.int64)
    rms = float(np.sqrt(np.mean(b * b)))
    floor = max(rms / 32.0, 1e-30)
    diff = np.abs(a - b)
    floored = diff / np.maximum(np.abs(b), floor)
    needs = (diff > tol * np.abs(b)) & (floored <= tol)
    return float(np.max(floored)), np.argwhere(needs)


def norm_err(a, b) -> float:
    """||a - b|| / ||b|| over one tensor."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def elem_err(a, b) -> float:
    """max_i |a_i - b_i| / (|b_i| + rms(b)) over one tensor: the element-wise companion of norm_err for
    mixed-precision results.  Both sides round to bfloat16 at the same points, but a value that sits next
    to a rounding boundary may round the other way (one part in 256 of that value), and an entry of a
    gradient sums many such values, so single entries differ by a few percent of their own size or of the
    tensor's scale, whichever is larger -- far more than the tensor norm does.  A wrong entry is another
    matter: a missing row, a value taken from a neighbour or a stale buffer is off by about the tensor's
    scale and gives a ratio of 0.5 or more."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    if a.size == 0:
        return 0.0
    # the tensor's scale: rms over the entries that are not exactly zero (an embedding gradient has rows of zeros for
    # the tokens that do not occur; they must not shrink the scale of the rows that do)
    nz = int(np.count_nonzero(b))
    rms = float(np.sqrt(np.sum(b * b) / nz)) if nz else 0.0
    return float(np.max(np.abs(a - b) / (np.abs(b) + max(rms, 1e-30))))


# Bound on elem_err for mixed-precision gradients: see check_bf16_tensor.
ELEM_TOL_BF16 = 0.25
observed_elem_err = {}          # largest ratio seen per tag, for the record printed at the end of a run


def check_bf16_tensor(a, b, norm_tol: float, tag, elem_tol: float = ELEM_TOL_BF16):
    """One mixed-precision tensor against the oracle: its norm-wise error (what bf16 rounding noise adds
    up to over the tensor) and every single entry (elem_err), so that neither a wrong block nor a single
    wrong entry of the size of the tensor's scale passes."""
    ne, ee = norm_err(a, b), elem_err(a, b)
    key = str(tag)
    observed_elem_err[key] = max(observed_elem_err.get(key, 0.0), ee)
    assert ne <= norm_tol, (tag, "norm", ne)
    assert ee <= elem_tol, (tag, "element", ee)


def check_bf16_relu_matrix(a, b, rows: int, cols: int, norm_tol: float, tag):
    """A weight gradient of a hidden ReLU layer in mixed precision.  Here single entries cannot be held to
    elem_err: activations that round to the neighbouring bfloat16 move the next layer's pre-activations by
    up to about 1e-3, a unit that close to the kink passes its gradient on one side and not on the other (both
    are valid subgradients), and that switches one batch row's term of every entry in the unit's row on or
    off -- for a few entries that is most of their value.  What a kernel error looks like is different: a
    wrong row, column or block is off everywhere in it.  So: the norm-wise bound, the median error ratio of
    every row and of every column (a wrong one has a median of 0.5 or more), and the 99.9th percentile of all
    entries; the layers that no gate decides (the output layer, every bias) keep the entry-wise bound."""
    assert norm_err(a, b) <= norm_tol, (tag, "norm")
    a2, b2 = np.asarray(a, np.float64).reshape(rows, cols), np.asarray(b, np.float64).reshape(rows, cols)
    ratio = np.abs(a2 - b2) / (np.abs(b2) + max(float(np.sqrt(np.mean(b2 * b2))), 1e-30))
    row_med, col_med = float(np.max(np.median(ratio, axis=1))), float(np.max(np.median(ratio, axis=0)))
    q = float(np.quantile(ratio, 0.999))
    observed_elem_err[str(tag) + " q99.9"] = q
    assert row_med <= 0.1 and col_med <= 0.1, (tag, "row/column median", row_med, col_med)
    assert q <= ELEM_TOL_BF16, (tag, "99.9th percentile", q)


def check_bf16_mlp_gradients(g_dev, g_ref, widths, norm_tol: float, tag):
    """All tensors of a mixed-precision ReLU MLP gradient (flat layout W_1, b_1, W_2, b_2, ...)."""
    off, L = 0, len(widths) - 1
    for i in range(L):
        d_in, d_out = widths[i], widths[i + 1]
        w_dev, w_ref = g_dev[off:off + d_out * d_in], g_ref[off:off + d_out * d_in]
        if i == L - 1:
            check_bf16_tensor(w_dev, w_ref, norm_tol, (tag, i, "W"))
        else:
            check_bf16_relu_matrix(w_dev, w_ref, d_out, d_in, norm_tol, (tag, i, "W"))
        off += d_out * d_in
        # a bias gradient sums the batch rows of one unit: a switched term weighs as in the weight rows
        assert norm_err(g_dev[off:off + d_out], g_ref[off:off + d_out]) <= norm_tol, (tag, i, "b")
        if i == L - 1:
            check_bf16_tensor(g_dev[off:off + d_out], g_ref[off:off + d_out], norm_tol, (tag, i, "b"))
        off += d_out


def ulp_diff_f32(a, b) -> int:
    a = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    return int(np.max(np.abs(a - b))) if a.size else 0


def oracle_config(d: dict) -> O.Config:
    extra = [O.Channel(*ch) for ch in d.get("extra", [])]
    keys = ["n_replicas", "total_steps", "sync_interval", "warm_steps", "lr_max", "f_div", "f_final",
            "pct_start", "alpha", "autolr_enabled", "beta", "sigma", "optimizer", "momentum", "beta1",
            "beta2", "eps", "weight_decay", "grad_mode", "seed", "gamma_override", "constant_lr"]
    kw = {k: d[k] for k in keys if k in d}
    if "lambda_" in d:
        kw["lam"] = d["lambda_"]
    kw["autolr_enabled"] = bool(d.get("autolr_enabled", False))
    kw["constant_lr"] = bool(d.get("constant_lr", False))
    kw["reshuffle_every_sync"] = bool(d.get("reshuffle_every_sync", False))
    # shared_opt_state is a storage choice of the library: the oracle keeps one set of moments per
    # replica, which in shared-gradient AdamW are identical by construction
    return O.Config(extra=extra, group_ends=list(d.get("group_end", [])), **kw)


def library_config(d: dict, **model):
    import paper_2604_24708_amd as H
    kw = {k: v for k, v in d.items() if k not in ("extra", "group_end")}
    kw["autolr_enabled"] = int(bool(d.get("autolr_enabled", False)))
    kw["constant_lr"] = int(bool(d.get("constant_lr", False)))
    kw["reshuffle_every_sync"] = int(bool(d.get("reshuffle_every_sync", False)))
    kw["shared_opt_state"] = int(bool(d.get("shared_opt_state", False)))
    kw.update(model)
    if d.get("extra"):
        kw["extra"] = d["extra"]
    if d.get("group_end"):
        kw["group_end"] = d["group_end"]
    return H.make_config(**kw)


def check_state(st, orc: O.HDETOracle, scalar_rtol=0.0, lr_ulps=0):
    """Schedule state against the oracle.  With the interval losses handed over as fp64 numbers
    (scalar_rtol = 0, the default) everything is compared bit for bit: t, k, the permutations and the
    flags, but also the base values, velocities, hypergradients, softmax weights, gamma and the fp32
    rate table -- both sides evaluate Eq. 4-8 as the same sequence of IEEE double operations (ordered
    sums, no fused multiply-add, the exponential written out).  When the library reduces the losses
    itself in fp32 (model handles), its L_r differ from the oracle's fp64 ones in the seventh digit,
    and the scalars are compared to `scalar_rtol` instead (lr_ulps = None)."""
    n = orc.cfg.n_replicas
    assert st.t == orc.t and st.k == orc.k
    assert bool(st.controller_active) == orc.controller_active
    assert st.nonfinite == orc.nonfinite
    assert st.n_channels == orc.n_ch
    exact = scalar_rtol == 0.0

    def same(a, b, what, atol=0.0):
        if exact:
            assert float(a) == float(b), f"{what}: {float(a)!r} != {float(b)!r}"
        else:
            assert np.isclose(a, b, rtol=scalar_rtol, atol=atol), what

    for j in range(orc.n_ch):
        assert [st.perm[j][r] for r in range(n)] == orc.perm[j].tolist(), f"perm[{j}]"
        assert [st.rho[j][r] for r in range(n)] == [float(x) for x in orc.rho[j]], f"rho[{j}]"
        if j >= orc.n_lr or orc.controller_active:
            same(st.base[j], orc.base[j], f"base[{j}]", 1e-300)
        # Delta and v are differences of nearly equal terms of the size of the base value:
        # in the tolerance mode their error is measured against that size
        scale = scalar_rtol * abs(orc.base[j]) + 1e-24
        same(st.vel[j], orc.vel[j], f"vel[{j}]", scale)
        same(st.delta[j], orc.delta[j], f"delta[{j}]", scale)
    for r in range(n):
        same(st.w[r], orc.w[r], f"w[{r}]")
    assert st.gamma == orc.gamma
    if orc.t > 0:
        lr = np.array([st.lr[r] for r in range(n)], dtype=np.float32)
        if lr_ulps is not None:
            assert ulp_diff_f32(lr, orc.lr_used) <= lr_ulps
        else:       # base rate known only to scalar_rtol
            assert np.allclose(lr, orc.lr_used, rtol=2 * scalar_rtol, atol=0)
