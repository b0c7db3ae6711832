"""CPU oracle: per-replica forward, mean cross-entropy and backward of an MLP.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

This is the "Forward + backward" of Algorithm 1 for one replica: loss l(theta_r, B_r) and
its gradient at the pre-update parameters.  The paper fixes no model; the benchmark
configurations name MLPs with Linear+bias layers, ReLU between layers and none after the
last, trained with mean cross-entropy over the batch.

Parameters live in one flat vector [W_1 (d_out x d_in row-major), b_1, W_2, b_2, ...].
Arithmetic is fp64.  With bf16=True the operands of every matrix product are rounded to
bfloat16 (round-to-nearest-even) where the mixed-precision path stores them in bf16:
the input batch, the weights, every hidden activation and every activation gradient;
the logits, the biases, the loss and the parameter gradients stay in full precision.

Pinned by tests/test_oracle_mlp.py (central finite differences, autograd of an
independent library in fp64, closed-form one-layer cases).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result returned as fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def split_params(flat: np.ndarray, widths: Sequence[int]) -> List[Tuple[np.ndarray, np.ndarray]]:
    out = []
    off = 0
    for i in range(len(widths) - 1):
        d_in, d_out = widths[i], widths[i + 1]
        w = flat[off:off + d_out * d_in].reshape(d_out, d_in)
        off += d_out * d_in
        b = flat[off:off + d_out]
        off += d_out
        out.append((w, b))
    assert off == flat.size
    return out


def softmax_xent(logits: np.ndarray, labels: np.ndarray, smoothing: float = 0.0) -> Tuple[float, np.ndarray]:
    """Mean over rows of the cross-entropy between the target distribution q and
    softmax(logits); returns (loss, dloss/dlogits).  q is the one-hot label for smoothing = 0;
    with label smoothing eps (one of the scalars Remark 1 names as explorable) it is the usual
    mixture q = (1 - eps) onehot + eps / C with the uniform distribution over the C classes."""
    z = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(z)
    s = e.sum(axis=1, keepdims=True)
    logp = z - np.log(s)
    n, c = logits.shape
    rows = np.arange(n)
    q = np.full((n, c), smoothing / c)
    q[rows, labels] += 1.0 - smoothing
    loss = float(-(q * logp).sum(axis=1).mean())
    d = (e / s - q) / n
    return loss, d


def mlp_loss_and_grad(flat: np.ndarray, x: np.ndarray, y: np.ndarray, widths: Sequence[int],
                      bf16: bool = False, info: dict = None, label_smoothing: float = 0.0,
                      relu_tie: Tuple[float, bool] = None) -> Tuple[float, np.ndarray]:
    """Loss and flat fp32 gradient for one replica.  x: [B, d_in], y: [B] int.

    If `info` is given, info["relu_margin"] receives the smallest |pre-activation| over all
    hidden units: the gradient is discontinuous where a pre-activation is zero, so a
    comparison against an implementation in another precision is only meaningful when this
    margin exceeds that implementation's rounding error.

    relu_tie = (tau, open): hidden units whose |pre-activation| is below tau -- ties at the kink of
    the ReLU as far as an fp32 implementation can tell -- are all taken as open (the unit passes its
    value and its gradient) or all as closed.  Both are valid subgradients; without the argument
    the sign of the fp64 pre-activation decides, as everywhere else."""
    def q(a):
        return round_bf16(a.astype(np.float32)).astype(np.float64) if bf16 else a.astype(np.float64)

    layers = split_params(flat, widths)
    n_layers = len(layers)
    acts = [q(x)]                                   # input of each layer (as the GEMM sees it)
    pre = []
    gates = []                                      # which hidden units pass
    for i, (w, b) in enumerate(layers):
        zi = acts[-1] @ q(w).T + b.astype(np.float64)
        pre.append(zi)
        if i + 1 < n_layers:
            gate = zi > 0.0
            if relu_tie is not None:
                gate = np.where(np.abs(zi) < relu_tie[0], bool(relu_tie[1]), gate)
            gates.append(gate)
            acts.append(q(np.where(gate, zi, 0.0)))
    if info is not None:
        info["relu_margin"] = min([float(np.min(np.abs(p))) for p in pre[:-1]] + [float("inf")])
    loss, dz = softmax_xent(pre[-1], y.astype(np.int64), label_smoothing)
    grads: List[np.ndarray] = [None] * (2 * n_layers)
    for i in range(n_layers - 1, -1, -1):
        w, _ = layers[i]
        dzq = q(dz)                                 # activation gradient as stored
        grads[2 * i] = (dzq.T @ acts[i]).astype(np.float32).ravel()
        grads[2 * i + 1] = dzq.sum(axis=0).astype(np.float32)
        if i > 0:
            da = dzq @ q(w)
            dz = da * gates[i - 1]
    return loss, np.concatenate(grads)


def mlp_logits(flat: np.ndarray, x: np.ndarray, widths: Sequence[int]) -> np.ndarray:
    layers = split_params(flat, widths)
    h = x.astype(np.float64)
    for i, (w, b) in enumerate(layers):
        h = h @ w.astype(np.float64).T + b.astype(np.float64)
        if i + 1 < len(layers):
            h = np.maximum(h, 0.0)
    return h
