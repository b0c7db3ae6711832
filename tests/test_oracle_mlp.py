"""Pins for oracle/mlp_oracle.py: finite differences, an independent autograd library in
fp64, closed-form one-layer cases, bf16 rounding against the library's conversion."""
import math

import numpy as np
import pytest
import torch

from oracle import mlp_oracle as M
import hdet_inputs as I


def _case(widths, B, seed=0):
    th = I.mlp_init(1, widths, 2024 + seed)[0]
    x, y = I.mlp_batch(1, B, widths[0], 1234 + seed, 0, widths, 4321)
    return th, x[0], y[0]


@pytest.mark.parametrize("widths,B", [([64, 128, 10], 32), ([7, 5, 6, 3], 9), ([5, 4], 3)])
def test_gradient_by_central_differences(widths, B):
    th, x, y = _case(widths, B)
    th64 = th.astype(np.float64)

    def loss_at(v):
        lg = M.mlp_logits(v, x, widths)
        return M.softmax_xent(lg, y.astype(np.int64))[0]

    _, g = M.mlp_loss_and_grad(th, x, y, widths)
    rng = np.random.default_rng(1)
    idx = rng.choice(th.size, size=min(th.size, 60), replace=False)
    for i in idx:
        h = 1e-6
        e = np.zeros_like(th64); e[i] = h
        fd = (loss_at(th64 + e) - loss_at(th64 - e)) / (2 * h)
        assert g[i] == pytest.approx(fd, rel=2e-5, abs=2e-8)


@pytest.mark.parametrize("widths,B", [([64, 128, 10], 32), ([16, 24, 24, 8], 12)])
def test_matches_autograd_library_fp64(widths, B):
    th, x, y = _case(widths, B, seed=3)
    loss, g = M.mlp_loss_and_grad(th, x, y, widths)
    p = torch.tensor(th, dtype=torch.float64, requires_grad=True)
    h = torch.tensor(x, dtype=torch.float64)
    off = 0
    nl = len(widths) - 1
    for i in range(nl):
        w = p[off:off + widths[i + 1] * widths[i]].view(widths[i + 1], widths[i]); off += w.numel()
        b = p[off:off + widths[i + 1]]; off += widths[i + 1]
        h = torch.nn.functional.linear(h, w, b)
        if i + 1 < nl:
            h = torch.relu(h)
    ref = torch.nn.functional.cross_entropy(h, torch.tensor(y, dtype=torch.long))
    ref.backward()
    assert loss == pytest.approx(ref.item(), rel=1e-13)
    assert np.allclose(g, p.grad.numpy(), rtol=1e-6, atol=1e-9)


def test_one_layer_closed_form():
    # single linear layer, zero weights: softmax is uniform, loss = log C,
    # dW[c] = mean_b (1/C - [y_b = c]) x_b, db[c] = 1/C - freq(c)
    C, D, B = 5, 3, 8
    rng = np.random.default_rng(0)
    x = rng.standard_normal((B, D)).astype(np.float32)
    y = rng.integers(0, C, B).astype(np.int32)
    th = np.zeros(C * D + C, dtype=np.float32)
    loss, g = M.mlp_loss_and_grad(th, x, y, [D, C])
    assert loss == pytest.approx(np.log(C), rel=1e-14)
    onehot = np.eye(C)[y]
    dW = ((1.0 / C - onehot).T @ x.astype(np.float64)) / B
    assert np.allclose(g[:C * D].reshape(C, D), dW, rtol=1e-6, atol=1e-8)
    assert np.allclose(g[C * D:], 1.0 / C - onehot.mean(0), rtol=1e-6, atol=1e-8)


def test_xent_shift_invariance_and_gradient_sums_to_zero():
    rng = np.random.default_rng(5)
    lg = rng.standard_normal((6, 11)) * 30
    y = rng.integers(0, 11, 6)
    l1, d1 = M.softmax_xent(lg, y)
    l2, d2 = M.softmax_xent(lg + 1000.0, y)
    assert l1 == pytest.approx(l2, rel=1e-12) and np.allclose(d1, d2, atol=1e-15)
    assert np.allclose(d1.sum(axis=1), 0.0, atol=1e-15)


def test_round_bf16_matches_library_conversion():
    rng = np.random.default_rng(6)
    a = np.concatenate([rng.standard_normal(5000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895314e38],
                                 dtype=np.float32)])
    lib = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(M.round_bf16(a).view(np.uint32), lib.view(np.uint32))
    # ties go to even: 1 + 2^-8 is half-way between 1 and 1 + 2^-7
    assert M.round_bf16(np.array([1.00390625], np.float32))[0] == 1.0
    assert M.round_bf16(np.array([1.01171875], np.float32))[0] == np.float32(1.015625)


def test_bf16_mode_close_to_full_precision():
    widths, B = [32, 48, 10], 16
    th, x, y = _case(widths, B, seed=7)
    l0, g0 = M.mlp_loss_and_grad(th, x, y, widths)
    l1, g1 = M.mlp_loss_and_grad(th, x, y, widths, bf16=True)
    assert abs(l0 - l1) < 2e-2 and l0 != l1
    assert np.linalg.norm(g0 - g1) / np.linalg.norm(g0) < 3e-2


def test_label_smoothing_closed_forms():
    """eps = 1 makes the target uniform: the loss is the mean of (logsumexp - mean logit) and the
    gradient softmax - 1/C; uniform logits give log C for every eps; and the library's
    cross-entropy with label_smoothing agrees for intermediate eps."""
    rng = np.random.default_rng(5)
    z = rng.normal(size=(7, 11)); y = rng.integers(0, 11, size=7)
    loss, d = M.softmax_xent(z, y, 1.0)
    lse = np.log(np.exp(z).sum(axis=1))
    assert loss == pytest.approx(float((lse - z.mean(axis=1)).mean()), rel=1e-13)
    sm = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    assert np.allclose(d, (sm - 1.0 / 11) / 7, rtol=1e-12, atol=1e-15)
    for eps in (0.0, 0.3, 1.0):
        assert M.softmax_xent(np.zeros((4, 11)), y[:4], eps)[0] == pytest.approx(math.log(11), rel=1e-13)
    for eps in (0.05, 0.4):
        loss, d = M.softmax_xent(z, y, eps)
        t = torch.tensor(z, dtype=torch.float64, requires_grad=True)
        ref = torch.nn.functional.cross_entropy(t, torch.tensor(y, dtype=torch.long), label_smoothing=eps)
        ref.backward()
        assert loss == pytest.approx(ref.item(), rel=1e-13)
        assert np.allclose(d, t.grad.numpy(), rtol=1e-11, atol=1e-15)
        assert np.allclose(d.sum(axis=1), 0.0, atol=1e-16)
    # the loss is linear in eps between the two closed forms
    l0, l1, lh = M.softmax_xent(z, y, 0.0)[0], M.softmax_xent(z, y, 1.0)[0], M.softmax_xent(z, y, 0.5)[0]
    assert lh == pytest.approx(0.5 * (l0 + l1), rel=1e-13)
