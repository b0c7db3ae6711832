"""Pins for oracle/transformer_oracle.py: autograd of an independent library in fp64, central
finite differences, dropout-mask statistics."""
import math

import numpy as np
import pytest
import torch

import hdet_inputs as I
from oracle import transformer_oracle as T

CFG = dict(n_blocks=2, d_model=16, n_heads=4, d_ff=40, seq_len=6, vocab=29)


def _case(cfg=CFG, B=3, seed=0):
    th = I.transformer_init(1, cfg, 2024 + seed, std=0.2, bias_std=0.1)[0]
    ids, tgt = I.zipf_tokens(1, B, cfg["seq_len"], cfg["vocab"], 1234 + seed, 0)
    return th, ids[0], tgt[0]


def torch_reference(th, ids, tgt, cfg, keep=None, p_drop=0.0, label_smoothing=0.0, attn_temp=1.0):
    """The same model written with the library's own layers and autograd (fp64)."""
    F = torch.nn.functional
    d, nh, S, L = cfg["d_model"], cfg["n_heads"], cfg["seq_len"], cfg["n_blocks"]
    dh = d // nh
    flat = torch.tensor(th, dtype=torch.float64, requires_grad=True)
    P, off = {}, 0
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape)); P[name] = flat[off:off + k].view(shape); off += k
    B = ids.shape[0]
    x = P["tok_emb"][torch.tensor(ids, dtype=torch.long)] + P["pos_emb"][None, :, :]
    for l in range(L):
        h = F.layer_norm(x, (d,), P[f"ln1_g.{l}"], P[f"ln1_b.{l}"], eps=1e-5)
        qkv = F.linear(h, P[f"w_qkv.{l}"], P[f"b_qkv.{l}"]).view(B, S, 3, nh, dh).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=True, scale=1.0 / (math.sqrt(dh) * attn_temp))
        o = F.linear(a.permute(0, 2, 1, 3).reshape(B, S, d), P[f"w_o.{l}"], P[f"b_o.{l}"])
        if keep is not None:
            o = o * torch.tensor(keep[2 * l].reshape(B, S, d), dtype=torch.float64) / (1 - p_drop)
        x = x + o
        h = F.layer_norm(x, (d,), P[f"ln2_g.{l}"], P[f"ln2_b.{l}"], eps=1e-5)
        y = F.linear(F.gelu(F.linear(h, P[f"w_1.{l}"], P[f"b_1.{l}"]), approximate="tanh"), P[f"w_2.{l}"], P[f"b_2.{l}"])
        if keep is not None:
            y = y * torch.tensor(keep[2 * l + 1].reshape(B, S, d), dtype=torch.float64) / (1 - p_drop)
        x = x + y
    logits = F.linear(F.layer_norm(x, (d,), P["lnf_g"], P["lnf_b"], eps=1e-5), P["w_head"], P["b_head"])
    loss = F.cross_entropy(logits.view(B * S, -1), torch.tensor(tgt.reshape(-1), dtype=torch.long),
                           label_smoothing=label_smoothing)
    loss.backward()
    return loss.item(), flat.grad.numpy()


def test_layout_matches_input_generator():
    assert T.layout(CFG) == I.transformer_shapes(CFG)
    big = dict(n_blocks=6, d_model=512, n_heads=8, d_ff=2048, seq_len=256, vocab=32000)
    assert I.transformer_param_count(big) == 51_846_400        # 6-layer d=512 case, untied head


def test_matches_autograd_library_fp64():
    th, ids, tgt = _case()
    loss, g = T.loss_and_grad(th, ids, tgt, CFG)
    ref_loss, ref_g = torch_reference(th, ids, tgt, CFG)
    assert loss == pytest.approx(ref_loss, rel=1e-12)
    assert np.allclose(g, ref_g, rtol=2e-6, atol=1e-9)
    assert np.count_nonzero(g) > 0.9 * g.size


def test_gradient_by_central_differences():
    th, ids, tgt = _case(seed=1)
    th64 = th.astype(np.float64)

    def loss_at(v):
        lg = T.logits_only(v, ids, CFG)
        z = lg - lg.max(axis=1, keepdims=True)
        lp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
        return -lp[np.arange(lg.shape[0]), tgt.reshape(-1)].mean()

    loss, g = T.loss_and_grad(th, ids, tgt, CFG)
    assert loss == pytest.approx(loss_at(th64), rel=1e-12)
    rng = np.random.default_rng(3)
    for i in rng.choice(th.size, size=80, replace=False):
        e = np.zeros_like(th64); e[i] = 1e-5
        fd = (loss_at(th64 + e) - loss_at(th64 - e)) / 2e-5
        assert g[i] == pytest.approx(fd, rel=5e-5, abs=1e-8)


def test_dropout_matches_autograd_with_the_same_mask():
    th, ids, tgt = _case(seed=2)
    dp = dict(p=0.25, seed=77, step=5, replica=3)
    B, S, d = ids.shape[0], CFG["seq_len"], CFG["d_model"]
    keep = [T.dropout_keep(77, 5, 3, site, B * S * d, 0.25) for site in range(2 * CFG["n_blocks"])]
    loss, g = T.loss_and_grad(th, ids, tgt, CFG, dropout=dp)
    ref_loss, ref_g = torch_reference(th, ids, tgt, CFG, keep=keep, p_drop=0.25)
    assert loss == pytest.approx(ref_loss, rel=1e-12)
    assert np.allclose(g, ref_g, rtol=2e-6, atol=1e-9)
    l0, _ = T.loss_and_grad(th, ids, tgt, CFG)
    assert l0 != loss


def test_dropout_mask_statistics_and_determinism():
    n = 40000
    for p in (0.1, 0.5):
        k = T.dropout_keep(1, 2, 3, 4, n, p)
        assert abs(k.mean() - (1 - p)) < 4 * math.sqrt(p * (1 - p) / n)
    a = T.dropout_keep(1, 2, 3, 4, 1000, 0.3)
    assert np.array_equal(a, T.dropout_keep(1, 2, 3, 4, 1000, 0.3))
    for other in [(2, 2, 3, 4), (1, 3, 3, 4), (1, 2, 4, 4), (1, 2, 3, 5)]:
        assert not np.array_equal(a, T.dropout_keep(*other, 1000, 0.3))
    assert T.dropout_keep(1, 2, 3, 4, 100, 0.0).all()
    # prefix property: the mask of element e does not depend on n
    assert np.array_equal(a[:37], T.dropout_keep(1, 2, 3, 4, 37, 0.3))


def test_gelu_and_layernorm_closed_forms():
    z = np.linspace(-4, 4, 41)
    assert np.allclose(T.gelu_tanh(z), torch.nn.functional.gelu(torch.tensor(z), approximate="tanh").numpy(), rtol=1e-12)
    h = 1e-6
    assert np.allclose(T.gelu_tanh_grad(z), (T.gelu_tanh(z + h) - T.gelu_tanh(z - h)) / (2 * h), rtol=1e-6, atol=1e-9)
    x = np.random.default_rng(0).standard_normal((5, 8))
    y, xhat, rstd = T.layer_norm(x, np.ones(8), np.zeros(8))
    assert np.allclose(y.mean(axis=1), 0, atol=1e-12) and np.allclose((y ** 2).mean(axis=1), 1, rtol=1e-4)


def test_bf16_mode_is_close_and_different():
    th, ids, tgt = _case(seed=4)
    l0, g0 = T.loss_and_grad(th, ids, tgt, CFG)
    l1, g1 = T.loss_and_grad(th, ids, tgt, CFG, bf16=True)
    assert l0 != l1 and abs(l0 - l1) < 3e-2
    assert np.linalg.norm(g0 - g1) / np.linalg.norm(g0) < 5e-2


def test_zipf_tokens():
    ids, tgt = I.zipf_tokens(2, 4, 64, 1000, 5, 0)
    assert ids.shape == (2, 4, 64) and np.array_equal(ids[..., 1:], tgt[..., :-1])
    big, _ = I.zipf_tokens(1, 64, 256, 32000, 5, 1)
    counts = np.bincount(big.ravel(), minlength=32000)
    assert counts[0] > counts[1] > counts[3] > counts[15]          # rank-frequency decreasing
    w = 1.0 / np.arange(1, 32001) ** 1.1
    assert abs(counts[0] / big.size - w[0] / w.sum()) < 0.01


def test_label_smoothing_and_attention_temperature_match_autograd_library():
    """Remark 1's further scalars: the library's own label_smoothing and attention scale."""
    th, ids, tgt = _case(seed=4)
    for eps, tau in [(0.1, 1.0), (0.0, 1.7), (0.25, 0.6)]:
        loss, g = T.loss_and_grad(th, ids, tgt, CFG, label_smoothing=eps, attn_temp=tau)
        ref_loss, ref_g = torch_reference(th, ids, tgt, CFG, label_smoothing=eps, attn_temp=tau)
        assert loss == pytest.approx(ref_loss, rel=1e-12)
        assert np.allclose(g, ref_g, rtol=2e-6, atol=1e-9)
    base, g0 = T.loss_and_grad(th, ids, tgt, CFG)
    assert T.loss_and_grad(th, ids, tgt, CFG, label_smoothing=0.1)[0] != base
    assert T.loss_and_grad(th, ids, tgt, CFG, attn_temp=1.7)[0] != base


def test_attention_temperature_equals_rescaled_query_weights():
    """softmax(q.k / (sqrt(d_h) tau)) is what dividing the query projection by tau gives:
    same loss, and the gradient of the key/value/other tensors is unchanged."""
    th, ids, tgt = _case(seed=5)
    tau = 1.6
    d = CFG["d_model"]
    scaled = th.astype(np.float64).copy()
    off = 0
    q_slices = []
    for name, shape in T.layout(CFG):
        k = int(np.prod(shape))
        if name.startswith("w_qkv"):
            scaled[off:off + d * d] /= tau; q_slices.append((off, off + d * d))
        if name.startswith("b_qkv"):
            scaled[off:off + d] /= tau; q_slices.append((off, off + d))
        off += k
    l1, g1 = T.loss_and_grad(th, ids, tgt, CFG, attn_temp=tau)
    l2, g2 = T.loss_and_grad(scaled, ids, tgt, CFG)
    assert l1 == pytest.approx(l2, rel=1e-12)
    for a, b in q_slices:                     # chain rule: d/dW_q at tau = (1/tau) d/dW_q' at W_q' = W_q/tau
        assert np.allclose(g1[a:b], g2[a:b] / tau, rtol=1e-5, atol=1e-10)
        g1[a:b] = 0; g2[a:b] = 0
    assert np.allclose(g1, g2, rtol=1e-5, atol=1e-10)
