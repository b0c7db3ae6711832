"""CPU oracle: per-replica forward, mean next-token cross-entropy and backward of a small
decoder-only transformer.

TEST INFRASTRUCTURE ONLY; shares no code with the HIP library.

This is the "Forward + backward" of Algorithm 1 for one replica.  The paper fixes no model;
the benchmark configurations name decoder-only transformers by (layers, d_model, heads, FFN,
sequence, vocabulary).  What they leave open is read as: pre-LayerNorm blocks, learned
positional embeddings, GELU in its tanh form, causal attention, biases on every Linear, an
untied output head with bias, a final LayerNorm, LayerNorm epsilon 1e-5.  Dropout, when a
rate p > 0 is given (Remark 1: the dropout rate as an explored hyperparameter; label
smoothing and the attention temperature are two more, see loss_and_grad), acts on the
two residual branches of every block (after the attention projection and after the MLP) with
keep-scaling 1/(1-p); its mask is a pure function of (seed, step, replica, site, element)
drawn from Philox-4x32-10, so both implementations regenerate it without exchanging it.

Flat parameter layout of one replica (all row-major):
  tok_emb [V, d], pos_emb [S, d],
  per block: ln1_g [d], ln1_b [d], w_qkv [3d, d], b_qkv [3d], w_o [d, d], b_o [d],
             ln2_g [d], ln2_b [d], w_1 [ff, d], b_1 [ff], w_2 [d, ff], b_2 [d],
  lnf_g [d], lnf_b [d], w_head [V, d], b_head [V].
Rows 0..d-1 of w_qkv produce q, d..2d-1 k, 2d..3d-1 v; head h owns columns h*dh..(h+1)*dh-1.

Arithmetic is fp64.  With bf16=True every tensor that the mixed-precision path keeps in
memory as bfloat16 is rounded (to nearest even) where it is stored: the residual stream,
every LayerNorm output, q/k/v, attention probabilities, attention output, MLP activations and
all their gradients, and the weights as the GEMMs see them; logits, attention scores,
LayerNorm statistics, biases, the loss and the parameter gradients stay in full precision.

Pinned by tests/test_oracle_transformer.py (autograd of an independent library in fp64,
central finite differences, dropout mask statistics and known-answer Philox vectors).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .hdet_oracle import philox4x32_10
from .mlp_oracle import round_bf16, softmax_xent

LN_EPS = 1e-5
DROPOUT_STREAM = 0x44524F50  # ASCII "DROP"


def layout(cfg: dict) -> List[Tuple[str, Tuple[int, ...]]]:
    d, ff, v, s = cfg["d_model"], cfg["d_ff"], cfg["vocab"], cfg["seq_len"]
    out = [("tok_emb", (v, d)), ("pos_emb", (s, d))]
    for l in range(cfg["n_blocks"]):
        out += [(f"ln1_g.{l}", (d,)), (f"ln1_b.{l}", (d,)), (f"w_qkv.{l}", (3 * d, d)), (f"b_qkv.{l}", (3 * d,)),
                (f"w_o.{l}", (d, d)), (f"b_o.{l}", (d,)), (f"ln2_g.{l}", (d,)), (f"ln2_b.{l}", (d,)),
                (f"w_1.{l}", (ff, d)), (f"b_1.{l}", (ff,)), (f"w_2.{l}", (d, ff)), (f"b_2.{l}", (d,))]
    out += [("lnf_g", (d,)), ("lnf_b", (d,)), ("w_head", (v, d)), ("b_head", (v,))]
    return out


def unpack(flat: np.ndarray, cfg: dict) -> Dict[str, np.ndarray]:
    p, off = {}, 0
    for name, shape in layout(cfg):
        n = int(np.prod(shape))
        p[name] = flat[off:off + n].reshape(shape)
        off += n
    assert off == flat.size
    return p


def dropout_keep(seed: int, step: int, replica: int, site: int, n: int, p: float) -> np.ndarray:
    """Keep mask of `n` elements for one dropout site: element e is kept iff its uniform
    u = word / 2^32 satisfies u >= p, where word is 32-bit word (e mod 4) of
    philox(counter = (e div 4, step, replica * 65536 + site, DROPOUT_STREAM), key = seed).
    The comparison is done on integers: word >= floor(p * 2^32)."""
    thresh = int(math.floor(float(p) * 4294967296.0))
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    keep = np.empty(n, dtype=bool)
    for blk in range((n + 3) // 4):
        w = philox4x32_10((blk, step & 0xFFFFFFFF, (replica * 65536 + site) & 0xFFFFFFFF, DROPOUT_STREAM), key)
        for j in range(4):
            e = 4 * blk + j
            if e < n:
                keep[e] = w[j] >= thresh
    return keep


def gelu_tanh(z):
    c = math.sqrt(2.0 / math.pi)
    return 0.5 * z * (1.0 + np.tanh(c * (z + 0.044715 * z ** 3)))


def gelu_tanh_grad(z):
    c = math.sqrt(2.0 / math.pi)
    u = c * (z + 0.044715 * z ** 3)
    t = np.tanh(u)
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * c * (1.0 + 3 * 0.044715 * z * z)


def layer_norm(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return xhat * g + b, xhat, rstd


def layer_norm_backward(dy, xhat, rstd, g):
    dg = (dy * xhat).sum(axis=0)
    db = dy.sum(axis=0)
    dxhat = dy * g
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True) - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def loss_and_grad(flat: np.ndarray, ids: np.ndarray, targets: np.ndarray, cfg: dict, bf16: bool = False,
                  dropout: Optional[dict] = None, label_smoothing: float = 0.0,
                  attn_temp: float = 1.0) -> Tuple[float, np.ndarray]:
    """ids, targets: [B, S] ints.  dropout: dict(p, seed, step, replica) or None.
    label_smoothing eps and attention temperature tau are two more of the scalars Remark 1
    names as explorable: the targets become (1 - eps) onehot + eps / V, and the attention
    scores are q.k / (sqrt(d_head) tau) (tau = 1: plain scaled dot-product attention).
    Returns (mean cross-entropy over the B*S positions, flat fp32 gradient)."""
    def q(a):
        return round_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64) if bf16 else np.asarray(a, np.float64)

    d, nh, ff, S, V, L = cfg["d_model"], cfg["n_heads"], cfg["d_ff"], cfg["seq_len"], cfg["vocab"], cfg["n_blocks"]
    dh = d // nh
    B = ids.shape[0]
    M = B * S
    P = unpack(flat, cfg)
    W = {k: v.astype(np.float64) for k, v in P.items()}
    p_drop = float(dropout["p"]) if dropout else 0.0

    def keep_mask(site):
        if p_drop <= 0.0:
            return None
        k = dropout_keep(dropout["seed"], dropout["step"], dropout["replica"], site, M * d, p_drop)
        return k.reshape(M, d)

    scale = 1.0 / (math.sqrt(dh) * attn_temp)
    causal = np.tril(np.ones((S, S), dtype=bool))
    pos = np.tile(np.arange(S), B)
    tok = ids.reshape(-1)
    x = q(W["tok_emb"][tok] + W["pos_emb"][pos])                       # [M, d]
    cache = []
    for l in range(L):
        c = {"x_in": x}
        y1, c["xhat1"], c["rstd1"] = layer_norm(x, W[f"ln1_g.{l}"], W[f"ln1_b.{l}"])
        c["h1"] = h1 = q(y1)
        c["qkv"] = qkv = q(h1 @ q(W[f"w_qkv.{l}"]).T + W[f"b_qkv.{l}"])  # [M, 3d]
        a = np.zeros((M, d))
        c["p"] = probs = np.zeros((B, nh, S, S))
        for b in range(B):
            rows = slice(b * S, (b + 1) * S)
            for h in range(nh):
                cq = qkv[rows, h * dh:(h + 1) * dh]
                ck = qkv[rows, d + h * dh:d + (h + 1) * dh]
                cv = qkv[rows, 2 * d + h * dh:2 * d + (h + 1) * dh]
                sc = (cq @ ck.T) * scale
                sc = np.where(causal, sc, -np.inf)
                sc = sc - sc.max(axis=1, keepdims=True)
                e = np.exp(sc)
                pr = q(e / e.sum(axis=1, keepdims=True))
                probs[b, h] = pr
                a[rows, h * dh:(h + 1) * dh] = pr @ cv
        c["a"] = a = q(a)
        o = q(a @ q(W[f"w_o.{l}"]).T + W[f"b_o.{l}"])
        c["keep1"] = k1 = keep_mask(2 * l)
        if k1 is not None:
            o = o * k1 / (1.0 - p_drop)
        x = q(x + o)
        c["x_mid"] = x
        y2, c["xhat2"], c["rstd2"] = layer_norm(x, W[f"ln2_g.{l}"], W[f"ln2_b.{l}"])
        c["h2"] = h2 = q(y2)
        c["z"] = z = q(h2 @ q(W[f"w_1.{l}"]).T + W[f"b_1.{l}"])
        c["f"] = f = q(gelu_tanh(z))
        y = q(f @ q(W[f"w_2.{l}"]).T + W[f"b_2.{l}"])
        c["keep2"] = k2 = keep_mask(2 * l + 1)
        if k2 is not None:
            y = y * k2 / (1.0 - p_drop)
        x = q(x + y)
        cache.append(c)
    yf, xhatf, rstdf = layer_norm(x, W["lnf_g"], W["lnf_b"])
    hf = q(yf)
    logits = hf @ q(W["w_head"]).T + W["b_head"]
    loss, dlogits = softmax_xent(logits, targets.reshape(-1).astype(np.int64), label_smoothing)

    G = {k: np.zeros_like(v, dtype=np.float64) for k, v in P.items()}
    dl = q(dlogits)
    G["w_head"] = dl.T @ hf
    G["b_head"] = dl.sum(axis=0)
    dhf = q(dl @ q(W["w_head"]))
    dx, G["lnf_g"], G["lnf_b"] = layer_norm_backward(dhf, xhatf, rstdf, W["lnf_g"])
    dx = q(dx)
    for l in range(L - 1, -1, -1):
        c = cache[l]
        # MLP branch: x_out = x_mid + drop(y)
        dy = dx
        if c["keep2"] is not None:
            dy = q(dx * c["keep2"] / (1.0 - p_drop))
        G[f"w_2.{l}"] = dy.T @ c["f"]
        G[f"b_2.{l}"] = dy.sum(axis=0)
        df = q(dy @ q(W[f"w_2.{l}"]))
        dz = q(df * gelu_tanh_grad(c["z"]))
        G[f"w_1.{l}"] = dz.T @ c["h2"]
        G[f"b_1.{l}"] = dz.sum(axis=0)
        dh2 = q(dz @ q(W[f"w_1.{l}"]))
        dln, G[f"ln2_g.{l}"], G[f"ln2_b.{l}"] = layer_norm_backward(dh2, c["xhat2"], c["rstd2"], W[f"ln2_g.{l}"])
        dx = q(dx + dln)                                              # gradient at x_mid
        # attention branch: x_mid = x_in + drop(o)
        do = dx
        if c["keep1"] is not None:
            do = q(dx * c["keep1"] / (1.0 - p_drop))
        G[f"w_o.{l}"] = do.T @ c["a"]
        G[f"b_o.{l}"] = do.sum(axis=0)
        da = q(do @ q(W[f"w_o.{l}"]))
        dqkv = np.zeros((M, 3 * d))
        qkv = c["qkv"]
        for b in range(B):
            rows = slice(b * S, (b + 1) * S)
            for h in range(nh):
                cq = qkv[rows, h * dh:(h + 1) * dh]
                ck = qkv[rows, d + h * dh:d + (h + 1) * dh]
                cv = qkv[rows, 2 * d + h * dh:2 * d + (h + 1) * dh]
                pr = c["p"][b, h]
                dah = da[rows, h * dh:(h + 1) * dh]
                dp = dah @ cv.T
                ds = q(pr * (dp - (dp * pr).sum(axis=1, keepdims=True)) * scale)
                dqkv[rows, h * dh:(h + 1) * dh] = ds @ ck
                dqkv[rows, d + h * dh:d + (h + 1) * dh] = ds.T @ cq
                dqkv[rows, 2 * d + h * dh:2 * d + (h + 1) * dh] = pr.T @ dah
        dqkv = q(dqkv)
        G[f"w_qkv.{l}"] = dqkv.T @ c["h1"]
        G[f"b_qkv.{l}"] = dqkv.sum(axis=0)
        dh1 = q(dqkv @ q(W[f"w_qkv.{l}"]))
        dln, G[f"ln1_g.{l}"], G[f"ln1_b.{l}"] = layer_norm_backward(dh1, c["xhat1"], c["rstd1"], W[f"ln1_g.{l}"])
        dx = q(dx + dln)                                              # gradient at x_in
    np.add.at(G["tok_emb"], tok, dx)
    np.add.at(G["pos_emb"], pos, dx)
    grad = np.concatenate([G[name].ravel() for name, _ in layout(cfg)]).astype(np.float32)
    return loss, grad


def logits_only(flat: np.ndarray, ids: np.ndarray, cfg: dict) -> np.ndarray:
    """Full-precision logits without dropout (used by the finite-difference pin)."""
    d, nh, S, L = cfg["d_model"], cfg["n_heads"], cfg["seq_len"], cfg["n_blocks"]
    dh = d // nh
    B = ids.shape[0]
    W = {k: v.astype(np.float64) for k, v in unpack(flat, cfg).items()}
    causal = np.tril(np.ones((S, S), dtype=bool))
    x = W["tok_emb"][ids.reshape(-1)] + W["pos_emb"][np.tile(np.arange(S), B)]
    for l in range(L):
        h1 = layer_norm(x, W[f"ln1_g.{l}"], W[f"ln1_b.{l}"])[0]
        qkv = h1 @ W[f"w_qkv.{l}"].T + W[f"b_qkv.{l}"]
        a = np.zeros_like(x)
        for b in range(B):
            rows = slice(b * S, (b + 1) * S)
            for h in range(nh):
                sc = qkv[rows, h * dh:(h + 1) * dh] @ qkv[rows, d + h * dh:d + (h + 1) * dh].T / math.sqrt(dh)
                sc = np.where(causal, sc, -np.inf)
                e = np.exp(sc - sc.max(axis=1, keepdims=True))
                a[rows, h * dh:(h + 1) * dh] = (e / e.sum(axis=1, keepdims=True)) @ qkv[rows, 2 * d + h * dh:2 * d + (h + 1) * dh]
        x = x + a @ W[f"w_o.{l}"].T + W[f"b_o.{l}"]
        h2 = layer_norm(x, W[f"ln2_g.{l}"], W[f"ln2_b.{l}"])[0]
        x = x + gelu_tanh(h2 @ W[f"w_1.{l}"].T + W[f"b_1.{l}"]) @ W[f"w_2.{l}"].T + W[f"b_2.{l}"]
    return layer_norm(x, W["lnf_g"], W["lnf_b"])[0] @ W["w_head"].T + W["b_head"]
