"""Transformer case: initial parameters and Zipf-distributed token ids."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def transformer_shapes(cfg: dict) -> List[Tuple[str, Tuple[int, ...]]]:
    """Tensor order and shapes inside one replica's flat parameter plane."""
    d, ff, v, s = cfg["d_model"], cfg["d_ff"], cfg["vocab"], cfg["seq_len"]
    out = [("tok_emb", (v, d)), ("pos_emb", (s, d))]
    for l in range(cfg["n_blocks"]):
        out += [(f"ln1_g.{l}", (d,)), (f"ln1_b.{l}", (d,)), (f"w_qkv.{l}", (3 * d, d)), (f"b_qkv.{l}", (3 * d,)),
                (f"w_o.{l}", (d, d)), (f"b_o.{l}", (d,)), (f"ln2_g.{l}", (d,)), (f"ln2_b.{l}", (d,)),
                (f"w_1.{l}", (ff, d)), (f"b_1.{l}", (ff,)), (f"w_2.{l}", (d, ff)), (f"b_2.{l}", (d,))]
    out += [("lnf_g", (d,)), ("lnf_b", (d,)), ("w_head", (v, d)), ("b_head", (v,))]
    return out


def transformer_param_count(cfg: dict) -> int:
    return sum(int(np.prod(shape)) for _, shape in transformer_shapes(cfg))


def transformer_init(n: int, cfg: dict, seed: int, std: float = 0.02, bias_std: float = 0.0) -> np.ndarray:
    """[N, P] initial parameters, identical across replicas: weights and embeddings
    ~N(0, std^2), LayerNorm gains 1 (+ small noise if bias_std > 0), biases 0 (or
    ~N(0, bias_std^2), which tests use so that no gradient path is trivially zero)."""
    rng = np.random.Generator(np.random.Philox(seed))
    parts = []
    for name, shape in transformer_shapes(cfg):
        k = int(np.prod(shape))
        base = name.split(".")[0]
        if base in ("ln1_g", "ln2_g", "lnf_g"):
            parts.append((1.0 + bias_std * rng.standard_normal(k)).astype(np.float32))
        elif len(shape) == 1:
            parts.append((bias_std * rng.standard_normal(k)).astype(np.float32))
        else:
            parts.append((std * rng.standard_normal(k)).astype(np.float32))
    one = np.concatenate(parts)
    return np.broadcast_to(one, (n, one.size)).copy()


def zipf_tokens(n: int, batch: int, seq_len: int, vocab: int, seed: int, step: int, s: float = 1.1):
    """Token ids ~Zipf(s) over `vocab` ranks (inverse CDF on the exact normalised table).
    Returns (ids [N, B, S], targets [N, B, S]) int32 with targets = ids shifted by one
    (S + 1 tokens are drawn per sequence)."""
    w = 1.0 / np.arange(1, vocab + 1, dtype=np.float64) ** s
    cdf = np.cumsum(w / w.sum())
    rng = np.random.Generator(np.random.Philox(key=[seed, step]))
    u = rng.random((n, batch, seq_len + 1))
    tok = np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1).astype(np.int32)
    return np.ascontiguousarray(tok[..., :-1]), np.ascontiguousarray(tok[..., 1:])
