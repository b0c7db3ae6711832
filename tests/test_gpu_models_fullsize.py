"""Parity of the mixed-precision forward/backward at the benchmark's full model sizes, in the launch
configuration bench.py times (N = 8 replicas, bf16 GEMMs, fp32 master weights).  The oracle is run
for sampled replicas only (its cost is per replica): the replicas are independent in
forward/backward, so a replica checks the same kernels, tile shapes and batch strides as all
eight do, and the first and the last one bound the replica indexing."""
import time

import numpy as np
import pytest
import torch

import hdet_inputs as I
import paper_2604_24708_amd as H
from harness import check_bf16_mlp_gradients, check_bf16_tensor, library_config, norm_err, oracle_config
from oracle import hdet_oracle as O
from oracle import mlp_oracle as M
from oracle import transformer_oracle as T

pytestmark = pytest.mark.gpu


def base(**kw):
    d = dict(n_replicas=8, total_steps=1000, sync_interval=16, warm_steps=300, lr_max=3e-4, alpha=0.1,
             autolr_enabled=True, optimizer=O.ADAMW, weight_decay=0.01, grad_mode=O.GRAD_PER_REPLICA,
             seed=I.SEED_PERM)
    d.update(kw)
    return d


def test_mlp_1024_4096x3_1000_batch_256():
    """The MLP workload: 1024-4096-4096-4096-1000, 256 rows per replica."""
    widths, batch, n = [1024, 4096, 4096, 4096, 1000], 256, 8
    P = I.mlp_param_count(widths)
    assert P == 41_858_024
    stride = (P + 3) // 4 * 4
    dev = "cuda:0"
    th0 = I.mlp_init(1, widths, I.SEED_INIT)[0]
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(th0).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.full_like(theta, 7.0)
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    d = base()
    cfg = library_config(d, widths=widths, batch=batch, model_kind=H.HDET_MLP, precision=H.HDET_BF16_GEMM_FP32_MASTER)
    _, _, ws = H.hdet_workspace_bytes(cfg, stride)
    wsb = torch.empty(ws, dtype=torch.uint8, device=dev)
    h = H.hdet_create(cfg, theta, m, v, grads=g, params_bf16=shadow, workspace=wsb, plane_stride=stride)
    x, y = I.mlp_batch(n, batch, widths[0], I.SEED_DATA, 1, widths, I.SEED_TEACHER)
    out = H.hdet_forward_backward(h, torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev), want_losses=True)
    for r in (0, 7):
        loss, ref = M.mlp_loss_and_grad(th0, x[r], y[r], widths, bf16=True)
        assert abs(out[r] - loss) <= 2e-3
        check_bf16_mlp_gradients(g[r, :P].cpu().numpy(), ref, widths, 2e-2, ("mlp-full", r))
    assert torch.all(g[:, P:] == 7.0)
    H.hdet_destroy(h)


def test_transformer_6l_d512_seq256_vocab32000():
    """The transformer workload: 6 layers, d_model 512, 8 heads, FFN 2048, 16 sequences of 256
    Zipf tokens per replica, vocabulary 32000 (fused attention, wide-row cross-entropy, every GEMM
    tile shape).  Replica 0 against the oracle (one replica is about 1 TFLOP of fp64 work)."""
    cfg = dict(n_blocks=6, d_model=512, n_heads=8, d_ff=2048, seq_len=256, vocab=32000)
    n, B = 8, 16
    P = I.transformer_param_count(cfg)
    stride = (P + 3) // 4 * 4
    dev = "cuda:0"
    th0 = I.transformer_init(1, cfg, I.SEED_INIT)[0]
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(th0).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.full_like(theta, 7.0)
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    d = base(total_steps=2000, sync_interval=32, warm_steps=600, lr_max=6e-4, alpha=0.15)
    lc = library_config(d, model_kind=H.HDET_TRANSFORMER, batch=B, precision=H.HDET_BF16_GEMM_FP32_MASTER, **cfg)
    _, _, ws = H.hdet_workspace_bytes(lc, stride)
    wsb = torch.empty(ws, dtype=torch.uint8, device=dev)
    h = H.hdet_create(lc, theta, m, v, grads=g, params_bf16=shadow, workspace=wsb, plane_stride=stride)
    ids, tgt = I.zipf_tokens(n, B, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, 0)
    out = H.hdet_forward_backward(h, torch.from_numpy(ids).to(dev), torch.from_numpy(tgt).to(dev), want_losses=True)
    losses = np.array([out[r] for r in range(n)])
    assert np.all(np.isfinite(losses)) and np.all(np.abs(losses - np.log(cfg["vocab"])) < 1.0)
    t0 = time.time()
    loss, ref = T.loss_and_grad(th0, ids[0], tgt[0], cfg, bf16=True)
    print(f"oracle: one replica in {time.time() - t0:.1f} s")
    assert abs(losses[0] - loss) <= 1e-2
    g_dev = g[0, :P].cpu().numpy()
    off = 0
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape))
        check_bf16_tensor(g_dev[off:off + k], ref[off:off + k], 4e-2, ("tf6-full", name))
        off += k
    assert torch.all(g[:, P:] == 7.0) if stride > P else True
    # ... and the loss curve of replica 0 over the first three steps (no converge inside T = 32, so the replica is
    # a training run of its own at the rate eta(t) rho_0): the oracle as a one-replica run at that rate
    d1 = dict(d, n_replicas=1, alpha=0.0, lr_max=d["lr_max"] * (1.0 - d["alpha"]), autolr_enabled=False)
    orc = O.HDETOracle(oracle_config(d1), th0[None, :])
    curve = [(float(losses[0]), float(loss))]
    H.hdet_fanout_step(h, None, 0)
    orc.fanout_step(ref[None, :], [loss])
    for t in (1, 2):
        ids, tgt = I.zipf_tokens(n, B, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, t)
        out = H.hdet_forward_backward(h, torch.from_numpy(ids).to(dev), torch.from_numpy(tgt).to(dev), want_losses=True)
        loss, ref = T.loss_and_grad(orc.theta[0], ids[0], tgt[0], cfg, bf16=True)
        curve.append((float(out[0]), float(loss)))
        H.hdet_fanout_step(h, None, 0)
        orc.fanout_step(ref[None, :], [loss])
    print("loss curve of replica 0 (device, oracle):", curve)
    assert all(abs(a - b) <= 1e-2 for a, b in curve), curve
    assert norm_err(theta[0, :P].cpu().numpy(), orc.theta[0]) <= 1e-3
    H.hdet_destroy(h)


def test_head_and_loss_at_the_12_layer_shapes():
    """The output head and the loss of the larger transformer workload in the launch shape of its 12-layer step:
    8192 rows per replica (16 sequences of 512 tokens) against the full vocabulary of 32000 at d_model 1024 -- the
    head product, the wide-row loss kernel walking several rows per block with the head bias sums, and the head's
    weight and input gradients (K = 32000 and K = 8192).  One block, two replicas, replica 1 against the oracle."""
    cfg = dict(n_blocks=1, d_model=1024, n_heads=16, d_ff=4096, seq_len=512, vocab=32000)
    n, B = 2, 16
    P = I.transformer_param_count(cfg)
    stride = (P + 63) // 64 * 64
    dev = "cuda:0"
    th0 = I.transformer_init(1, cfg, I.SEED_INIT)[0]
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(th0).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.full_like(theta, 7.0)
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    d = base(n_replicas=n, total_steps=4000, sync_interval=64, warm_steps=1200, lr_max=3e-4, alpha=0.15)
    lc = library_config(d, model_kind=H.HDET_TRANSFORMER, batch=B, precision=H.HDET_BF16_GEMM_FP32_MASTER, **cfg)
    _, _, ws = H.hdet_workspace_bytes(lc, stride)
    wsb = torch.empty(ws, dtype=torch.uint8, device=dev)
    h = H.hdet_create(lc, theta, m, v, grads=g, params_bf16=shadow, workspace=wsb, plane_stride=stride)
    ids, tgt = I.zipf_tokens(n, B, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, 0)
    out = H.hdet_forward_backward(h, torch.from_numpy(ids).to(dev), torch.from_numpy(tgt).to(dev), want_losses=True)
    t0 = time.time()
    loss, ref = T.loss_and_grad(th0, ids[1], tgt[1], cfg, bf16=True)
    print(f"oracle: one replica in {time.time() - t0:.1f} s")
    assert abs(out[1] - loss) <= 1e-2
    g_dev = g[1, :P].cpu().numpy()
    off = 0
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape))
        check_bf16_tensor(g_dev[off:off + k], ref[off:off + k], 4e-2, ("tf12-head", name))
        off += k
    assert torch.all(g[:, P:] == 7.0) if stride > P else True
    H.hdet_destroy(h)


def test_transformer_block_at_the_12_layer_shapes():
    """One block of the larger transformer workload at its full layer shapes: d_model 1024, 16 heads,
    FFN 4096, 16 sequences of 512 tokens per replica, with the dropout and weight-decay channels of
    that workload.  Every kernel runs in the launch shape the 12-layer step uses it in (256x256 GEMM
    tiles at K = 1024 and 4096, the two-blocks-per-CU tile of the GELU-gradient product, attention
    over eight key tiles, two register chunks per lane in LayerNorm, 64 row chunks in the column sums);
    the vocabulary is cut to 4096 and the depth to one block so that a replica of the oracle stays
    at about 1 TFLOP.  Replica 0 against the oracle."""
    cfg = dict(n_blocks=1, d_model=1024, n_heads=16, d_ff=4096, seq_len=512, vocab=4096)
    n, B = 2, 16
    P = I.transformer_param_count(cfg)
    stride = (P + 63) // 64 * 64
    dev = "cuda:0"
    th0 = I.transformer_init(1, cfg, I.SEED_INIT)[0]
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(th0).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.full_like(theta, 7.0)
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    extra = [(O.CH_DROPOUT, 0.1, 0.5, 0.5, 0.0, 0.5), (O.CH_WD, 0.01, 0.5, 0.5, 0.0, float("inf"))]
    d = base(n_replicas=n, total_steps=4000, sync_interval=64, warm_steps=1200, lr_max=3e-4, alpha=0.15, extra=extra)
    lc = library_config(d, model_kind=H.HDET_TRANSFORMER, batch=B, precision=H.HDET_BF16_GEMM_FP32_MASTER, **cfg)
    _, _, ws = H.hdet_workspace_bytes(lc, stride)
    wsb = torch.empty(ws, dtype=torch.uint8, device=dev)
    h = H.hdet_create(lc, theta, m, v, grads=g, params_bf16=shadow, workspace=wsb, plane_stride=stride)
    orc = O.HDETOracle(oracle_config(d), np.stack([th0] * n))
    ids, tgt = I.zipf_tokens(n, B, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, 0)
    out = H.hdet_forward_backward(h, torch.from_numpy(ids).to(dev), torch.from_numpy(tgt).to(dev), want_losses=True)
    p = orc.dropout_table()
    assert p[0] > 0
    t0 = time.time()
    loss, ref = T.loss_and_grad(th0, ids[0], tgt[0], cfg, bf16=True,
                                dropout=dict(p=float(p[0]), seed=d["seed"], step=1, replica=0))
    print(f"oracle: one replica in {time.time() - t0:.1f} s")
    assert abs(out[0] - loss) <= 1e-2
    g_dev = g[0, :P].cpu().numpy()
    off = 0
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape))
        check_bf16_tensor(g_dev[off:off + k], ref[off:off + k], 4e-2, ("tf12-block", name))
        off += k
    assert torch.all(g[:, P:] == 7.0) if stride > P else True
    H.hdet_destroy(h)


def _model_run(kind, dims, batch, d, stride, th0, P, dev="cuda:0"):
    n = d["n_replicas"]
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(th0).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.full_like(theta, 7.0)
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    lc = library_config(d, model_kind=kind, batch=batch, precision=H.HDET_BF16_GEMM_FP32_MASTER, **dims)
    _, _, ws = H.hdet_workspace_bytes(lc, stride)
    wsb = torch.empty(ws, dtype=torch.uint8, device=dev)
    h = H.hdet_create(lc, theta, m, v, grads=g, params_bf16=shadow, workspace=wsb, plane_stride=stride)
    return dict(h=h, theta=theta, m=m, v=v, g=g, shadow=shadow, ws=wsb)


@pytest.mark.parametrize("which", ["mlp", "transformer"])
def test_one_call_step_at_the_benchmark_shapes_equals_the_two_calls(which):
    """hdet_train_step in the launch configuration bench.py times (N = 8, the MLP and the 6-layer transformer at full
    size): parameters, moments and the bfloat16 copy after three steps, the last one a sync step with the fused
    converge, are those of hdet_forward_backward + hdet_fanout_step bit for bit, and no weight gradient was written.
    (The two-call sequence is what the other tests of this file hold against the oracle.)"""
    n = 8
    if which == "mlp":
        widths, batch = [1024, 4096, 4096, 4096, 1000], 256
        P = I.mlp_param_count(widths)
        th0 = I.mlp_init(1, widths, I.SEED_INIT)[0]
        d = base(sync_interval=3)
        kind, dims = H.HDET_MLP, dict(widths=widths)
        x, y = I.mlp_batch(n, batch, widths[0], I.SEED_DATA, 1, widths, I.SEED_TEACHER)
        off, mats = 0, []
        for i in range(len(widths) - 1):
            mats.append((off, widths[i + 1] * widths[i]))
            off += widths[i + 1] * widths[i] + widths[i + 1]
    else:
        cfg = dict(n_blocks=6, d_model=512, n_heads=8, d_ff=2048, seq_len=256, vocab=32000)
        batch = 16
        P = I.transformer_param_count(cfg)
        th0 = I.transformer_init(1, cfg, I.SEED_INIT)[0]
        d = base(total_steps=2000, sync_interval=3, warm_steps=600, lr_max=6e-4, alpha=0.15)
        kind, dims = H.HDET_TRANSFORMER, cfg
        x, y = I.zipf_tokens(n, batch, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, 1)
        off, mats = 0, []
        for name, shape in I.transformer_shapes(cfg):
            k = int(np.prod(shape))
            if name.startswith("w_"):
                # by default only products with at least one 256 x 256 tile per compute unit carry their update
                if -(-shape[0] // 256) * -(-shape[1] // 256) * n >= 256:
                    mats.append((off, k))
            off += k
        assert len(mats) == 1        # at these shapes: the head
    stride = (P + 63) // 64 * 64
    two = _model_run(kind, dims, batch, d, stride, th0, P)
    one = _model_run(kind, dims, batch, d, stride, th0, P)
    xd, yd = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0")
    for t in range(1, 4):
        l2 = H.hdet_forward_backward(two["h"], xd, yd, want_losses=True)
        H.hdet_fanout_step(two["h"], None, H.HDET_FUSE_CONVERGE)
        l1 = H.hdet_train_step(one["h"], xd, yd, H.HDET_FUSE_CONVERGE, want_losses=True)
        assert [l1[r] for r in range(n)] == [l2[r] for r in range(n)], t
        for r in (two, one):
            if t % 3 == 0:
                H.hdet_converge(r["h"])
                H.hdet_autolr_update(r["h"], None)
        for name in ("theta", "m", "v"):
            assert torch.equal(two[name].view(torch.int32), one[name].view(torch.int32)), (t, name)
        assert torch.equal(two["shadow"].view(torch.int16), one["shadow"].view(torch.int16)), t
    for off, k in mats:      # sampled: the first and last 4096 entries of every matrix in every plane
        assert torch.all(one["g"][:, off:off + 4096] == 7.0) and torch.all(one["g"][:, off + k - 4096:off + k] == 7.0), off
    assert torch.all(one["theta"][0, :P] == one["theta"][7, :P])          # the sync step averaged the replicas
    H.hdet_destroy(two["h"]); H.hdet_destroy(one["h"])
