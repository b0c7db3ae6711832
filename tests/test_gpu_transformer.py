"""Parity of the transformer forward/backward (and of the whole HDET loop on it) between the
HIP path and the CPU oracle: full precision element-wise, mixed precision by loss curve."""
import numpy as np
import pytest
import torch

import hdet_inputs as I
import paper_2604_24708_amd as H
from harness import check_bf16_tensor, check_state, library_config, oracle_config, rel_err
from oracle import hdet_oracle as O
from oracle import transformer_oracle as T

pytestmark = pytest.mark.gpu

TINY = dict(n_blocks=2, d_model=16, n_heads=4, d_ff=40, seq_len=6, vocab=29)
SMALL = dict(n_blocks=2, d_model=64, n_heads=4, d_ff=256, seq_len=32, vocab=512)      # several tiles
ODD = dict(n_blocks=1, d_model=24, n_heads=3, d_ff=50, seq_len=70, vocab=131)        # ragged everywhere
# two register chunks per lane in LayerNorm (d > 512) and softmax (S > 256), wide-row cross-entropy
MID = dict(n_blocks=1, d_model=576, n_heads=9, d_ff=1152, seq_len=264, vocab=2304)
# LayerNorm widths beyond what its backward kernel reduces itself (1024) and beyond the vector kernels (2048)
WIDE = dict(n_blocks=1, d_model=1088, n_heads=17, d_ff=64, seq_len=8, vocab=40)
WIDER = dict(n_blocks=1, d_model=2112, n_heads=33, d_ff=32, seq_len=6, vocab=24)
# head size 64 and sequence lengths that are multiples of 64: the shapes the fused attention kernels take
# (one, three and four 64-row blocks per sequence; one and two heads)
FUSE1 = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=64, seq_len=64, vocab=50)
FUSE3 = dict(n_blocks=2, d_model=128, n_heads=2, d_ff=96, seq_len=192, vocab=61)
FUSE4 = dict(n_blocks=1, d_model=128, n_heads=2, d_ff=64, seq_len=256, vocab=40)
FUSE5 = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=64, seq_len=320, vocab=40)      # last 128-row block half empty
FUSE8 = dict(n_blocks=1, d_model=128, n_heads=2, d_ff=64, seq_len=512, vocab=40)
FUSE16 = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=64, seq_len=1024, vocab=40)


def norm_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def base(**kw):
    d = dict(n_replicas=3, total_steps=12, sync_interval=4, warm_steps=4, lr_max=0.02, alpha=0.2,
             autolr_enabled=True, optimizer=O.SGDM, momentum=0.9, weight_decay=0.0,
             grad_mode=O.GRAD_PER_REPLICA, seed=I.SEED_PERM)
    d.update(kw)
    return d


class TfRun:
    def __init__(self, d, cfg, batch, bf16=False):
        self.d, self.cfg, self.batch, self.bf16 = d, cfg, batch, bf16
        self.n = n = d["n_replicas"]
        self.P = P = I.transformer_param_count(cfg)
        self.stride = (P + 3) // 4 * 4
        th0 = I.transformer_init(n, cfg, I.SEED_INIT, std=0.1, bias_std=0.05)
        self.orc = O.HDETOracle(oracle_config(d), th0)
        dev = "cuda:0"
        host = np.zeros((n, self.stride), np.float32)
        host[:, :P] = th0
        self.theta = torch.from_numpy(host).to(dev)
        self.m, self.v = torch.zeros_like(self.theta), torch.zeros_like(self.theta)
        self.g = torch.full_like(self.theta, 7.0)        # stale values must all be overwritten
        self.shadow = torch.zeros((n, self.stride), dtype=torch.bfloat16, device=dev) if bf16 else None
        lc = library_config(d, model_kind=H.HDET_TRANSFORMER, batch=batch,
                            precision=H.HDET_BF16_GEMM_FP32_MASTER if bf16 else H.HDET_FP32, **cfg)
        _, _, ws = H.hdet_workspace_bytes(lc, self.stride)
        self.ws = torch.empty(ws, dtype=torch.uint8, device=dev)
        self.h = H.hdet_create(lc, self.theta, self.m, self.v if d["optimizer"] == O.ADAMW else None,
                               grads=self.g, params_bf16=self.shadow, workspace=self.ws, plane_stride=self.stride)

    def oracle_grads(self, theta, ids, tgt, step):
        n = self.n
        losses, grads = np.zeros(n), np.zeros((n, self.P), np.float32)
        p = self.orc.dropout_table()
        eps, tau = self.orc.label_smoothing_table(), self.orc.attn_temp_table()
        for r in range(n):
            dp = dict(p=float(p[r]), seed=self.d["seed"], step=step, replica=r) if p[r] > 0 else None
            losses[r], grads[r] = T.loss_and_grad(theta[r], ids[r], tgt[r], self.cfg, bf16=self.bf16, dropout=dp,
                                                  label_smoothing=float(eps[r]), attn_temp=float(tau[r]))
        return losses, grads

    def forward_backward(self, t):
        ids, tgt = I.zipf_tokens(self.n, self.batch, self.cfg["seq_len"], self.cfg["vocab"], I.SEED_DATA, t)
        out = H.hdet_forward_backward(self.h, torch.from_numpy(ids).to("cuda:0"), torch.from_numpy(tgt).to("cuda:0"),
                                      want_losses=True)
        return ids, tgt, np.array([out[r] for r in range(self.n)])

    def finish_step(self, t, grads, losses, fuse=False):
        H.hdet_fanout_step(self.h, None, H.HDET_FUSE_CONVERGE if fuse else 0)
        self.orc.fanout_step(grads, losses)
        if t % self.d["sync_interval"] == 0:
            H.hdet_converge(self.h)
            self.orc.converge()
            H.hdet_autolr_update(self.h, None)
            self.orc.autolr_update()

    def close(self):
        H.hdet_destroy(self.h)


def check_bf16_gradients(cfg, g_dev, g_ref, norm_tol, tag):
    """Every gradient tensor of a mixed-precision replica: norm-wise and entry by entry."""
    off = 0
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape))
        check_bf16_tensor(g_dev[off:off + k], g_ref[off:off + k], norm_tol, (tag, name))
        off += k


def per_tensor_errors(cfg, g_dev, g_ref):
    out, off = {}, 0
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape))
        out[name] = norm_err(g_dev[off:off + k], g_ref[off:off + k])
        off += k
    return out


@pytest.mark.parametrize("cfg,batch,n", [(TINY, 3, 3), (SMALL, 4, 2), (ODD, 2, 2), (MID, 2, 2), (WIDE, 5, 2), (WIDER, 2, 2)])
def test_fp32_loss_and_every_gradient_tensor(cfg, batch, n):
    run = TfRun(base(n_replicas=n), cfg, batch)
    ids, tgt, gl = run.forward_backward(1)
    losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, 1)
    assert np.max(np.abs(gl - losses) / np.maximum(1.0, np.abs(losses))) <= 1e-5     # relative for losses above 1
    g_dev = run.g.cpu().numpy()[:, :run.P]
    for r in range(n):
        errs = per_tensor_errors(cfg, g_dev[r], grads[r])
        bad = {k: v for k, v in errs.items() if v > 2e-5}
        assert not bad, (r, bad)
    # entry-wise over the whole plane (tensors of very different scale, dot products of up to
    # M or V fp32 terms): an intermediate, bounded loosely; the per-tensor norms above are the check
    # (not for the wide cases: a few tokens against dot products of 1000-2000 fp32 terms that cancel)
    if cfg not in (WIDE, WIDER):
        assert rel_err(g_dev, grads) <= (2e-4 if cfg is not MID else 5e-3)
    run.close()


@pytest.mark.parametrize("cfg,batch,n", [(TINY, 3, 3), (SMALL, 4, 2)])
def test_fp32_full_loop_trajectory(cfg, batch, n):
    d = base(n_replicas=n)
    run = TfRun(d, cfg, batch)
    first = last = None
    for t in range(1, 13):
        ids, tgt, gl = run.forward_backward(t)
        losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, t)
        assert np.max(np.abs(gl - losses)) <= 1e-4
        run.finish_step(t, grads, losses, fuse=(t == 8))
        assert rel_err(run.theta.cpu().numpy()[:, :run.P], run.orc.theta) <= min(t * 1e-5, 1e-4)
        check_state(H.hdet_get_state(run.h), run.orc, scalar_rtol=5e-6, lr_ulps=None)
        first = losses.mean() if first is None else first
        last = losses.mean()
    assert last < first
    run.close()


def test_fp32_dropout_and_weight_decay_channels():
    """Three explored scalars (rate, dropout, weight decay) with independent permutations
    (Remark 1); dropout masks regenerated on both sides from (seed, step, replica, site)."""
    extra = [(O.CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45), (O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))]
    d = base(n_replicas=4, optimizer=O.ADAMW, lr_max=2e-3, alpha=0.15, extra=extra, total_steps=10, sync_interval=2,
             warm_steps=2)
    run = TfRun(d, TINY, 3)
    for t in range(1, 9):
        # compare each step from the device's own state (Adam's early steps are ill-conditioned in g)
        run.orc.theta = run.theta.cpu().numpy()[:, :run.P].copy()
        run.orc.m = run.m.cpu().numpy()[:, :run.P].copy()
        run.orc.v = run.v.cpu().numpy()[:, :run.P].copy()
        ids, tgt, gl = run.forward_backward(t)
        p = run.orc.dropout_table()
        assert p.max() > 0.15 and p.min() < 0.05
        losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, t)
        assert np.max(np.abs(gl - losses)) <= 2e-5
        g_dev = run.g.cpu().numpy()[:, :run.P]
        for r in range(4):
            assert norm_err(g_dev[r], grads[r]) <= 2e-5, (t, r)
        run.finish_step(t, grads, losses)
        st = H.hdet_get_state(run.h)
        assert st.k == run.orc.k
        for j in range(3):
            assert [st.perm[j][r] for r in range(4)] == run.orc.perm[j].tolist()
    assert st.k == 4 and len({tuple(st.perm[j][r] for r in range(4)) for j in range(3)}) >= 2
    run.close()


@pytest.mark.parametrize("cfg,batch,n,steps", [(TINY, 3, 3, 12), (SMALL, 4, 2, 12), (ODD, 2, 2, 6), (MID, 2, 2, 2)])
def test_bf16_loss_curve_within_1e2(cfg, batch, n, steps):
    d = base(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, weight_decay=0.01, total_steps=steps)
    run = TfRun(d, cfg, batch, bf16=True)
    for t in range(1, steps + 1):
        ids, tgt, gl = run.forward_backward(t)
        losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, t)
        assert np.max(np.abs(gl - losses)) <= 1e-2
        if t == 1:
            g_dev = run.g.cpu().numpy()[:, :run.P]
            for r in range(n):
                check_bf16_gradients(cfg, g_dev[r], grads[r], 4e-2, ("curve", cfg["d_model"], r))
        run.finish_step(t, grads, losses, fuse=(t == 8))
    run.close()


def test_bf16_weight_gradients_formed_in_pieces_along_the_batch():
    """1024 rows per replica and matrices of one or two tiles: every weight gradient is formed in two pieces along the
    contraction (as extra batch items) and the pieces are added in a fixed order.  Against the oracle entry by entry,
    and bit-reproducible from run to run."""
    cfg = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=128, seq_len=64, vocab=56)
    d = base(n_replicas=2, optimizer=O.ADAMW, lr_max=2e-3)
    run = TfRun(d, cfg, 16, bf16=True)
    ids, tgt, gl = run.forward_backward(1)
    losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, 1)
    assert np.max(np.abs(gl - losses)) <= 1e-2
    g1 = run.g.clone()
    for r in range(2):
        check_bf16_gradients(cfg, g1[r, :run.P].cpu().numpy(), grads[r], 4e-2, ("pieces", r))
    run.g.fill_(7.0)
    run.forward_backward(1)
    assert torch.equal(g1[:, :run.P], run.g[:, :run.P])
    run.close()


def test_bf16_dropout_loss_matches():
    extra = [(O.CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45)]
    d = base(n_replicas=4, optimizer=O.ADAMW, lr_max=2e-3, extra=extra)
    run = TfRun(d, SMALL, 2, bf16=True)
    for t in range(1, 4):
        ids, tgt, gl = run.forward_backward(t)
        losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, t)
        assert np.max(np.abs(gl - losses)) <= 1e-2
        run.finish_step(t, grads, losses)
    run.close()


@pytest.mark.parametrize("cfg,batch", [(TINY, 3), (SMALL, 2)])
def test_fp32_label_smoothing_and_attention_temperature_channels(cfg, batch):
    """Two more of Remark 1's scalars as channels: replica r smooths its targets by eps_r and
    divides its attention scores by tau_r; five channels with the dropout and weight-decay
    ones, each with its own permutation."""
    n = 4
    extra = [(O.CH_LABEL_SMOOTH, 0.1, 0.5, 0.5, 0.0, 0.5), (O.CH_ATTN_TEMP, 1.2, 0.4, 0.5, 0.25, 4.0),
             (O.CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45), (O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))]
    d = base(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, extra=extra)
    run = TfRun(d, cfg, batch)
    for t in range(1, 13):
        ids, tgt, gl = run.forward_backward(t)
        losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, t)
        assert np.max(np.abs(gl - losses)) <= 1e-4
        if t in (1, 9):
            g_dev = run.g.cpu().numpy()[:, :run.P]
            for r in range(n):
                at_dev = T.loss_and_grad(run.theta.cpu().numpy()[r, :run.P], ids[r], tgt[r], cfg,
                                         dropout=dict(p=float(run.orc.dropout_table()[r]), seed=d["seed"], step=t, replica=r),
                                         label_smoothing=float(run.orc.label_smoothing_table()[r]),
                                         attn_temp=float(run.orc.attn_temp_table()[r]))[1]
                bad = {k: v for k, v in per_tensor_errors(cfg, g_dev[r], at_dev).items() if v > 5e-5}
                assert not bad, (t, r, bad)
        run.finish_step(t, grads, losses, fuse=(t == 8))
        st = H.hdet_get_state(run.h)
        assert st.k == run.orc.k and st.n_channels == 5
        for j in range(5):
            assert [st.perm[j][r] for r in range(n)] == run.orc.perm[j].tolist()
    tau = run.orc.attn_temp_table()
    assert len(set(tau.tolist())) == n and tau.min() > 0.5
    # a run without the two channels gives different losses: the scalars do reach the kernels
    plain = TfRun(base(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, extra=extra[2:]), cfg, batch)
    _, _, gl0 = plain.forward_backward(1)
    run2 = TfRun(d, cfg, batch)
    _, _, gl1 = run2.forward_backward(1)
    assert np.min(np.abs(gl0 - gl1)) > 1e-4
    for x in (run, plain, run2):
        x.close()


# wide vocabularies with enough rows that the loss kernel takes several rows per block and forms the
# first stage of the head bias gradient itself: 3 x 42 x 70 rows = 8 per block with a ragged last block;
# 2104 classes = 526 four-element chunks over 256 threads, 8200 = 2050 over 512 threads
LOSS_A = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=64, seq_len=70, vocab=2104)
LOSS_B = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=64, seq_len=70, vocab=8200)


@pytest.mark.parametrize("cfg,bf16", [(LOSS_A, False), (LOSS_A, True), (LOSS_B, False), (LOSS_B, True)])
def test_wide_row_loss_with_head_bias_partial_sums(cfg, bf16):
    """Loss, head bias gradient and every other tensor when the cross-entropy kernel walks several rows
    per block, with a label-smoothing channel (eps_r differs per replica)."""
    n, batch = 3, 42
    extra = [(O.CH_LABEL_SMOOTH, 0.1, 0.5, 0.5, 0.0, 0.5)]
    run = TfRun(base(n_replicas=n, extra=extra), cfg, batch, bf16=bf16)
    assert (n * batch * cfg["seq_len"]) // 1024 == 8 and (batch * cfg["seq_len"]) % 8 != 0
    ids, tgt, gl = run.forward_backward(1)
    eps = run.orc.label_smoothing_table()
    assert len(set(eps.tolist())) == n and eps.min() > 0.02
    losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, 1)
    assert np.max(np.abs(gl - losses) / np.maximum(1.0, np.abs(losses))) <= (1e-2 if bf16 else 1e-5)
    g_dev = run.g.cpu().numpy()[:, :run.P]
    for r in range(n):
        if bf16:
            check_bf16_gradients(cfg, g_dev[r], grads[r], 4e-2, ("wide", cfg["vocab"], r))
        else:
            bad = {k: v for k, v in per_tensor_errors(cfg, g_dev[r], grads[r]).items() if v > 2e-5}
            assert not bad, (r, bad)
    assert torch.all(run.g[:, run.P:] == 7.0) if run.stride > run.P else True
    run.close()


@pytest.mark.parametrize("cfg,batch,n", [(FUSE1, 2, 2), (FUSE3, 2, 3), (FUSE4, 3, 2), (FUSE5, 2, 2), (FUSE8, 2, 2), (FUSE16, 1, 2)])
def test_bf16_fused_attention_against_oracle_and_unfused_path(cfg, batch, n):
    """The fused attention kernels (scores kept on chip) against the oracle, at the mixed-precision
    bar, and against the library's own path through separate GEMM and softmax kernels, with which
    they share every bf16 rounding point: those two agree far more closely.  An attention
    temperature channel makes the score scale differ per replica."""
    extra = [(O.CH_ATTN_TEMP, 1.2, 0.4, 0.5, 0.25, 4.0)]
    d = base(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, extra=extra)
    fused, plain = TfRun(d, cfg, batch, bf16=True), TfRun(d, cfg, batch, bf16=True)
    H.hdet_set_launch_shape(plain.h, 2, 0)                # separate kernels, scores in device memory
    for t in range(1, 4):
        ids, tgt, gl = fused.forward_backward(t)
        losses, grads = fused.oracle_grads(fused.orc.theta, ids, tgt, t)
        assert np.max(np.abs(gl - losses)) <= 1e-2
        gf = fused.g.cpu().numpy()[:, :fused.P]
        for r in range(n):
            check_bf16_gradients(cfg, gf[r], grads[r], 4e-2, ("fused", cfg["seq_len"], t, r))
        if t == 1:      # same parameters on both handles only before the first update
            _, _, gl_plain = plain.forward_backward(t)
            assert np.max(np.abs(gl - gl_plain)) <= 5e-4    # a few bf16 roundings flip with the order of the fp32 row sums
            gp = plain.g.cpu().numpy()[:, :fused.P]
            for r in range(n):
                bad = {k: v for k, v in per_tensor_errors(cfg, gf[r], gp[r]).items() if v > 5e-3}
                assert not bad, ("unfused", t, r, bad)
        fused.finish_step(t, grads, losses)
    fused.close(); plain.close()


@pytest.mark.parametrize("cfg,batch,bf16", [(SMALL, 4, False), (FUSE3, 3, True), (MID, 2, True)])
def test_gradients_are_bit_reproducible(cfg, batch, bf16):
    """Every reduction of the forward/backward pass has a fixed order (the token-embedding gradient is
    formed from sorted rows, not with atomics): two handles fed the same batch give identical bits,
    losses included, also when other work ran on the device in between."""
    d = base(n_replicas=3, optimizer=O.ADAMW, lr_max=2e-3)
    a, b = TfRun(d, cfg, batch, bf16=bf16), TfRun(d, cfg, batch, bf16=bf16)
    _, _, la = a.forward_backward(1)
    torch.randn(1 << 22, device="cuda:0").sum().item()
    _, _, lb = b.forward_backward(1)
    assert np.array_equal(la, lb)
    assert torch.equal(a.g, b.g)
    _, _, la2 = a.forward_backward(1)
    assert torch.equal(a.g, b.g) and np.array_equal(la, la2)
    a.close(); b.close()


def test_checkpoint_resume_is_bit_exact_on_the_transformer():
    """Parameters, optimizer state and hdet_get_state after 5 steps, loaded into a fresh handle, continue
    exactly as the uninterrupted run does for 7 more steps (mixed precision, a dropout channel whose masks
    are keyed on the step counter, AdamW, two sync steps with the controller on either side of the break)."""
    extra = [(O.CH_DROPOUT, 0.1, 0.5, 0.5, 0.0, 0.5)]
    d = base(n_replicas=3, optimizer=O.ADAMW, lr_max=2e-3, weight_decay=0.01, extra=extra)
    a = TfRun(d, FUSE3, 2, bf16=True)

    def step(run, t):
        ids, tgt = I.zipf_tokens(run.n, run.batch, run.cfg["seq_len"], run.cfg["vocab"], I.SEED_DATA, t)
        H.hdet_forward_backward(run.h, torch.from_numpy(ids).to("cuda:0"), torch.from_numpy(tgt).to("cuda:0"))
        H.hdet_fanout_step(run.h, None, H.HDET_FUSE_CONVERGE if t == 8 else 0)
        if t % d["sync_interval"] == 0:
            H.hdet_converge(run.h)
            H.hdet_autolr_update(run.h, None)

    for t in range(1, 6):
        step(a, t)
    st = H.hdet_get_state(a.h)
    b = TfRun(d, FUSE3, 2, bf16=True)
    b.theta.copy_(a.theta); b.m.copy_(a.m); b.v.copy_(a.v); b.shadow.copy_(a.shadow)
    H.hdet_set_state(b.h, st)
    for t in range(6, 13):
        step(a, t)
        step(b, t)
    assert torch.equal(a.theta, b.theta) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v) and torch.equal(a.shadow, b.shadow)
    sa, sb = H.hdet_get_state(a.h), H.hdet_get_state(b.h)
    assert sa.k == sb.k and sa.t == sb.t
    for j in range(2):
        assert sa.base[j] == sb.base[j] and sa.vel[j] == sb.vel[j]
        assert [sa.perm[j][r] for r in range(3)] == [sb.perm[j][r] for r in range(3)]
    a.close(); b.close()


# a vocabulary wide enough that the head's weight gradient (128 tiles of 256 x 256) is formed as one product over the rows of all replicas
BIGV = dict(n_blocks=1, d_model=64, n_heads=1, d_ff=64, seq_len=32, vocab=32768)


def device_mean_gradient(cfg, g, n):
    """What the update applies in shared-gradient mode, rebuilt from the gradient buffer: a weight matrix of at least
    128 tiles of 256 x 256 is left as the sum over the replicas in plane 0 (the other planes untouched), every other
    tensor as one gradient per replica."""
    out, off, summed = np.empty(g.shape[1], np.float32), 0, []
    for name, shape in I.transformer_shapes(cfg):
        k = int(np.prod(shape))
        if len(shape) == 2 and -(-shape[0] // 256) * -(-shape[1] // 256) >= 128 and "emb" not in name:
            assert np.all(g[1:, off:off + k] == 7.0), name
            out[off:off + k] = (g[0, off:off + k].astype(np.float64) / n).astype(np.float32)
            summed.append(name)
        else:
            out[off:off + k] = O.shared_gradient(g[:, off:off + k])
        off += k
    return out, summed


@pytest.mark.parametrize("cfg,batch,n,bf16", [(TINY, 3, 3, False), (SMALL, 4, 4, False), (SMALL, 4, 4, True), (FUSE3, 2, 2, True),
                                              (BIGV, 2, 3, False), (BIGV, 2, 3, True)])
def test_shared_gradient_mode_applies_the_replica_mean(cfg, batch, n, bf16):
    """Algorithm 1's gradient exchange on the transformer: a weight matrix large enough to fill the chip is formed as one
    product over the rows of all replicas (their sum, in plane 0 of the gradient buffer), every other gradient per
    replica, and the update applies the replica mean of either to every replica at its own rate."""
    d = base(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, grad_mode=O.GRAD_SHARED)
    run = TfRun(d, cfg, batch, bf16=bf16)
    for t in range(1, 6):
        run.orc.theta = run.theta.cpu().numpy()[:, :run.P].copy()
        run.orc.m = run.m.cpu().numpy()[:, :run.P].copy()
        run.orc.v = run.v.cpu().numpy()[:, :run.P].copy()
        run.g.fill_(7.0)
        ids, tgt, gl = run.forward_backward(t)
        losses, grads = run.oracle_grads(run.orc.theta, ids, tgt, t)
        gbar = O.shared_gradient(grads)
        assert np.max(np.abs(gl - losses)) <= (1e-2 if bf16 else 2e-5)
        g0, summed = device_mean_gradient(cfg, run.g.cpu().numpy()[:, :run.P], n)
        assert len(summed) == (1 if cfg is BIGV else 0), summed
        if bf16:
            check_bf16_gradients(cfg, g0, gbar, 4e-2, ("shared", cfg["d_model"], t))
        else:
            bad = {k: v for k, v in per_tensor_errors(cfg, g0, gbar).items() if v > 2e-5}
            assert not bad, (t, bad)
        run.finish_step(t, grads, losses, fuse=(t == 4))
        # AdamW from identical state: bounded over the tensor (its early steps magnify a rounding difference of a
        # near-zero gradient entry up to the full step lr); the gradient check above is the entry-wise one
        assert norm_err(run.theta.cpu().numpy()[:, :run.P], run.orc.theta) <= (1e-3 if not bf16 else 1e-2), t
    st = H.hdet_get_state(run.h)
    assert st.k == run.orc.k == 1
    run.close()
