"""hdet_train_step: forward, backward and the fan-out update in one call, with the update of a weight matrix applied
inside the product that forms its gradient (Eq. 2 on the tile; Algorithm 1's "Forward + backward" and update lines).

Two kinds of check: (1) against the oracle, from the device's own state before the call (the gradient itself never
reaches memory, so parameters and moments after the step are what can be compared); (2) against the library's own
two-call sequence hdet_forward_backward + hdet_fanout_step, bit for bit, over runs with converge and controller."""
import numpy as np
import pytest
import torch

import hdet_inputs as I
import paper_2604_24708_amd as H
from harness import norm_err
from oracle import hdet_oracle as O
from oracle import mlp_oracle as M
from test_gpu_mlp import MlpRun, cfg0
from test_gpu_transformer import FUSE3, SMALL, TfRun, base

pytestmark = pytest.mark.gpu

WD = (O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))


def snapshot(run):
    out = [run.theta.clone(), run.m.clone(), run.v.clone()]
    if run.shadow is not None:
        out.append(run.shadow.clone())
    return out


def assert_same_bits(a, b, what):
    for x, y, name in zip(snapshot(a), snapshot(b), ("theta", "m", "v", "bf16 copy")):
        assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x.view(torch.int16),
                           y.view(torch.int32) if y.dtype == torch.float32 else y.view(torch.int16)), (what, name)


def same_state(a, b):
    sa, sb = H.hdet_get_state(a.h), H.hdet_get_state(b.h)
    assert (sa.t, sa.k, sa.controller_active) == (sb.t, sb.k, sb.controller_active)
    for j in range(sa.n_channels):
        assert sa.base[j] == sb.base[j] and sa.vel[j] == sb.vel[j]
        assert [sa.perm[j][r] for r in range(sa.n_replicas)] == [sb.perm[j][r] for r in range(sa.n_replicas)]
    assert [sa.l_step[r] for r in range(sa.n_replicas)] == [sb.l_step[r] for r in range(sa.n_replicas)]


def weight_slices(widths):
    """(offset, size, fusable): the matrix-core product that can carry the update takes matrices whose two dimensions are
    multiples of 8 (whole 16-byte chunks of bfloat16); the others keep the separate gradient and update."""
    off, out = 0, []
    for i in range(len(widths) - 1):
        out.append((off, widths[i + 1] * widths[i], widths[i + 1] % 8 == 0 and widths[i] % 8 == 0))
        off += widths[i + 1] * widths[i] + widths[i + 1]
    return out


@pytest.mark.parametrize("widths,batch,n,extra,groups", [([256, 384, 136], 160, 4, [], None),
                                                          ([70, 200, 36], 50, 3, [WD], None), ([72, 200, 36], 50, 3, [WD], None),
                                                          ([128, 256, 256, 64], 96, 2, [WD], "layers"),
                                                          ([128, 256, 256, 64], 96, 2, [], "split")])
def test_mlp_one_call_equals_two_calls_bit_for_bit(widths, batch, n, extra, groups):
    d = cfg0(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, total_steps=12, warm_steps=4, weight_decay=0.01, extra=extra)
    split = None
    if groups == "layers":      # one rate channel per layer (weights + bias): group ends at the layer boundaries
        ends, off = [], 0
        for i in range(len(widths) - 1):
            off += widths[i + 1] * widths[i] + widths[i + 1]
            ends.append(off)
        d["group_end"] = ends
    if groups == "split":       # a group boundary inside the first matrix: that matrix keeps the separate update
        split = 0
        d["group_end"] = [widths[1] * widths[0] // 2, I.mlp_param_count(widths)]
    two, one = MlpRun(d, widths, batch, bf16=True), MlpRun(d, widths, batch, bf16=True)
    H.hdet_set_launch_shape(one.h, 4, 0)       # products of any size carry their update (by default only chip-filling ones)
    for t in range(1, 13):
        x, y = I.mlp_batch(n, batch, widths[0], I.SEED_DATA, t, widths, I.SEED_TEACHER)
        xd, yd = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0")
        flags = H.HDET_FUSE_CONVERGE if t in (4, 12) else 0
        l2 = H.hdet_forward_backward(two.h, xd, yd, want_losses=True)
        H.hdet_fanout_step(two.h, None, flags)
        one.g.fill_(7.0)
        l1 = H.hdet_train_step(one.h, xd, yd, flags, want_losses=True)
        assert [l1[r] for r in range(n)] == [l2[r] for r in range(n)], t
        # the weight gradients were never written; the bias gradients were
        g = one.g.cpu().numpy()
        for off, size, fusable in weight_slices(widths):
            fusable = fusable and off != split
            assert np.all(g[:, off:off + size] == 7.0) if fusable else not np.any(g[:, off:off + size] == 7.0), (t, off)
            assert not np.any(g[:, off + size:off + size + 4] == 7.0), (t, off)
        for r in (two, one):
            if t % d["sync_interval"] == 0:
                H.hdet_converge(r.h)
                H.hdet_autolr_update(r.h, None)
        assert_same_bits(two, one, t)
        same_state(two, one)
    assert H.hdet_get_state(one.h).k == 3
    two.close(); one.close()


def test_mlp_one_call_against_the_oracle_from_the_device_state():
    """Each step: the oracle takes the device's parameters and moments before the call, forms its own mixed-precision
    gradient there and applies Eq. 2 / AdamW at the replica's rate; parameters and moments after the step are compared
    (AdamW from identical state: bounded over the tensor, as in the other trajectory tests)."""
    widths, batch, n = [256, 384, 136], 160, 4
    d = cfg0(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, total_steps=8, warm_steps=4, weight_decay=0.01)
    run = MlpRun(d, widths, batch, bf16=True)
    H.hdet_set_launch_shape(run.h, 4, 0)
    P = run.P
    for t in range(1, 9):
        x, y = I.mlp_batch(n, batch, widths[0], I.SEED_DATA, t, widths, I.SEED_TEACHER)
        run.orc.theta = run.theta.cpu().numpy()[:, :P].copy()
        run.orc.m = run.m.cpu().numpy()[:, :P].copy()
        run.orc.v = run.v.cpu().numpy()[:, :P].copy()
        per_replica = [M.mlp_loss_and_grad(run.orc.theta[r], x[r], y[r], widths, bf16=True) for r in range(n)]
        out = H.hdet_train_step(run.h, torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0"), 0, want_losses=True)
        losses = np.array([o[0] for o in per_replica])
        assert np.max(np.abs(np.array([out[r] for r in range(n)]) - losses)) <= 2e-3, t
        run.orc.fanout_step(np.stack([o[1] for o in per_replica]), losses)
        if t % d["sync_interval"] == 0:
            H.hdet_converge(run.h); run.orc.converge()
            H.hdet_autolr_update(run.h, None); run.orc.autolr_update()
        assert norm_err(run.theta.cpu().numpy()[:, :P], run.orc.theta) <= 1e-3, t
        assert norm_err(run.m.cpu().numpy()[:, :P], run.orc.m) <= 2e-2, t
        assert norm_err(run.v.cpu().numpy()[:, :P], run.orc.v) <= 4e-2, t
    st = H.hdet_get_state(run.h)
    assert st.k == run.orc.k == 2
    run.close()


@pytest.mark.parametrize("cfg,batch,n,extra", [(SMALL, 4, 4, []), (FUSE3, 2, 2, [(O.CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45), WD])])
def test_transformer_one_call_equals_two_calls_bit_for_bit(cfg, batch, n, extra):
    d = base(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, weight_decay=0.01, extra=extra)
    two, one = TfRun(d, cfg, batch, bf16=True), TfRun(d, cfg, batch, bf16=True)
    H.hdet_set_launch_shape(one.h, 4, 0)
    shapes, off, mats = I.transformer_shapes(cfg), 0, []
    for name, shape in shapes:
        k = int(np.prod(shape))
        if name.startswith("w_"):
            mats.append((name, off, k, shape[0] % 8 == 0 and shape[1] % 8 == 0))       # see weight_slices
        off += k
    for t in range(1, 9):
        ids, tgt = I.zipf_tokens(n, batch, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, t)
        xd, yd = torch.from_numpy(ids).to("cuda:0"), torch.from_numpy(tgt).to("cuda:0")
        flags = H.HDET_FUSE_CONVERGE if t == 4 else 0
        l2 = H.hdet_forward_backward(two.h, xd, yd, want_losses=True)
        H.hdet_fanout_step(two.h, None, flags)
        one.g.fill_(7.0)
        l1 = H.hdet_train_step(one.h, xd, yd, flags, want_losses=True)
        assert [l1[r] for r in range(n)] == [l2[r] for r in range(n)], t
        g = one.g.cpu().numpy()
        for name, o, k, fusable in mats:
            assert np.all(g[:, o:o + k] == 7.0) if fusable else not np.any(g[:, o:o + k] == 7.0), (t, name)
        for r in (two, one):
            if t % d["sync_interval"] == 0:
                H.hdet_converge(r.h)
                H.hdet_autolr_update(r.h, None)
        assert_same_bits(two, one, t)
        same_state(two, one)
    two.close(); one.close()


def test_configurations_that_cannot_fuse_take_the_ordinary_update():
    """fp32, SGD-momentum or shared gradients: the call is the two calls in sequence, gradients included."""
    widths, batch, n = [64, 128, 10], 32, 4
    for kw, bf16 in ((dict(), False), (dict(optimizer=O.ADAMW, lr_max=2e-3, grad_mode=O.GRAD_SHARED), True), (dict(), True)):
        d = cfg0(n_replicas=n, total_steps=8, warm_steps=4, **kw)
        two, one = MlpRun(d, widths, batch, bf16=bf16), MlpRun(d, widths, batch, bf16=bf16)
        for t in range(1, 9):
            x, y = I.mlp_batch(n, batch, widths[0], I.SEED_DATA, t, widths, I.SEED_TEACHER)
            xd, yd = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0")
            H.hdet_forward_backward(two.h, xd, yd)
            H.hdet_fanout_step(two.h, None, H.HDET_FUSE_CONVERGE)
            H.hdet_train_step(one.h, xd, yd, H.HDET_FUSE_CONVERGE)
            assert torch.equal(two.g, one.g), (kw, t)
            for r in (two, one):
                if t % d["sync_interval"] == 0:
                    H.hdet_converge(r.h)
                    H.hdet_autolr_update(r.h, None)
            assert torch.equal(two.theta, one.theta) and torch.equal(two.m, one.m), (kw, t)
        two.close(); one.close()


def test_argument_errors():
    d = cfg0(n_replicas=2, total_steps=2)
    run = MlpRun(d, [64, 128, 10], 32)
    x, y = I.mlp_batch(2, 32, 64, I.SEED_DATA, 1, [64, 128, 10], I.SEED_TEACHER)
    xd, yd = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0")
    with pytest.raises(H.HdetError):
        H.hdet_train_step(run.h, xd, yd, 2)                 # unknown flag
    with pytest.raises(H.HdetError):
        H.hdet_train_step(run.h, None, yd, 0)
    H.hdet_train_step(run.h, xd, yd, 0)
    H.hdet_train_step(run.h, xd, yd, 0)
    with pytest.raises(H.HdetError):
        H.hdet_train_step(run.h, xd, yd, 0)                 # all total_steps updates are done
    run.close()


def test_small_products_keep_the_separate_update_by_default():
    """Without the tuning flag a product with fewer 256 x 256 tiles than the chip has compute units is not worth fusing:
    its gradient is written and the plane-wide update applies it -- same bits either way."""
    widths, batch, n = [256, 384, 136], 160, 4
    d = cfg0(n_replicas=n, optimizer=O.ADAMW, lr_max=2e-3, total_steps=4, warm_steps=2, weight_decay=0.01)
    forced, default = MlpRun(d, widths, batch, bf16=True), MlpRun(d, widths, batch, bf16=True)
    H.hdet_set_launch_shape(forced.h, 4, 0)
    for t in range(1, 5):
        x, y = I.mlp_batch(n, batch, widths[0], I.SEED_DATA, t, widths, I.SEED_TEACHER)
        xd, yd = torch.from_numpy(x).to("cuda:0"), torch.from_numpy(y).to("cuda:0")
        default.g.fill_(7.0)
        H.hdet_train_step(forced.h, xd, yd, 0)
        H.hdet_train_step(default.h, xd, yd, 0)
        assert not torch.any(default.g[:, :default.P] == 7.0), t
        for r in (forced, default):
            if t % d["sync_interval"] == 0:
                H.hdet_converge(r.h)
                H.hdet_autolr_update(r.h, None)
        assert_same_bits(forced, default, t)
    forced.close(); default.close()
