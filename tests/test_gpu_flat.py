"""Parity of the HIP path with the CPU oracle on flat parameter buffers: fan-out update
(SGD-momentum / AdamW, shared and per-replica gradients), converge (standalone and fused
into the update) and the auto-LR controller, element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import hdet_inputs as I
import paper_2604_24708_amd as H
from harness import check_state, library_config, oracle_config, rel_err, rel_err_detail
from oracle import hdet_oracle as O

pytestmark = pytest.mark.gpu

TOL_STEP = 1e-5      # max relative error per step on fp32 parameter paths
TOL_100 = 1e-4       # after 100 steps


def tol_at(t):
    """Bound on a trajectory compared after t steps run separately on both sides: each step
    may add the per-step 1e-5, and the total stays within the 100-step bound of 1e-4."""
    return min(t * TOL_STEP, TOL_100)


def base_cfg(**kw):
    d = dict(n_replicas=4, total_steps=24, sync_interval=4, warm_steps=8, lr_max=0.05, alpha=0.2,
             autolr_enabled=True, optimizer=O.ADAMW, weight_decay=0.01, grad_mode=O.GRAD_PER_REPLICA,
             seed=7)
    d.update(kw)
    return d


class FlatRun:
    """Same run on both sides; `stride` > P leaves padding that must stay untouched."""

    def __init__(self, d, P, stride=None, variant=0, blocks=0, grad_std=0.1):
        self.d, self.P = d, P
        self.n = d["n_replicas"]
        self.stride = stride or ((P + 3) // 4) * 4
        self.grad_std = grad_std
        dev = "cuda:0"
        th0 = I.flat_theta0(self.n, P, 5)
        self.orc = O.HDETOracle(oracle_config(d), th0)
        self.pad = np.float32(123.25)
        host = np.full((self.n, self.stride), self.pad, dtype=np.float32)
        host[:, :P] = th0
        self.theta = torch.from_numpy(host).to(dev)
        self.shared_state = bool(d.get("shared_opt_state", False))     # one plane of moments for all replicas
        planes = 1 if self.shared_state else self.n
        self.m = torch.zeros((planes, self.stride), device=dev)
        self.v = torch.zeros((planes, self.stride), device=dev)
        self.g = torch.zeros((self.n, self.stride), device=dev)
        cfg = library_config(d, n_params=P, model_kind=H.HDET_FLAT)
        self.h = H.hdet_create(cfg, self.theta, self.m, self.v if d["optimizer"] == O.ADAMW else None,
                               plane_stride=self.stride)
        if variant or blocks:
            H.hdet_set_launch_shape(self.h, variant, blocks)

    def step(self, t, fuse):
        n, P = self.n, self.P
        # size of the operands each parameter has been formed from so far: the largest value it (any replica of
        # it: a converge mixes them) has had, and the largest step it has taken
        prev = np.max(np.abs(self.orc.theta.astype(np.float64)), axis=0)
        self.theta_scale = np.maximum(getattr(self, "theta_scale", prev), prev)
        self.theta_prev = self.orc.theta.copy()
        g = I.flat_grads(n, P, 99, t, std=self.grad_std)
        losses = I.flat_losses(n, t)
        self.g[:, :P] = torch.from_numpy(g).to(self.g.device)
        H.hdet_fanout_step(self.h, self.g, H.HDET_FUSE_CONVERGE if fuse else 0)
        self.orc.fanout_step(g, losses)
        if t % self.d["sync_interval"] == 0:
            H.hdet_converge(self.h)
            self.orc.converge()
            lr_interval = self.orc.l_acc / self.d["sync_interval"]
            H.hdet_autolr_update(self.h, lr_interval.tolist())
            self.orc.autolr_update()

    def compare(self, tol):
        P = self.P
        th = self.theta.cpu().numpy()
        err, floored = rel_err_detail(th[:, :P], self.orc.theta, tol)
        assert err <= tol
        # The entries that pass only thanks to the floor of the error metric must be exactly the case the
        # floor exists for: a result much smaller than the operands it was formed from (a parameter that
        # has been larger, or a step as large as the parameter, cancelling), off by no more than a few fp32
        # roundings of those operands per step run -- not a small entry that is simply wrong.
        self.floored_entries = getattr(self, "floored_entries", 0) + len(floored)
        if len(floored) and hasattr(self, "theta_prev"):
            r, i = floored[:, 0], floored[:, 1]
            new = self.orc.theta.astype(np.float64)[r, i]
            moved = np.abs(self.theta_prev.astype(np.float64)[r, i] - new)
            self.theta_scale[i] = np.maximum(self.theta_scale[i], moved)
            scale = self.theta_scale[i]
            diff = np.abs(th[r, i].astype(np.float64) - new)
            assert np.all(np.abs(new) < scale), "a floored entry is not smaller than its operands"
            assert np.all(diff <= max(self.orc.t, 1) * 16.0 * 2.0 ** -24 * scale), "a floored entry is off by more than fp32 roundings of its operands"
        om, ov = (self.orc.m[:1], self.orc.v[:1]) if self.shared_state else (self.orc.m, self.orc.v)
        assert rel_err(self.m.cpu().numpy()[:, :P], om) <= tol
        if self.d["optimizer"] == O.ADAMW:
            assert rel_err(self.v.cpu().numpy()[:, :P], ov) <= tol
        if self.shared_state:
            assert np.all(self.m.cpu().numpy()[:, P:] == 0) and np.all(self.v.cpu().numpy()[:, P:] == 0)
        assert np.all(th[:, P:] == self.pad)
        check_state(H.hdet_get_state(self.h), self.orc)

    def close(self):
        H.hdet_destroy(self.h)


@pytest.mark.parametrize("opt", [O.SGDM, O.ADAMW])
@pytest.mark.parametrize("mode", [O.GRAD_SHARED, O.GRAD_PER_REPLICA])
@pytest.mark.parametrize("n,P", [(1, 5), (2, 1), (3, 1023), (4, 4), (4, 70001), (8, 3), (8, 262147), (5, 4099)])
def test_update_converge_controller_parity(opt, mode, n, P):
    d = base_cfg(n_replicas=n, optimizer=opt, grad_mode=mode)
    run = FlatRun(d, P)
    for t in range(1, 17):
        run.step(t, fuse=(t % 8 == 0))          # alternate fused and standalone converge
        run.compare(tol_at(t))
    st = H.hdet_get_state(run.h)
    assert st.k == 3 and st.controller_active == 1
    run.close()


@pytest.mark.parametrize("mode", [O.GRAD_SHARED, O.GRAD_PER_REPLICA])
@pytest.mark.parametrize("n", [3, 8, 16, 17, 64])
def test_kernel_variants_agree_bit_for_bit(n, mode):
    """The general loop kernel (forced, small grid) and the default kernels (plane / wave for
    N <= 16, loop beyond) must give identical bits, and both match the oracle."""
    d = base_cfg(n_replicas=n, grad_mode=mode)
    a = FlatRun(d, 50003, stride=50176, variant=1, blocks=7)
    b = FlatRun(d, 50003, stride=50176)
    for t in range(1, 6):
        a.step(t, fuse=(t == 4))
        b.step(t, fuse=(t == 4))
        a.compare(tol_at(t))
        assert torch.equal(a.theta, b.theta) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v)
    a.close(); b.close()


def test_single_step_error_is_within_1e5():
    """One update from identical state: the per-step bound itself."""
    for opt in (O.SGDM, O.ADAMW):
        d = base_cfg(n_replicas=8, optimizer=opt, total_steps=200)
        run = FlatRun(d, 100001)
        for t in range(1, 4):
            # restart both sides from the oracle's state so that only one step's error shows
            run.theta[:, :run.P] = torch.from_numpy(run.orc.theta).to(run.theta.device)
            run.m[:, :run.P] = torch.from_numpy(run.orc.m).to(run.theta.device)
            run.v[:, :run.P] = torch.from_numpy(run.orc.v).to(run.theta.device)
            run.step(t, fuse=False)
            run.compare(TOL_STEP)
        run.close()


def test_hundred_steps_within_1e4():
    d = base_cfg(n_replicas=4, total_steps=100, sync_interval=5, warm_steps=30, lr_max=3e-3, alpha=0.1)
    run = FlatRun(d, 20011, grad_std=1e-3)
    for t in range(1, 101):
        run.step(t, fuse=(t % 2 == 0))
        if t % 10 == 0:
            run.compare(TOL_100)
    th = run.theta.cpu().numpy()
    assert all(np.array_equal(th[0, :run.P], th[r, :run.P]) for r in range(4))   # t = 100 is a sync step
    with pytest.raises(H.HdetError) as e:
        H.hdet_fanout_step(run.h, run.g, 0)                                      # beyond S
    assert e.value.code == H.HDET_ESTATE
    run.close()


def test_weight_decay_channel_and_three_permutations():
    extra = [(O.CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45), (O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))]
    d = base_cfg(n_replicas=8, extra=extra, lr_max=3e-3, alpha=0.15)
    run = FlatRun(d, 4099)
    for t in range(1, 21):
        run.step(t, fuse=False)
        run.compare(tol_at(t))
    st = H.hdet_get_state(run.h)
    perms = {tuple(st.perm[j][r] for r in range(8)) for j in range(3)}
    assert len(perms) == 3
    run.close()


def test_invariants_on_device():
    """alpha = 0 with identical gradients: replicas stay bit-identical and converge is a
    bit-exact no-op; fused and standalone converge give identical planes."""
    d = base_cfg(n_replicas=8, alpha=0.0, autolr_enabled=False)
    P = 30001
    run = FlatRun(d, P)
    g = I.flat_grads(1, P, 99, 1, std=0.1)
    run.g[:, :P] = torch.from_numpy(np.broadcast_to(g, (8, P)).copy()).to(run.g.device)
    for t in range(1, 5):
        H.hdet_fanout_step(run.h, run.g, 0)
    before = run.theta.clone()
    H.hdet_converge(run.h)
    assert torch.equal(before, run.theta)
    assert all(torch.equal(run.theta[0], run.theta[r]) for r in range(8))
    run.close()


def test_equal_losses_give_zero_delta():
    d = base_cfg(n_replicas=8, warm_steps=0, gamma_override=0.0)
    run = FlatRun(d, 64)
    for t in range(1, 5):
        H.hdet_fanout_step(run.h, run.g, 0)
    H.hdet_converge(run.h)
    H.hdet_autolr_update(run.h, [2.5] * 8)
    st = H.hdet_get_state(run.h)
    assert st.delta[0] == 0.0 and st.vel[0] == 0.0 and st.k == 1
    assert st.base[0] == O.onecycle_lr(3, 24, 0.05, 25.0, 1e4, 0.3)     # untouched at gamma = 0
    assert abs(sum(st.w[r] for r in range(8)) - 1.0) < 1e-15
    run.close()


def test_call_order_and_argument_errors():
    d = base_cfg()
    run = FlatRun(d, 64)
    with pytest.raises(H.HdetError) as e:
        H.hdet_autolr_update(run.h, [1.0] * 4)        # t = 0: not a sync step
    assert e.value.code == H.HDET_ESTATE
    for t in range(1, 5):
        H.hdet_fanout_step(run.h, run.g, 0)
    H.hdet_autolr_update(run.h, [1.0] * 4)
    with pytest.raises(H.HdetError) as e:
        H.hdet_autolr_update(run.h, [1.0] * 4)        # twice on one sync step
    assert e.value.code == H.HDET_ESTATE
    with pytest.raises(H.HdetError) as e:
        H.hdet_fanout_step(run.h, run.g.data_ptr() + 4, 0)      # misaligned gradients
    assert e.value.code == H.HDET_EINVAL
    with pytest.raises(H.HdetError) as e:
        H.hdet_forward_backward(run.h, run.g, run.g)            # flat handle
    assert e.value.code == H.HDET_ESTATE
    with pytest.raises(H.HdetError) as e:
        H.hdet_set_launch_shape(run.h, 8, 0)                    # no such kernel variant
    assert e.value.code == H.HDET_EINVAL
    assert "variant" in H.hdet_last_error(run.h)
    run.close()
    cfg = library_config(d, n_params=64, model_kind=H.HDET_FLAT)
    with pytest.raises(H.HdetError):
        H.hdet_create(cfg, run.theta, run.m, None, plane_stride=64)       # AdamW without v
    with pytest.raises(H.HdetError):
        H.hdet_create(cfg, run.theta.data_ptr() + 4, run.m, run.v, plane_stride=64)


def test_nonfinite_loss_skips_the_controller():
    d = base_cfg(warm_steps=0)
    run = FlatRun(d, 64)
    for t in range(1, 5):
        H.hdet_fanout_step(run.h, run.g, 0)
        run.orc.fanout_step(np.zeros((4, 64), np.float32), [0.0] * 4)
    with pytest.raises(H.HdetError) as e:
        H.hdet_autolr_update(run.h, [1.0, float("nan"), 1.0, 1.0])
    assert e.value.code == H.HDET_ENONFINITE                     # reported; the sync step still counts as processed
    run.orc.autolr_update([1.0, float("nan"), 1.0, 1.0])
    st = H.hdet_get_state(run.h)
    assert st.nonfinite == 1 and st.k == 0 and st.controller_active == 0 and st.autolr_done == 1
    check_state(st, run.orc)
    with pytest.raises(H.HdetError) as e:
        H.hdet_autolr_update(run.h, [1.0] * 4)
    assert e.value.code == H.HDET_ESTATE
    # the next interval is finite again: the controller takes over as if nothing had happened
    for t in range(5, 9):
        H.hdet_fanout_step(run.h, run.g, 0)
        run.orc.fanout_step(np.zeros((4, 64), np.float32), [0.0] * 4)
    H.hdet_autolr_update(run.h, [1.0, 1.1, 0.9, 1.0])
    run.orc.autolr_update([1.0, 1.1, 0.9, 1.0])
    check_state(H.hdet_get_state(run.h), run.orc)
    # before warm_steps a non-finite loss is only recorded as L_r: the controller was not due, no error
    d2 = base_cfg(warm_steps=8)
    run2 = FlatRun(d2, 64)
    for t in range(1, 5):
        H.hdet_fanout_step(run2.h, run2.g, 0)
    H.hdet_autolr_update(run2.h, [1.0, float("inf"), 1.0, 1.0])
    assert H.hdet_get_state(run2.h).nonfinite == 0
    with pytest.raises(ValueError):
        H.hdet_autolr_update(run2.h, [1.0] * 3)                  # the binding refuses a list that is not N long
    run.close(); run2.close()


def test_state_saved_between_update_and_controller_call_resumes():
    """A snapshot taken on a sync step after hdet_fanout_step but before hdet_autolr_update carries
    autolr_done = 0, and the handle it is loaded into still runs the controller for that sync step."""
    d = base_cfg(n_replicas=4, warm_steps=0)
    a = FlatRun(d, 257)
    for t in range(1, 4):
        a.step(t, fuse=False)
    g = I.flat_grads(4, 257, 99, 4, std=0.1)
    a.g[:, :257] = torch.from_numpy(g).to(a.g.device)
    H.hdet_fanout_step(a.h, a.g, 0)
    H.hdet_converge(a.h)
    st = H.hdet_get_state(a.h)
    assert st.t == 4 and st.autolr_done == 0
    b = FlatRun(d, 257)
    b.theta.copy_(a.theta); b.m.copy_(a.m); b.v.copy_(a.v)
    H.hdet_set_state(b.h, st)
    losses = [1.0, 1.2, 0.8, 1.1]
    H.hdet_autolr_update(a.h, losses)
    H.hdet_autolr_update(b.h, losses)                            # would be HDET_ESTATE if the flag were guessed from t
    sa, sb = H.hdet_get_state(a.h), H.hdet_get_state(b.h)
    assert sa.k == sb.k == 1 and sa.base[0] == sb.base[0] and sb.autolr_done == 1
    assert [sa.perm[0][r] for r in range(4)] == [sb.perm[0][r] for r in range(4)]
    H.hdet_set_state(b.h, sb)
    with pytest.raises(H.HdetError) as e:
        H.hdet_autolr_update(b.h, losses)                        # a snapshot taken after the call keeps refusing a second one
    assert e.value.code == H.HDET_ESTATE
    a.close(); b.close()


def test_channel_base_driven_to_its_upper_bound_stays_in_range():
    """A dropout channel whose centre value the controller pushes up (large lambda, losses falling with
    the value) is clamped at hi; every replica's value stays below hi * (1 + alpha) < 1, and the state
    still matches the oracle bit for bit."""
    extra = [(O.CH_DROPOUT, 0.3, 1.0, 50.0, 0.0, 0.45)]
    d = base_cfg(n_replicas=4, warm_steps=0, extra=extra, total_steps=40)
    run = FlatRun(d, 64)
    hit = False
    for t in range(1, 25):
        H.hdet_fanout_step(run.h, run.g, 0)
        run.orc.fanout_step(np.zeros((4, 64), np.float32), [0.0] * 4)
        if t % 4 == 0:
            st = H.hdet_get_state(run.h)
            # the replica with the largest dropout value reports the lowest loss
            vals = [st.base[1] * st.rho[1][st.perm[1][r]] for r in range(4)]
            losses = [2.0 - v for v in vals]
            H.hdet_autolr_update(run.h, losses)
            run.orc.autolr_update(losses)
            st = H.hdet_get_state(run.h)
            check_state(st, run.orc)
            assert 0.0 <= st.base[1] <= 0.45
            assert all(st.base[1] * st.rho[1][st.perm[1][r]] < 1.0 for r in range(4))
            hit = hit or st.base[1] == 0.45
    assert hit
    run.close()


def test_state_round_trip_resumes_bit_exactly():
    d = base_cfg(n_replicas=4)
    a = FlatRun(d, 1001)
    for t in range(1, 13):
        a.step(t, fuse=False)
    st = H.hdet_get_state(a.h)
    b = FlatRun(d, 1001)
    b.theta.copy_(a.theta); b.m.copy_(a.m); b.v.copy_(a.v)
    H.hdet_set_state(b.h, st)
    for t in range(13, 21):
        a.step(t, fuse=False)
        g = I.flat_grads(4, 1001, 99, t, std=0.1)
        b.g[:, :1001] = torch.from_numpy(g).to(b.g.device)
        H.hdet_fanout_step(b.h, b.g, 0)
        if t % 4 == 0:
            H.hdet_converge(b.h)
            H.hdet_autolr_update(b.h, [H.hdet_get_state(a.h).l_last[r] for r in range(4)])
    assert torch.equal(a.theta, b.theta) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v)
    sa, sb = H.hdet_get_state(a.h), H.hdet_get_state(b.h)
    assert sa.k == sb.k and sa.base[0] == sb.base[0] and sa.vel[0] == sb.vel[0]
    assert [sa.perm[0][r] for r in range(4)] == [sb.perm[0][r] for r in range(4)]
    a.close(); b.close()


@pytest.mark.parametrize("n,P", [(4, 100003), (8, 5), (3, 4096)])
def test_warm_noisy_init_matches_oracle(n, P):
    """Eq. 10: every replica starts from the checkpoint plus its own Gaussian perturbation."""
    d = base_cfg(n_replicas=n)
    run = FlatRun(d, P)
    theta0 = (np.random.default_rng(3).standard_normal(P) * 0.05).astype(np.float32)
    t0 = torch.from_numpy(theta0).to("cuda:0")
    H.hdet_warm_init(run.h, t0, 0.01, 4242)
    ref = O.warm_noisy_init(theta0, n, 0.01, 4242)
    th = run.theta.cpu().numpy()
    assert rel_err(th[:, :P], ref) <= 1e-6
    assert np.all(th[:, P:] == run.pad)
    eps = th[:, :P].astype(np.float64) - theta0
    if P > 1000:
        assert np.sum(eps[0] ** 2) == pytest.approx(1e-4 * np.sum(theta0.astype(np.float64) ** 2), rel=0.05)
        assert abs(np.corrcoef(eps[0], eps[1])[0, 1]) < 0.02
    with pytest.raises(H.HdetError):
        H.hdet_warm_init(run.h, run.theta, 0.01, 1)              # overlaps the parameter planes
    H.hdet_fanout_step(run.h, run.g, 0)
    with pytest.raises(H.HdetError) as e:
        H.hdet_warm_init(run.h, t0, 0.01, 4242)                  # only before the first update
    assert e.value.code == H.HDET_ESTATE
    run.close()


@pytest.mark.parametrize("opt,mode", [(O.ADAMW, O.GRAD_PER_REPLICA), (O.SGDM, O.GRAD_SHARED)])
def test_parameter_groups_with_own_rate_channels(opt, mode):
    """Four parameter groups, each with its own base rate, velocity and permutation, plus a
    weight-decay channel: 5 channels driven by the same weights."""
    P = 70001
    extra = [(O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))]
    d = base_cfg(n_replicas=8, optimizer=opt, grad_mode=mode, group_end=[4096, 20000, 50004, P], extra=extra,
                 total_steps=400)
    run = FlatRun(d, P)
    for t in range(1, 21):
        run.step(t, fuse=(t % 8 == 0))
        run.compare(tol_at(t))
    st = H.hdet_get_state(run.h)
    assert st.n_channels == 5 and st.k == 4
    assert len({tuple(st.perm[j][r] for r in range(8)) for j in range(5)}) >= 4
    assert len({st.base[j] for j in range(4)}) == 4 and min(st.base[j] for j in range(4)) > 0.0
    run.close()
    bad = base_cfg(n_replicas=8, group_end=[4098, P])             # not a multiple of 4
    with pytest.raises(H.HdetError):
        FlatRun(bad, P)


@pytest.mark.parametrize("n,P", [(1, 5), (3, 1023), (8, 70001), (8, 262147), (20, 4099)])
def test_shared_optimizer_state_matches_per_replica_state(n, P):
    """AdamW on the mean gradient: the moments do not depend on the replica, so one plane of each
    gives the oracle's trajectory (whose per-replica moments are identical) and, bit for bit, the
    trajectory of the library's own per-replica-state run."""
    d = base_cfg(n_replicas=n, optimizer=O.ADAMW, grad_mode=O.GRAD_SHARED, shared_opt_state=True,
                 extra=[(O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))])
    run = FlatRun(d, P)
    ref = FlatRun(dict(d, shared_opt_state=False), P)
    for t in range(1, 17):
        run.step(t, fuse=(t % 8 == 0))
        ref.step(t, fuse=(t % 8 == 0))
        run.compare(tol_at(t))
        assert np.all(run.orc.m == run.orc.m[:1]) and np.all(run.orc.v == run.orc.v[:1])
    assert torch.equal(run.theta, ref.theta)
    assert torch.equal(run.m[0], ref.m[0]) and torch.equal(run.v[0], ref.v[n - 1])
    run.close(); ref.close()
    for bad in (dict(optimizer=O.SGDM, grad_mode=O.GRAD_SHARED), dict(optimizer=O.ADAMW, grad_mode=O.GRAD_PER_REPLICA)):
        with pytest.raises(H.HdetError):
            FlatRun(base_cfg(n_replicas=2, shared_opt_state=True, **bad), 64)


def test_shared_optimizer_state_with_parameter_groups_and_loop_kernel():
    P = 50004
    d = base_cfg(n_replicas=8, optimizer=O.ADAMW, grad_mode=O.GRAD_SHARED, shared_opt_state=True,
                 group_end=[4096, 20000, P], total_steps=400)
    a, b = FlatRun(d, P), FlatRun(d, P, variant=1, blocks=7)
    for t in range(1, 13):
        a.step(t, fuse=(t % 8 == 0)); b.step(t, fuse=(t % 8 == 0))
        a.compare(tol_at(t))
    assert torch.equal(a.theta, b.theta) and torch.equal(a.m, b.m) and torch.equal(a.v, b.v)
    a.close(); b.close()


def test_reshuffle_every_sync_before_and_after_hand_over():
    """Fig. 1's reading: permutations change at every sync step from the first one on (the
    controller starts at t = 8 here), numbered by the sync step; parity includes them."""
    d = base_cfg(n_replicas=8, reshuffle_every_sync=True, extra=[(O.CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))])
    run = FlatRun(d, 4099)
    perms = []
    for t in range(1, 21):
        run.step(t, fuse=False)
        run.compare(tol_at(t))
        if t % 4 == 0:
            st = H.hdet_get_state(run.h)
            perms.append(tuple(st.perm[0][r] for r in range(8)))
            assert list(perms[-1]) == O.permutation(7, t // 4, 0, 8).tolist()
    assert perms[0] != tuple(range(8)) and len(set(perms)) == len(perms)
    assert H.hdet_get_state(run.h).k == 4
    run.close()
