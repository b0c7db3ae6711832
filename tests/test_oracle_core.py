"""Pins for oracle/hdet_oracle.py: values the paper prints, closed forms, invariants,
library special cases and brute force.  CPU only."""
import itertools
import math

import numpy as np
import pytest
import torch

from conftest import load_golden
from oracle import hdet_oracle as O
import hdet_inputs as I


# ---------------------------------------------------------------- Eq. 1 spread
def test_spread_paper_worked_example():
    g = load_golden("spread_n8.txt")
    n = int(g["n"][0])
    alpha = g["alpha_num_den"][0] / g["alpha_num_den"][1]
    lr = O.spread_multipliers(n, alpha) * g["eta_max"][0]
    assert lr[0] == pytest.approx(g["lowest"][0], rel=1e-12)
    assert lr[-1] == pytest.approx(g["highest"][0], rel=1e-12)
    assert lr.mean() == pytest.approx(g["mean"][0], rel=1e-12)
    # evenly spaced in between: 8.000e-4, 8.286e-4, ..., 1.000e-3
    assert np.allclose(np.diff(lr), (1e-3 - 8e-4) / 7, rtol=1e-10)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 8, 16, 33])
@pytest.mark.parametrize("alpha", [0.0, 0.1, 0.2, 1.0])
def test_spread_invariants(n, alpha):
    rho = O.spread_multipliers(n, alpha)
    assert rho.sum() == pytest.approx(n, rel=1e-14)             # sum rho = N
    assert np.all(rho >= 1 - alpha - 1e-15) and np.all(rho <= 1 + alpha + 1e-15)
    assert np.allclose(rho + rho[::-1], 2.0, atol=1e-15)        # symmetric about 1
    if n > 1:
        assert rho[0] == pytest.approx(1 - alpha) and rho[-1] == pytest.approx(1 + alpha)
        assert np.all(np.diff(rho) >= 0)
    else:
        assert rho[0] == 1.0                                    # delta = 1/2, r - 0 = 0


def test_spread_closed_forms():
    assert np.allclose(O.spread_multipliers(2, 0.3), [0.7, 1.3])
    assert np.allclose(O.spread_multipliers(4, 0.2), [0.8, 1 - 0.2 / 3, 1 + 0.2 / 3, 1.2])
    assert np.all(O.spread_multipliers(8, 0.0) == 1.0)           # alpha = 0: plain DDP


# ---------------------------------------------------------------- one-cycle base schedule
def test_onecycle_endpoints_midpoints_monotone():
    S, lr_max, fd, ff, p = 40, 0.05, 25.0, 1e4, 0.3
    f = lambda i: O.onecycle_lr(i, S, lr_max, fd, ff, p)
    assert f(0) == pytest.approx(lr_max / fd, rel=1e-14)
    assert f(11) == pytest.approx(lr_max, rel=1e-14)             # p*S - 1 = 11
    assert f(S - 1) == pytest.approx(lr_max / (fd * ff), rel=1e-9)
    up = [f(i) for i in range(0, 12)]
    down = [f(i) for i in range(11, S)]
    assert all(a < b for a, b in zip(up, up[1:]))
    assert all(a > b for a, b in zip(down, down[1:]))
    # half-way through a phase the cosine term vanishes: arithmetic mean of the phase ends
    assert O.onecycle_lr(5.5, S, lr_max, fd, ff, p) == pytest.approx((lr_max / fd + lr_max) / 2)
    assert O.onecycle_lr(11 + 14, S, lr_max, fd, ff, p) == pytest.approx(
        (lr_max + lr_max / (fd * ff)) / 2)


@pytest.mark.parametrize("S,p,fd,ff", [(40, 0.3, 25.0, 1e4), (1000, 0.3, 25.0, 1e4),
                                       (100, 0.25, 10.0, 100.0), (64, 0.5, 4.0, 8.0)])
def test_onecycle_matches_library_scheduler(S, p, fd, ff):
    """The paper builds on PyTorch's OneCycleLR; the library scheduler (cosine annealing,
    two phases, momentum cycling off) must give the same curve."""
    lr_max = 3e-4
    prm = torch.nn.Parameter(torch.zeros(1))
    opt = torch.optim.SGD([prm], lr=lr_max)
    sch = torch.optim.lr_scheduler.OneCycleLR(opt, max_lr=lr_max, total_steps=S, pct_start=p,
                                              div_factor=fd, final_div_factor=ff,
                                              anneal_strategy="cos", cycle_momentum=False,
                                              three_phase=False)
    for idx in range(S):
        lib = opt.param_groups[0]["lr"]
        assert O.onecycle_lr(idx, S, lr_max, fd, ff, p) == pytest.approx(lib, rel=1e-9, abs=1e-18)
        opt.step()
        if idx + 1 < S:
            sch.step()


# ---------------------------------------------------------------- Eq. 8 decay
def test_gamma_reaches_onecycle_floor():
    S, Sw, T, fd, ff = 40, 12, 4, 25.0, 1e4
    g = O.decay_gamma(S, Sw, T, fd, ff)
    K = (S - Sw) / T
    assert 0.0 < g < 1.0                                          # a decay, not growth
    assert (1 - g) ** K == pytest.approx(1.0 / (fd * ff), rel=1e-12)
    assert g == pytest.approx(0.830619, abs=1e-6)
    # K need not be an integer
    g2 = O.decay_gamma(1000, 300, 16, fd, ff)
    assert (1 - g2) ** 43.75 == pytest.approx(4e-6, rel=1e-12)
    # with zero velocity the controller lands on eta_max / (f_div f_final) after K syncs
    eta = 0.05
    for _ in range(int(K)):
        _, eta = O.velocity_update(0.0, eta, 0.0, 0.9, g, 0.5)
    assert eta == pytest.approx(0.05 / (fd * ff), rel=1e-10)
    assert O.decay_gamma(10, 10, 2, fd, ff) == 0.0


# ---------------------------------------------------------------- Philox + permutation
def test_philox_known_answers():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        assert O.philox4x32_10(w[:4], w[4:6]) == w[6:]
        n += 1
    assert n == 3


def test_permutation_properties():
    for n in [1, 2, 3, 4, 8, 13, 64]:
        for k in range(1, 6):
            p = O.permutation(7, k, 0, n)
            assert sorted(p.tolist()) == list(range(n))
    # pure function of (seed, k, channel); channels and syncs are decorrelated
    assert np.array_equal(O.permutation(7, 3, 1, 8), O.permutation(7, 3, 1, 8))
    draws = {tuple(O.permutation(7, k, j, 8)) for k in range(1, 9) for j in range(3)}
    assert len(draws) == 24
    assert not np.array_equal(O.permutation(7, 3, 0, 8), O.permutation(8, 3, 0, 8))


def test_permutation_by_hand_from_the_known_answer_words():
    """Fisher-Yates worked by hand on the first known-answer block of the generator,
    philox((0,0,0,0), key (0,0)) = 6627e8d5 e169c58d bc57ac4c 9b00dbd8 (tests/golden/philox4x32_10_kat.txt).
    N = 4, start [0, 1, 2, 3]:
      i = 3: bound 4, every word is accepted (2^32 is a multiple of 4); 0x6627e8d5 mod 4 = 1 -> swap 3, 1: [0, 3, 2, 1]
      i = 2: bound 3, words below 0xffffffff are accepted; 0xe169c58d = 3781805453 = 3 * 1260601817 + 2 -> j = 2: no move
      i = 1: bound 2; 0xbc57ac4c is even -> j = 0 -> swap 1, 0: [3, 0, 2, 1]
    A walk from the bottom index up, a word taken out of order or a reduction without the top-down
    bound would give another ordering."""
    kat = [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    assert O.philox4x32_10((0, 0, 0, 0), (0, 0)) == kat
    it = iter(kat)
    assert O.permutation_from_words(lambda: next(it), 4).tolist() == [3, 0, 2, 1]
    # rejection: for bound 3 the word 0xffffffff (the one value at or above the largest multiple of 3) is
    # skipped and the next word is used; a plain modulo would have taken 0xffffffff mod 3 = 0
    it = iter([0x6627e8d5, 0xffffffff, 0xe169c58d, 0xbc57ac4c])
    assert O.permutation_from_words(lambda: next(it), 4).tolist() == [3, 0, 2, 1]
    it = iter([0x00000000, 0xffffffff, 0x00000001, 0x00000001])
    # i = 3: j = 0 -> [3, 1, 2, 0]; i = 2: 0xffffffff rejected, 1 mod 3 = 1 -> swap 2, 1 -> [3, 2, 1, 0]; i = 1: j = 1: no move
    assert O.permutation_from_words(lambda: next(it), 4).tolist() == [3, 2, 1, 0]
    # the keyed form consumes block 0, 1, ... of counter (block, k, channel, "HDET"), four words each in order
    words = []
    for block in range(3):
        words += O.philox4x32_10((block, 5, 2, O.PERM_STREAM), (7, 0))
    it = iter(words)
    assert O.permutation(7, 5, 2, 8).tolist() == O.permutation_from_words(lambda: next(it), 8).tolist()


def test_exp_spec_is_the_exponential_to_two_units_in_the_last_place():
    """The softmax of Eq. 4 uses a written-out exponential so that the schedule state is reproducible bit
    for bit; it must still be the exponential: checked against a 50-digit evaluation, and for the
    properties the controller relies on."""
    from decimal import Decimal, getcontext
    getcontext().prec = 50
    rng = np.random.default_rng(11)
    xs = np.concatenate([-rng.random(4000) * 708.0, -rng.random(4000) * 5.0, -rng.random(2000) * 1e-3,
                         -np.arange(0, 40) * math.log(2.0), [-708.0, -1e-300, -0.0, 0.0]])
    worst = 0.0
    for x in xs.tolist():
        e = O.exp_spec(x)
        worst = max(worst, float(abs(Decimal(e) - Decimal(x).exp()) / Decimal(math.ulp(e))))
    assert worst <= 2.0
    assert O.exp_spec(0.0) == 1.0 and O.exp_spec(-0.0) == 1.0
    assert O.exp_spec(-708.1) == 0.0 and O.exp_spec(-1e9) == 0.0 and O.exp_spec(float("-inf")) == 0.0
    grid = np.linspace(-50.0, 0.0, 20001)
    vals = np.array([O.exp_spec(x) for x in grid.tolist()])
    assert np.all(np.diff(vals) >= 0.0)
    with pytest.raises(ValueError):
        O.exp_spec(1e-3)


def test_permutation_uniform_chi2():
    """Eq. 9 asks for a uniformly random permutation: over many syncs all 24 orderings of
    N = 4 must appear equally often (chi-square, 23 dof; 99.9% quantile = 49.7)."""
    counts = {p: 0 for p in itertools.permutations(range(4))}
    trials = 4800
    for k in range(1, trials + 1):
        counts[tuple(O.permutation(12345, k, 0, 4).tolist())] += 1
    exp = trials / 24
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 49.7
    # every position sees every value about equally often for N = 8
    pos = np.zeros((8, 8))
    for k in range(1, 2001):
        p = O.permutation(99, k, 2, 8)
        pos[np.arange(8), p] += 1
    assert np.all(np.abs(pos - 250) < 5 * math.sqrt(250 * 7 / 8))


# ---------------------------------------------------------------- Eq. 2 update
def test_sgd_without_momentum_is_eq2():
    rng = np.random.default_rng(0)
    th = rng.standard_normal(50).astype(np.float32)
    g = rng.standard_normal(50).astype(np.float32)
    out, buf = O.sgdm_update(th, g, np.zeros_like(th), 0.1, 0.0, 0.0, False)
    assert np.array_equal(out, (th.astype(np.float64) - 0.1 * g.astype(np.float64)).astype(np.float32))
    assert np.array_equal(buf, g)


def test_sgdm_hand_trajectory():
    # theta=1, g=0.5 constant, mu=0.9, lr=0.1, wd=0: buf = 0.5, 0.95, 1.355; theta = 0.95, 0.855, 0.7195
    th = np.array([1.0]); buf = np.array([0.0]); g = np.array([0.5])
    exp_b = [0.5, 0.95, 1.355]; exp_t = [0.95, 0.855, 0.7195]
    for t in range(3):
        th, buf = O.sgdm_update(th, g, buf, 0.1, 0.0, 0.9, t == 0, store=np.float64)
        assert buf[0] == pytest.approx(exp_b[t], rel=1e-14)
        assert th[0] == pytest.approx(exp_t[t], rel=1e-14)
    # coupled L2: g' = g + wd*theta
    th2, b2 = O.sgdm_update(np.array([2.0]), np.array([0.5]), np.array([0.0]), 0.1, 0.25, 0.9, True,
                            store=np.float64)
    assert b2[0] == pytest.approx(1.0) and th2[0] == pytest.approx(1.9)


def test_sgdm_matches_library_optimizer():
    rng = np.random.default_rng(1)
    th0 = rng.standard_normal(64)
    prm = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.SGD([prm], lr=0.05, momentum=0.9, weight_decay=0.01)
    th = th0.copy(); buf = np.zeros_like(th)
    for t in range(1, 8):
        g = rng.standard_normal(64)
        prm.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, buf = O.sgdm_update(th, g, buf, 0.05, 0.01, 0.9, t == 1, store=np.float64)
        assert np.allclose(th, prm.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adamw_first_step_is_sign_step():
    # from m = v = 0 with wd = 0: m_hat = g, v_hat = g^2  =>  theta' = theta - lr g/(|g| + eps)
    g = np.array([0.3, -2.0, 1e-3, -7e-5]); th = np.array([1.0, -1.0, 0.5, 0.25])
    out, m, v = O.adamw_update(th, g, np.zeros(4), np.zeros(4), 0.01, 0.0, 0.9, 0.999, 1e-8, 1,
                               store=np.float64)
    assert np.allclose(out, th - 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_adamw_constant_gradient_closed_form():
    # constant g: bias-corrected moments stay (g, g^2) at every t, so each step moves by
    # lr*g/(|g|+eps) after the decoupled decay theta *= (1 - lr*wd)
    g = np.array([0.02, -0.5]); th = np.array([1.0, 2.0]); m = np.zeros(2); v = np.zeros(2)
    ref = th.copy()
    for t in range(1, 30):
        th, m, v = O.adamw_update(th, g, m, v, 0.01, 0.1, 0.9, 0.999, 1e-8, t, store=np.float64)
        ref = ref * (1 - 0.01 * 0.1) - 0.01 * g / (np.abs(g) + 1e-8)
        assert np.allclose(th, ref, rtol=1e-11)


def test_adamw_matches_library_optimizer():
    rng = np.random.default_rng(2)
    th0 = rng.standard_normal(64)
    prm = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.AdamW([prm], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    th = th0.copy(); m = np.zeros(64); v = np.zeros(64)
    for t in range(1, 12):
        g = rng.standard_normal(64) * 1e-3
        prm.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = O.adamw_update(th, g, m, v, 3e-3, 0.01, 0.9, 0.999, 1e-8, t, store=np.float64)
        assert np.allclose(th, prm.detach().numpy(), rtol=1e-11, atol=1e-14)


def test_fp32_storage_rounds_once():
    th = np.array([1.0], dtype=np.float32); g = np.array([1e-9], dtype=np.float32)
    out, _ = O.sgdm_update(th, g, np.zeros(1, np.float32), 1.0, 0.0, 0.0, True)
    assert out.dtype == np.float32 and out[0] == np.float32(1.0 - 1e-9)


# ---------------------------------------------------------------- Eq. 3 converge, grad mean
def test_converge_brute_force_and_invariants():
    rng = np.random.default_rng(3)
    for n in [1, 2, 3, 4, 8]:
        th = rng.standard_normal((n, 37)).astype(np.float32)
        out = O.converge(th)
        for i in range(37):
            s = 0.0
            for r in range(n):
                s += float(th[r, i])
            assert out[0, i] == np.float32(s / n)
        assert all(np.array_equal(out[0], out[r]) for r in range(n))      # planes identical
        same = np.broadcast_to(th[0], th.shape).copy()
        if n in (1, 2, 4, 8):
            assert np.array_equal(O.converge(same), same)                 # exact no-op
        assert np.allclose(out[0].astype(np.float64) * n, th.astype(np.float64).sum(0),
                           rtol=1e-6, atol=1e-6)
    g = rng.standard_normal((4, 9)).astype(np.float32)
    assert np.allclose(O.shared_gradient(g), g.astype(np.float64).mean(0), rtol=1e-7)


# ---------------------------------------------------------------- Eq. 4-7 controller
def test_controller_n2_closed_form():
    # N = 2, identity pi: Delta = alpha * eta * tanh((L0 - L1) / (2 sigma))
    eta, alpha, sigma = 0.05, 0.2, 0.1
    L = [2.30, 2.28]
    w = O.controller_weights(L, sigma)
    assert w.sum() == pytest.approx(1.0, abs=1e-15)
    assert w[1] == pytest.approx(1 / (1 + math.exp(-0.2)), rel=1e-13)    # logistic of (L0-L1)/sigma
    h = eta * O.spread_multipliers(2, alpha)
    d = O.hypergradient(w, h)
    assert d == pytest.approx(alpha * eta * math.tanh((L[0] - L[1]) / (2 * sigma)), rel=1e-12)
    assert d == pytest.approx(9.966799e-4, rel=1e-6)
    v, base = O.velocity_update(0.0, eta, d, 0.9, 0.0, 0.5)
    assert v == pytest.approx(0.1 * d) and base == pytest.approx(eta + 0.05 * d)


def test_controller_n4_pairwise_form():
    # independent formula: w_r = 1 / sum_r' exp((L_r - L_r') / sigma)
    L = [2.31, 2.30, 2.29, 2.27]; sigma = 0.1
    w = O.controller_weights(L, sigma)
    for r in range(4):
        assert w[r] == pytest.approx(1.0 / sum(math.exp((L[r] - L[q]) / sigma) for q in range(4)),
                                     rel=1e-13)
    h = 0.05 * O.spread_multipliers(4, 0.2)
    d = O.hypergradient(w, h)
    assert d == pytest.approx(sum(w[r] * h[r] for r in range(4)) - sum(h) / 4, rel=1e-10)
    assert d == pytest.approx(1.101131e-3, rel=1e-5)
    assert d > 0        # loss falls with rank (higher rate is better) => base should rise


def test_controller_invariants():
    rng = np.random.default_rng(4)
    for n in [1, 2, 3, 8]:
        L = (2.0 + 0.05 * rng.standard_normal(n)).tolist()
        w = O.controller_weights(L, 0.1)
        assert w.sum() == pytest.approx(1.0, abs=1e-14)
        w2 = O.controller_weights([x + 3.5 for x in L], 0.1)             # shift invariance
        assert np.allclose(w, w2, rtol=1e-9)
        h = 1e-3 * O.spread_multipliers(n, 0.15)
        assert abs(O.hypergradient(w, h)) <= 0.15 * 1e-3 + 1e-18          # |Delta| <= alpha eta
        weq = O.controller_weights([1.7] * n, 0.1)
        assert np.all(weq == 1.0 / n) and O.hypergradient(weq, h) == 0.0  # equal losses: exactly 0
        # sigma -> inf: no push; sigma -> 0: all weight on the best replica
        assert abs(O.hypergradient(O.controller_weights(L, 1e9), h)) < 1e-12
        best = int(np.argmin(L))
        d0 = O.hypergradient(O.controller_weights(L, 1e-6), h)
        assert d0 == pytest.approx(h[best] - h.mean(), abs=1e-15)
    # sign flips with the ranking
    h = 1e-3 * O.spread_multipliers(4, 0.1)
    assert O.hypergradient(O.controller_weights([1.0, 1.1, 1.2, 1.3], 0.1), h) < 0


# ---------------------------------------------------------------- whole loop
def _cfg(**kw):
    d = dict(n_replicas=4, total_steps=40, sync_interval=4, warm_steps=12, lr_max=0.05,
             alpha=0.2, autolr_enabled=True, optimizer=O.SGDM, momentum=0.9,
             grad_mode=O.GRAD_PER_REPLICA, seed=7)
    d.update(kw)
    return O.Config(**d)


def _run(cfg, P=33, steps=None, loss_fn=None, identical_grads=False):
    n = cfg.n_replicas
    orc = O.HDETOracle(cfg, I.flat_theta0(n, P, 5))
    hist = []
    for t in range(1, (steps or cfg.total_steps) + 1):
        g = I.flat_grads(n, P, 99, t, std=0.1)
        if identical_grads:
            g[:] = g[0]
        losses = loss_fn(t) if loss_fn else I.flat_losses(n, t)
        orc.step(g, losses)
        hist.append((orc.theta.copy(), orc.lr_used.copy()))
    return orc, hist


def test_alpha_zero_is_plain_data_parallel():
    """alpha = 0 with identical batches: replicas stay bit-identical, converge is a no-op and
    every replica follows the single-model trajectory (Sec. 3.2)."""
    for opt in (O.SGDM, O.ADAMW):
        cfg = _cfg(alpha=0.0, autolr_enabled=False, optimizer=opt, weight_decay=0.01)
        orc, hist = _run(cfg, identical_grads=True)
        single = O.HDETOracle(_cfg(n_replicas=1, alpha=0.0, autolr_enabled=False, optimizer=opt,
                                   weight_decay=0.01), I.flat_theta0(1, 33, 5))
        for t in range(1, 41):
            g = I.flat_grads(4, 33, 99, t, std=0.1)[:1]
            single.step(g, [0.0])
            th = hist[t - 1][0]
            assert all(np.array_equal(th[0], th[r]) for r in range(4))
            assert np.array_equal(th[0], single.theta[0])


def test_shared_sgd_t1_mean_equals_single_step_at_base_rate():
    """Plain SGD, T = 1, shared gradients: because sum rho = N the averaged update is one
    step at the base rate."""
    cfg = _cfg(optimizer=O.SGDM, momentum=0.0, sync_interval=1, grad_mode=O.GRAD_SHARED,
               autolr_enabled=False, alpha=0.2)
    n, P = 4, 33
    orc = O.HDETOracle(cfg, I.flat_theta0(n, P, 5))
    ref = I.flat_theta0(1, P, 5)[0].astype(np.float64)
    for t in range(1, 21):
        g = I.flat_grads(n, P, 99, t, std=0.1)
        orc.step(g, [0.0] * n)
        eta = O.onecycle_lr(t - 1, 40, 0.05, 25.0, 1e4, 0.3)
        ref = ref - eta * g.astype(np.float64).mean(0)
        assert np.allclose(orc.theta[0], ref, rtol=2e-6, atol=1e-7)
        assert all(np.array_equal(orc.theta[0], orc.theta[r]) for r in range(n))


def test_shared_adamw_moments_identical_across_replicas():
    cfg = _cfg(optimizer=O.ADAMW, grad_mode=O.GRAD_SHARED, weight_decay=0.01)
    orc, _ = _run(cfg, steps=10)
    assert all(np.array_equal(orc.m[0], orc.m[r]) and np.array_equal(orc.v[0], orc.v[r])
               for r in range(4))
    assert not np.array_equal(orc.theta[0], orc.theta[1])      # t = 10 is not a sync step


def test_equal_losses_leave_base_to_decay_only():
    cfg = _cfg()
    orc, _ = _run(cfg, loss_fn=lambda t: [2.0] * 4)
    assert orc.controller_active and orc.k == 8                # syncs at t = 12, 16, ..., 40
    assert all(v == 0.0 for v in orc.vel) and orc.delta[0] == 0.0
    eta12 = O.onecycle_lr(11, 40, 0.05, 25.0, 1e4, 0.3)
    assert orc.base[0] == pytest.approx(eta12 * (1 - orc.gamma) ** 8, rel=1e-12)
    # with gamma = 0 as well the base is untouched
    orc2, _ = _run(_cfg(gamma_override=0.0), loss_fn=lambda t: [2.0] * 4)
    assert orc2.base[0] == eta12


def test_loop_state_machine_and_final_identity():
    cfg = _cfg()
    orc, hist = _run(cfg)
    assert orc.t == 40 and orc.k == 8
    assert all(np.array_equal(orc.theta[0], orc.theta[r]) for r in range(4))   # Algorithm 1, return
    # before hand-over: one-cycle times rho with identity permutation
    rho = O.spread_multipliers(4, 0.2)
    for t in range(1, 13):
        eta = O.onecycle_lr(t - 1, 40, 0.05, 25.0, 1e4, 0.3)
        assert np.array_equal(hist[t - 1][1], (eta * rho).astype(np.float32))
    # after hand-over: piecewise constant between syncs, a permutation of base * rho
    for t in range(13, 41):
        lr = hist[t - 1][1]
        if (t - 1) % 4 != 0:
            assert np.array_equal(lr, hist[t - 2][1])
        assert np.allclose(np.sort(lr) / np.sort(lr).mean(), rho, rtol=1e-6)
    # L_acc is reset at every sync, so l_last is the mean of the last T losses only
    exp = np.mean([I.flat_losses(4, t) for t in range(37, 41)], axis=0)
    assert np.allclose(orc.l_last, exp, rtol=1e-14)
    with pytest.raises(RuntimeError):
        orc.fanout_step(I.flat_grads(4, 33, 99, 41))


def test_loop_n2_by_hand():
    """N = 2, P = 1, plain SGD, T = 2, constant base rate: two steps and a converge by hand."""
    cfg = O.Config(n_replicas=2, total_steps=8, sync_interval=2, warm_steps=0, lr_max=0.1,
                   alpha=0.5, autolr_enabled=True, optimizer=O.SGDM, momentum=0.0,
                   grad_mode=O.GRAD_PER_REPLICA, constant_lr=True, gamma_override=0.0,
                   sigma=0.1, beta=0.9, lam=0.5)
    orc = O.HDETOracle(cfg, np.array([[1.0], [1.0]], dtype=np.float32))
    g = np.array([[0.5], [0.25]], dtype=np.float32)
    orc.step(g, [1.0, 0.9])       # lr = (0.05, 0.15): theta = (0.975, 0.9625)
    assert np.allclose(orc.theta[:, 0], [0.975, 0.9625], rtol=1e-7)
    orc.step(g, [1.0, 0.9])       # theta = (0.95, 0.925) -> mean 0.9375
    assert np.allclose(orc.theta[:, 0], [0.9375, 0.9375], rtol=1e-7)
    # controller: L = (1.0, 0.9); Delta = alpha*eta*tanh(0.1/0.2); v = 0.1*Delta; base += 0.5 v
    d = 0.5 * 0.1 * math.tanh(0.5)
    assert orc.delta[0] == pytest.approx(d, rel=1e-12)
    assert orc.vel[0] == pytest.approx(0.1 * d, rel=1e-12)
    assert orc.base[0] == pytest.approx(0.1 + 0.05 * d, rel=1e-12)
    assert orc.k == 1 and sorted(orc.perm[0].tolist()) == [0, 1]
    lr3 = orc.lr_table(3)
    assert np.allclose(np.sort(lr3), np.array([0.5, 1.5]) * orc.base[0], rtol=1e-7)


def test_multichannel_independent_permutations_and_clamp():
    extra = [O.Channel(O.CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45), O.Channel(O.CH_WD, 0.05, 0.5, 0.5, 0.0)]
    cfg = _cfg(n_replicas=8, optimizer=O.ADAMW, extra=extra, lr_max=3e-4, alpha=0.15)
    orc, _ = _run(cfg)
    assert np.allclose(np.sort(orc.dropout_table()) / orc.base[1], O.spread_multipliers(8, 1.0),
                       atol=1e-6)
    assert np.allclose(np.sort(orc.wd_table()) / orc.base[2], O.spread_multipliers(8, 0.5), rtol=1e-6)
    assert len({tuple(p.tolist()) for p in orc.perm}) == 3
    assert 0.0 <= orc.base[1] <= 0.9 and orc.base[2] >= 0.0
    # a channel's Delta is bounded by its own spread: |Delta_j| <= alpha_j * max base_j
    assert abs(orc.delta[1]) <= 1.0 * 0.9 and abs(orc.delta[2]) <= 0.5 * max(orc.base[2], 0.05) * 1.5


def test_nonfinite_loss_leaves_state_untouched():
    cfg = _cfg()
    orc, _ = _run(cfg, steps=16, loss_fn=lambda t: [2.0, float("nan"), 2.0, 2.0] if t > 12 else [2.0] * 4)
    assert orc.nonfinite == 1 and orc.k == 1


# ---------------------------------------------------------------- Eq. 10 warm noisy initialisation
def test_warm_init_noise_scale_and_independence():
    from scipy import stats
    rng = np.random.default_rng(9)
    theta0 = (rng.standard_normal(20000) * 0.3).astype(np.float32)
    nu = load_golden("controller_defaults.txt")["nu"][0]            # the paper uses nu = 0.01
    out = O.warm_noisy_init(theta0, 4, nu, 123, store=np.float64)
    eps = out - theta0.astype(np.float64)
    norm2 = float(np.sum(theta0.astype(np.float64) ** 2))
    d = theta0.size
    for r in range(4):
        # E ||eps_r||^2 = nu^2 ||theta0||^2 ; chi-square with d dof has relative sd sqrt(2/d)
        assert np.sum(eps[r] ** 2) == pytest.approx(nu ** 2 * norm2, rel=5 * math.sqrt(2.0 / d))
        assert abs(eps[r].mean()) < 5 * nu * math.sqrt(norm2 / d) / math.sqrt(d)
        z = eps[r] / (nu * math.sqrt(norm2 / d))
        assert stats.kstest(z, "norm").pvalue > 1e-3                  # Gaussian
    c = np.corrcoef(eps)
    assert np.all(np.abs(c[~np.eye(4, dtype=bool)]) < 5 / math.sqrt(d))   # replicas independent
    # deterministic in (seed, replica, index); nu = 0 returns the checkpoint itself
    assert np.array_equal(O.warm_noisy_init(theta0, 2, nu, 123), O.warm_noisy_init(theta0, 4, nu, 123)[:2])
    assert not np.array_equal(O.warm_noisy_init(theta0, 1, nu, 124), O.warm_noisy_init(theta0, 1, nu, 123))
    assert np.array_equal(O.warm_noisy_init(theta0, 3, 0.0, 5), np.broadcast_to(theta0, (3, d)))
    assert np.array_equal(O.standard_normals(7, 1, 10), O.standard_normals(7, 1, 37)[:10])


def test_box_muller_pairs_by_hand():
    w = O.philox4x32_10((0, 2, 0, O.WARM_STREAM), (11, 0))
    z = O.standard_normals(11, 2, 4)
    for h in range(2):
        u, v = (w[2 * h] + 1) / 2.0 ** 32, w[2 * h + 1] / 2.0 ** 32
        assert z[2 * h] ** 2 + z[2 * h + 1] ** 2 == pytest.approx(-2 * math.log(u), rel=1e-12)
        assert math.atan2(z[2 * h + 1], z[2 * h]) % (2 * math.pi) == pytest.approx(2 * math.pi * v, abs=1e-9)


def test_parameter_groups_have_independent_rate_channels():
    """Four parameter groups as in the paper's experiment: same one-cycle before hand-over,
    then own base, velocity and permutation each; with one group the old behaviour."""
    ends = [8, 16, 28, 33]
    cfg = _cfg(n_replicas=8, group_ends=ends)
    orc, hist = _run(cfg)
    assert orc.n_lr == 4 and orc.n_ch == 4 and orc.k == 8
    assert len({tuple(p.tolist()) for p in orc.perm}) == 4                   # independent permutations
    assert len({round(b, 15) for b in orc.base}) == 4                         # bases drift apart
    for g in range(4):
        lr = orc.lr_table(40, g)
        assert np.allclose(np.sort(lr) / orc.base[g], O.spread_multipliers(8, 0.2), rtol=1e-6)
    # before hand-over every group used the same rates: identical to the single-group run
    one, hist1 = _run(_cfg(n_replicas=8))
    assert np.array_equal(hist[10][0], hist1[10][0])
    # a group's slice only ever sees its own rate: zero gradient outside group 2 leaves the rest untouched
    orc2 = O.HDETOracle(_cfg(n_replicas=2, group_ends=ends, optimizer=O.SGDM, momentum=0.0, autolr_enabled=False),
                        I.flat_theta0(2, 33, 5))
    g = np.zeros((2, 33), np.float32); g[:, 16:28] = 1.0
    before = orc2.theta.copy()
    orc2.fanout_step(g, [0.0, 0.0])
    assert np.array_equal(before[:, :16], orc2.theta[:, :16]) and np.array_equal(before[:, 28:], orc2.theta[:, 28:])
    assert not np.array_equal(before[:, 16:28], orc2.theta[:, 16:28])


def test_reshuffle_every_sync_redraws_before_the_controller_runs():
    """Fig. 1's reading: a fresh assignment at every sync step, numbered by the sync step; with
    the flag off nothing moves before the first controller update (Algorithm 1)."""
    cfg_on = _cfg(n_replicas=8, reshuffle_every_sync=True)
    cfg_off = _cfg(n_replicas=8)
    on = O.HDETOracle(cfg_on, I.flat_theta0(8, 33, 5))
    off = O.HDETOracle(cfg_off, I.flat_theta0(8, 33, 5))
    T = cfg_on.sync_interval
    seen = []
    for t in range(1, cfg_on.total_steps + 1):
        g = I.flat_grads(8, 33, 99, t, std=0.1)
        on.step(g, I.flat_losses(8, t)); off.step(g, I.flat_losses(8, t))
        if t % T == 0:
            assert on.perm[0].tolist() == O.permutation(cfg_on.seed, t // T, 0, 8).tolist()
            assert sorted(on.perm[0].tolist()) == list(range(8))
            seen.append(tuple(on.perm[0].tolist()))
            if t < cfg_off.warm_steps:
                assert off.perm[0].tolist() == list(range(8)) and on.k == 0
            else:
                assert off.perm[0].tolist() == O.permutation(cfg_off.seed, off.k, 0, 8).tolist()
    assert len(set(seen)) == len(seen)               # all different draws
    assert on.k == off.k                             # the controller itself runs at the same steps
    # a non-finite interval loss leaves the assignment alone under both readings
    bad = O.HDETOracle(cfg_on, I.flat_theta0(8, 33, 5))
    for t in range(1, cfg_on.warm_steps + 1):
        bad.fanout_step(I.flat_grads(8, 33, 99, t, std=0.1), I.flat_losses(8, t))
        if t % T == 0:
            bad.converge()
            before = bad.perm[0].copy()
            if t == cfg_on.warm_steps:
                bad.autolr_update([float("nan")] + [1.0] * 7)
                assert bad.perm[0].tolist() == before.tolist() and bad.nonfinite == 1
            else:
                bad.autolr_update()
