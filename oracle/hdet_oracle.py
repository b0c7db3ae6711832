"""CPU oracle for the HDET training step (fan-out, converge, auto-LR controller).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, deliberately unoptimised
restatement of the method so that a reader can check it against the paper by eye.
Nothing in the product path may import it; it shares no code with the HIP library.

Conventions
-----------
* Tensors the GPU keeps in fp32 (parameters, gradients, optimizer state) are kept in
  fp32 here too; the arithmetic of every step is carried out in fp64 and rounded to
  fp32 once, on store.  All schedule / controller scalars are fp64.
* Replica axis first: arrays are ``[N, P]``.
* Steps are counted t = 1..S as in Algorithm 1; update t uses schedule index t-1.

Where the paper is silent the reading taken is stated next to the code.

Parity pins: every function here is pinned by tests/test_oracle_*.py (paper's
worked example for the spread, closed forms, library special cases, brute force).
The loss figures of Table 1 and the curves of Fig. 2-3 are parity unpinned: they
need the paper's proprietary data and backbone.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

SGDM = 0
ADAMW = 1
GRAD_SHARED = 0
GRAD_PER_REPLICA = 1
CH_LR = 0
CH_DROPOUT = 1
CH_WD = 2
CH_LABEL_SMOOTH = 3     # label smoothing eps of the cross-entropy (Remark 1)
CH_ATTN_TEMP = 4        # attention temperature tau (Remark 1)


# --------------------------------------------------------------------------------------
# Sec. 3.2, Eq. 1: symmetric spread multipliers
# --------------------------------------------------------------------------------------
def spread_multipliers(n: int, alpha: float) -> np.ndarray:
    """rho_r = 1 + alpha * (r - (N-1)/2) / delta, delta = max((N-1)/2, 1/2)  (Eq. 1)."""
    delta = max((n - 1) / 2.0, 0.5)
    centre = (n - 1) / 2.0
    return np.array([1.0 + alpha * ((r - centre) / delta) for r in range(n)], dtype=np.float64)


# --------------------------------------------------------------------------------------
# Base schedule eta(t): one-cycle policy with parameters (eta_max, f_div, f_final, p)
# (Algorithm 1, Require).  The paper only names the parameters; the reading taken is
# the two-phase cosine one-cycle policy: eta rises from eta_max/f_div to eta_max over
# schedule indices 0 .. p*S-1 and falls to eta_max/(f_div*f_final) at index S-1, each
# phase following  end + (start-end)/2 * (1 + cos(pi * pct)).
# --------------------------------------------------------------------------------------
def onecycle_lr(idx: int, total_steps: int, lr_max: float, f_div: float, f_final: float,
                pct_start: float) -> float:
    lr_init = lr_max / f_div
    lr_min = lr_init / f_final
    end1 = float(pct_start * total_steps) - 1.0
    end2 = float(total_steps) - 1.0

    def anneal(start: float, end: float, pct: float) -> float:
        return end + (start - end) / 2.0 * (1.0 + math.cos(math.pi * pct))

    if idx <= end1:
        pct = idx / end1 if end1 > 0.0 else 1.0
        return anneal(lr_init, lr_max, pct)
    span = end2 - end1
    pct = (idx - end1) / span if span > 0.0 else 1.0
    return anneal(lr_max, lr_min, pct)


# --------------------------------------------------------------------------------------
# Sec. 3.4, Eq. 8: per-sync decay gamma.
# The printed formula, read with the divisor convention of the one-cycle parameters
# (f_div = 25, f_final = 1e4), gives a negative gamma, i.e. growth, which contradicts the
# sentence that gamma reproduces the schedule's decay floor.  Reading taken: gamma is the
# per-sync decay for which K syncs take eta_max down to the one-cycle floor,
#   (1 - gamma)^K = eta_min / eta_max = 1 / (f_div * f_final),
# with K = (S - S_warm) / T as a real number.  K <= 0 (no sync left) gives gamma = 0.
# --------------------------------------------------------------------------------------
def decay_gamma(total_steps: int, warm_steps: int, sync_interval: int, f_div: float,
                f_final: float) -> float:
    k_sync = (total_steps - warm_steps) / float(sync_interval)
    if k_sync <= 0.0:
        return 0.0
    return 1.0 - math.exp(-math.log(f_div * f_final) / k_sync)


# --------------------------------------------------------------------------------------
# Counter-based generator: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw,
# "Parallel random numbers: as easy as 1, 2, 3", SC'11).  Used for the permutation of
# Eq. 9 and for dropout masks.
# --------------------------------------------------------------------------------------
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter: Sequence[int], key: Sequence[int]) -> List[int]:
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK32
        hi1, lo1 = p1 >> 32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK32, lo1, (hi0 ^ c3 ^ k1) & _MASK32, lo0
    return [c0, c1, c2, c3]


PERM_STREAM = 0x48444554  # ASCII "HDET": separates permutation draws from other uses


def permutation_from_words(next_word, n: int) -> np.ndarray:
    """Fisher-Yates from the top index down on the identity: for i = n-1 .. 1 draw j uniform on
    [0, i] and swap entries i and j.  A draw takes successive 32-bit words from `next_word()` and
    rejects those at or above the largest multiple of i+1 below 2^32 (no modulo bias), then reduces
    the accepted word modulo i+1."""
    pi = list(range(n))
    for i in range(n - 1, 0, -1):
        bound = i + 1
        limit = (1 << 32) - ((1 << 32) % bound)
        while True:
            x = next_word()
            if x < limit:
                break
        j = x % bound
        pi[i], pi[j] = pi[j], pi[i]
    return np.array(pi, dtype=np.int32)


def permutation(seed: int, k: int, channel: int, n: int) -> np.ndarray:
    """Fresh permutation pi of Eq. 9 for controller update number k and hyperparameter
    channel `channel`; a pure function of (seed, k, channel) so that every rank (here:
    both implementations) agrees without an exchange.

    The paper does not name a generator.  Reading taken: permutation_from_words on the words
    of the blocks philox(counter=(block, k, channel, PERM_STREAM), key=(seed_lo, seed_hi)),
    block = 0, 1, ..., each block's four words in order.
    """
    key = (seed & _MASK32, (seed >> 32) & _MASK32)
    words: List[int] = []
    block = 0

    def next_word() -> int:
        nonlocal block
        if not words:
            words.extend(philox4x32_10((block, k & _MASK32, channel, PERM_STREAM), key))
            block += 1
        return words.pop(0)

    return permutation_from_words(next_word, n)


# --------------------------------------------------------------------------------------
# Sec. 3.5, Eq. 10: warm noisy initialisation
# --------------------------------------------------------------------------------------
WARM_STREAM = 0x5741524D  # ASCII "WARM"


def standard_normals(seed: int, replica: int, n: int) -> np.ndarray:
    """n standard normal draws for one replica, a pure function of (seed, replica, index).
    Elements 4b..4b+3 come from philox(counter = (b, replica, 0, WARM_STREAM), key = seed):
    with u = (word + 1) / 2^32 in (0, 1] and v = word / 2^32 in [0, 1), the Box-Muller pairs
    are (sqrt(-2 ln u0) cos(2 pi v1), sqrt(-2 ln u0) sin(2 pi v1)) from words (0, 1) and
    likewise from words (2, 3)."""
    key = (seed & _MASK32, (seed >> 32) & _MASK32)
    out = np.empty(4 * ((n + 3) // 4), dtype=np.float64)
    for b in range((n + 3) // 4):
        w = philox4x32_10((b, replica, 0, WARM_STREAM), key)
        for h in range(2):
            u = (w[2 * h] + 1) / 4294967296.0
            v = w[2 * h + 1] / 4294967296.0
            rad = math.sqrt(-2.0 * math.log(u))
            out[4 * b + 2 * h] = rad * math.cos(2.0 * math.pi * v)
            out[4 * b + 2 * h + 1] = rad * math.sin(2.0 * math.pi * v)
    return out[:n]


def warm_noisy_init(theta0: np.ndarray, n_replicas: int, nu: float, seed: int, store=np.float32) -> np.ndarray:
    """theta_r = theta0 + eps_r, eps_r ~ N(0, nu^2 ||theta0||^2 / d) independently per replica
    and element (Eq. 10); d = number of parameters."""
    t0 = theta0.astype(np.float64)
    d = t0.size
    sigma = nu * math.sqrt(float(np.sum(t0 * t0)) / d)
    out = np.empty((n_replicas, d), dtype=store)
    for r in range(n_replicas):
        out[r] = (t0 + sigma * standard_normals(seed, r, d)).astype(store)
    return out


# --------------------------------------------------------------------------------------
# Gradient exchange (Algorithm 1, "AllReduce gradients"): replica-axis mean.
# --------------------------------------------------------------------------------------
def shared_gradient(g: np.ndarray) -> np.ndarray:
    """g_bar = (1/N) sum_r g_r, summed in the order r = 0..N-1; returned in fp32."""
    n = g.shape[0]
    acc = np.zeros(g.shape[1:], dtype=np.float64)
    for r in range(n):
        acc = acc + g[r].astype(np.float64)
    return (acc / n).astype(np.float32)


# --------------------------------------------------------------------------------------
# Sec. 3.2, Eq. 2 generalised to the optimizers the experiments use ("Adam", Sec. 4.1).
# Eq. 2 itself is plain SGD; momentum 0 and weight decay 0 reduce sgdm_update to it.
# --------------------------------------------------------------------------------------
def sgdm_update(theta, g, buf, lr: float, weight_decay: float, momentum: float, first_step: bool,
                store=np.float32):
    """Heavy-ball SGD with coupled L2: g' = g + wd*theta; buf = g' on the first step, else
    mu*buf + g'; theta -= lr*buf."""
    th = theta.astype(np.float64)
    gp = g.astype(np.float64) + weight_decay * th
    if first_step:
        nb = gp
    else:
        nb = momentum * buf.astype(np.float64) + gp
    nb_s = nb.astype(store)
    th = th - lr * nb
    return th.astype(store), nb_s


def adamw_update(theta, g, m, v, lr: float, weight_decay: float, beta1: float, beta2: float,
                 eps: float, t: int, store=np.float32):
    """AdamW (decoupled weight decay; Loshchilov & Hutter): theta *= 1 - lr*wd;
    m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
    theta -= lr/(1-b1^t) * m / (sqrt(v)/sqrt(1-b2^t) + eps)."""
    th = theta.astype(np.float64) * (1.0 - lr * weight_decay)
    g64 = g.astype(np.float64)
    nm = beta1 * m.astype(np.float64) + (1.0 - beta1) * g64
    nv = beta2 * v.astype(np.float64) + (1.0 - beta2) * g64 * g64
    bc1 = 1.0 - beta1 ** t
    bc2 = 1.0 - beta2 ** t
    denom = np.sqrt(nv) / math.sqrt(bc2) + eps
    th = th - (lr / bc1) * nm / denom
    return th.astype(store), nm.astype(store), nv.astype(store)


# --------------------------------------------------------------------------------------
# Sec. 3.3, Eq. 3: converge
# --------------------------------------------------------------------------------------
def converge(theta: np.ndarray, store=np.float32) -> np.ndarray:
    """theta_r <- (1/N) sum_r' theta_r' for every r (sum in the order r' = 0..N-1)."""
    n = theta.shape[0]
    acc = np.zeros(theta.shape[1:], dtype=np.float64)
    for r in range(n):
        acc = acc + theta[r].astype(np.float64)
    mean = (acc / n).astype(store)
    return np.broadcast_to(mean, theta.shape).copy()


# --------------------------------------------------------------------------------------
# Sec. 3.4, Eq. 4-7: controller
# --------------------------------------------------------------------------------------
_LOG2E = 1.4426950408889634
_LN2_HI = 6.93147180369123816490e-01      # the leading 32 bits of ln 2: k * _LN2_HI is exact for |k| < 2^20
_LN2_LO = 1.90821492927058770002e-10
_INV_FACT = [1.0 / math.factorial(i) for i in range(14)]


def exp_spec(x: float) -> float:
    """exp(x) for x <= 0, the exponential of Eq. 4's softmax after the maximum score is subtracted.

    The schedule state must be reproducible bit for bit, and math libraries differ in the last place
    of exp.  The exponential is therefore a fixed sequence of IEEE double operations (no fused
    multiply-add): 0 below -708; otherwise k = x log2(e) rounded to the nearest integer (ties to
    even), r = (x - k LN2_HI) - k LN2_LO, the Taylor polynomial of degree 13 at r by Horner's rule
    with coefficients 1/i! (each the correctly rounded quotient), scaled by 2^k.  Within two units
    in the last place of the true exponential (pinned against a 50-digit evaluation)."""
    if x > 0.0:
        raise ValueError("exp_spec is specified for x <= 0")
    if not (x >= -708.0):
        return 0.0
    k = float(round(x * _LOG2E))
    r = (x - k * _LN2_HI) - k * _LN2_LO
    p = _INV_FACT[13]
    for i in range(12, -1, -1):
        p = p * r + _INV_FACT[i]
    return p * math.ldexp(1.0, int(k))


def controller_weights(losses: Sequence[float], sigma: float) -> np.ndarray:
    """s_r = (Lbar - L_r)/sigma, w = softmax(s)  (Eq. 4); the maximum score is subtracted
    before exponentiation, which leaves w unchanged.  The exponential is exp_spec."""
    n = len(losses)
    lbar = 0.0
    for r in range(n):
        lbar += float(losses[r])
    lbar /= n
    s = [(lbar - float(losses[r])) / sigma for r in range(n)]
    smax = max(s)
    e = [exp_spec(x - smax) for x in s]
    z = 0.0
    for r in range(n):
        z += e[r]
    return np.array([x / z for x in e], dtype=np.float64)


def hypergradient(w: Sequence[float], h: Sequence[float]) -> float:
    """Delta = sum_r w_r h_r - (1/N) sum_r h_r  (Eq. 5-6), evaluated as
    sum_r (w_r - 1/N) h_r in ascending r: the same number, and exactly zero whenever all
    weights equal 1/N (equal losses)."""
    n = len(w)
    inv_n = 1.0 / n
    d = 0.0
    for r in range(n):
        d += (float(w[r]) - inv_n) * float(h[r])
    return d


def velocity_update(vel: float, base: float, delta: float, beta: float, gamma: float,
                    lam: float):
    """v <- beta v + (1-beta) Delta;  base <- base (1-gamma) + v lambda   (Eq. 7)."""
    nv = beta * vel + (1.0 - beta) * delta
    nb = base * (1.0 - gamma) + nv * lam
    return nv, nb


# --------------------------------------------------------------------------------------
# Whole loop (Algorithm 1) over flat parameter buffers
# --------------------------------------------------------------------------------------
@dataclass
class Channel:
    """One explored scalar hyperparameter (Remark 1).  The first channels are learning rates
    (one per parameter group); their base follows the one-cycle schedule until the controller
    takes over."""
    kind: int
    base: float
    alpha: float
    lam: float = 0.5
    lo: float = 0.0
    hi: float = float("inf")


@dataclass
class Config:
    n_replicas: int
    total_steps: int
    sync_interval: int
    warm_steps: int
    lr_max: float
    f_div: float = 25.0
    f_final: float = 1e4
    pct_start: float = 0.3
    alpha: float = 0.0
    autolr_enabled: bool = False
    beta: float = 0.9
    sigma: float = 0.1
    lam: float = 0.5
    optimizer: int = ADAMW
    momentum: float = 0.9
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    grad_mode: int = GRAD_PER_REPLICA
    seed: int = 7
    gamma_override: float = -1.0          # >= 0 replaces Eq. 8
    constant_lr: bool = False             # base schedule eta(t) = lr_max for all t
    extra: List[Channel] = field(default_factory=list)   # channels after the rates (dropout, wd)
    group_ends: List[int] = field(default_factory=list)  # parameter groups with a rate channel each:
                                                         # group g = plane slice [ends[g-1], ends[g])
    reshuffle_every_sync: bool = False    # Fig. 1's reading: new permutations at every sync step,
                                          # also while the controller does not run yet


class HDETOracle:
    """Algorithm 1 with the replicas as the leading axis of [N, P] arrays.

    Readings (the paper is silent or inconsistent on each):
    * The accumulated loss is the forward-pass loss at the pre-update parameters.
    * L_acc is reset at every sync step, controller on or off, so that L_r is always the
      mean over the last T steps as Sec. 3.4 defines it.
    * From the first controller update on, the one-cycle formula is no longer consulted:
      the base is piecewise constant and changes only through Eq. 7.  At hand-over the
      base is the mean of the rates in effect, i.e. the one-cycle value of that step.
    * The rates entering Eq. 5 are those in effect at the sync step.
    * Permutations are redrawn only when the controller runs (Algorithm 1), numbered by the
      controller update k.  With reshuffle_every_sync (the caption of Fig. 1: reshuffled before
      every cycle) they are redrawn at every sync step, numbered by the sync step t / T; a sync
      step whose losses are not finite still leaves everything untouched.
    * Optimizer state is not averaged by converge (Eq. 3 names the parameters only).
    * Channels other than the learning rates use gamma = 0 and are clamped to [lo, hi].
    * Parameter groups (Sec. 3.4: per-group rates, each with an independent permutation)
      share one one-cycle schedule until hand-over; afterwards every group has its own base
      rate and velocity, driven by the same weights w through its own permutation.
    """

    def __init__(self, cfg: Config, theta0: np.ndarray):
        self.cfg = cfg
        n = cfg.n_replicas
        assert theta0.shape[0] == n
        self.theta = theta0.astype(np.float32).copy()
        self.m = np.zeros_like(self.theta)      # AdamW first moment / SGD momentum buffer
        self.v = np.zeros_like(self.theta)      # AdamW second moment
        self.t = 0
        self.k = 0
        self.controller_active = False
        self.n_lr = max(len(cfg.group_ends), 1)
        self.group_ends = list(cfg.group_ends) if len(cfg.group_ends) > 1 else [theta0.shape[1]]
        self.channels = [Channel(CH_LR, cfg.lr_max, cfg.alpha, cfg.lam) for _ in range(self.n_lr)] + list(cfg.extra)
        self.n_ch = len(self.channels)
        self.rho = [spread_multipliers(n, ch.alpha) for ch in self.channels]
        self.perm = [np.arange(n, dtype=np.int32) for _ in self.channels]
        self.base = [ch.base for ch in self.channels]       # h_bar_j (lr: set per step)
        self.vel = [0.0 for _ in self.channels]
        self.delta = [0.0 for _ in self.channels]
        self.w = np.full(n, 1.0 / n)
        self.l_acc = np.zeros(n, dtype=np.float64)
        self.l_last = np.zeros(n, dtype=np.float64)
        self.gamma = (cfg.gamma_override if cfg.gamma_override >= 0.0 else
                      decay_gamma(cfg.total_steps, cfg.warm_steps, cfg.sync_interval,
                                  cfg.f_div, cfg.f_final))
        self.nonfinite = 0

    # ---- schedule ---------------------------------------------------------------
    def base_lr(self, t: int, group: int = 0) -> float:
        """eta_bar used by update t (1-based) for a parameter group."""
        if self.controller_active:
            return self.base[group]
        if self.cfg.constant_lr:
            return self.cfg.lr_max
        c = self.cfg
        return onecycle_lr(t - 1, c.total_steps, c.lr_max, c.f_div, c.f_final, c.pct_start)

    def values(self, j: int, base: Optional[float] = None) -> np.ndarray:
        """h_{j,r} = h_bar_j * rho_{j, pi_j(r)} in fp64."""
        b = self.base[j] if base is None else base
        return np.array([b * self.rho[j][self.perm[j][r]] for r in range(self.cfg.n_replicas)],
                        dtype=np.float64)

    def channel_index(self, kind: int) -> int:
        for j, ch in enumerate(self.channels):
            if ch.kind == kind:
                return j
        return -1

    def lr_table(self, t: int, group: int = 0) -> np.ndarray:
        """Per-replica learning rates of a parameter group handed to the update, rounded to fp32."""
        return self.values(group, self.base_lr(t, group)).astype(np.float32)

    def wd_table(self) -> np.ndarray:
        j = self.channel_index(CH_WD)
        n = self.cfg.n_replicas
        if j < 0:
            return np.full(n, self.cfg.weight_decay, dtype=np.float64).astype(np.float32)
        return self.values(j).astype(np.float32)

    def dropout_table(self) -> np.ndarray:
        j = self.channel_index(CH_DROPOUT)
        n = self.cfg.n_replicas
        if j < 0:
            return np.zeros(n, dtype=np.float32)
        return self.values(j).astype(np.float32)

    def label_smoothing_table(self) -> np.ndarray:
        """eps_r handed to the loss of replica r, rounded to fp32 (0 without such a channel)."""
        j = self.channel_index(CH_LABEL_SMOOTH)
        if j < 0:
            return np.zeros(self.cfg.n_replicas, dtype=np.float32)
        return self.values(j).astype(np.float32)

    def attn_temp_table(self) -> np.ndarray:
        """tau_r handed to the attention of replica r, rounded to fp32 (1 without such a channel)."""
        j = self.channel_index(CH_ATTN_TEMP)
        if j < 0:
            return np.ones(self.cfg.n_replicas, dtype=np.float32)
        return self.values(j).astype(np.float32)

    def is_sync(self) -> bool:
        return self.t > 0 and self.t % self.cfg.sync_interval == 0

    # ---- one step of Algorithm 1 ---------------------------------------------------
    def fanout_step(self, grads: np.ndarray, losses: Optional[Sequence[float]] = None):
        """Update t (Algorithm 1, the gradient exchange and the update), then the loss
        accumulation.  `grads` is [N, P] fp32 (per-replica gradients); in shared mode their
        replica mean is what every replica applies."""
        c = self.cfg
        n = c.n_replicas
        if self.t >= c.total_steps:
            raise RuntimeError("step beyond total_steps")
        self.t += 1
        t = self.t
        wd = self.wd_table()
        self.lr_used = self.lr_table(t, 0)
        if c.grad_mode == GRAD_SHARED:
            gbar = shared_gradient(grads)
        begin = 0
        for grp, end in enumerate(self.group_ends):
            lr = self.lr_table(t, grp)
            sl = slice(begin, end)
            for r in range(n):
                g = gbar[sl] if c.grad_mode == GRAD_SHARED else grads[r][sl]
                if c.optimizer == SGDM:
                    self.theta[r, sl], self.m[r, sl] = sgdm_update(self.theta[r, sl], g, self.m[r, sl], float(lr[r]),
                                                                   float(wd[r]), c.momentum, t == 1)
                else:
                    self.theta[r, sl], self.m[r, sl], self.v[r, sl] = adamw_update(
                        self.theta[r, sl], g, self.m[r, sl], self.v[r, sl], float(lr[r]), float(wd[r]),
                        c.beta1, c.beta2, c.eps, t)
            begin = end
        if losses is not None:
            self.accumulate_loss(losses)

    def accumulate_loss(self, losses: Sequence[float]):
        for r in range(self.cfg.n_replicas):
            self.l_acc[r] += float(losses[r])

    def converge(self):
        self.theta = converge(self.theta)

    def autolr_update(self, interval_losses: Optional[Sequence[float]] = None):
        """Sync-step bookkeeping (Algorithm 1, inside `t mod T = 0`): L_r, reset of the
        accumulator, and -- if enabled and t >= S_warm -- Eq. 4-9."""
        c = self.cfg
        n = c.n_replicas
        if not self.is_sync():
            raise RuntimeError("autolr_update off a sync step")
        if interval_losses is None:
            l_r = self.l_acc / float(c.sync_interval)
        else:
            l_r = np.array([float(x) for x in interval_losses], dtype=np.float64)
        self.l_acc = np.zeros(n, dtype=np.float64)
        self.l_last = l_r
        if not (c.autolr_enabled and self.t >= c.warm_steps):
            if c.reshuffle_every_sync:
                for j in range(self.n_ch):
                    self.perm[j] = permutation(c.seed, self.t // c.sync_interval, j, n)
            return
        if not np.all(np.isfinite(l_r)):
            # a non-finite loss carries no ranking signal: state is left untouched
            self.nonfinite += 1
            return
        if not self.controller_active:
            # hand-over: base = mean of the rates in effect = schedule value of this step
            eta = self.base_lr(self.t)
            for g in range(self.n_lr):
                self.base[g] = eta
            self.controller_active = True
        w = controller_weights(l_r, c.sigma)
        self.w = w
        for j, ch in enumerate(self.channels):
            h = self.values(j)
            d = hypergradient(w, h)
            gamma = self.gamma if ch.kind == CH_LR else 0.0
            self.vel[j], nb = velocity_update(self.vel[j], self.base[j], d, c.beta, gamma, ch.lam)
            self.delta[j] = d
            self.base[j] = min(max(nb, ch.lo), ch.hi)
        self.k += 1
        draw = self.t // c.sync_interval if c.reshuffle_every_sync else self.k
        for j in range(self.n_ch):
            self.perm[j] = permutation(c.seed, draw, j, n)

    def step(self, grads: np.ndarray, losses: Sequence[float]):
        """One full iteration of Algorithm 1's loop body."""
        self.fanout_step(grads, losses)
        if self.is_sync():
            self.converge()
            self.autolr_update()
