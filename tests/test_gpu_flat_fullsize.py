"""Parity at the benchmark's full size (N = 8 replicas x P = 1e9 fp32, AdamW, the launch
configuration bench.py times): the update is elementwise along P, so the oracle replays it on
sampled columns -- all 8 replicas of 2^16 sampled parameter indices, across plain steps, a
fused-converge sync step, a standalone-converge sync step and the controller."""
import numpy as np
import pytest
import torch

import hdet_inputs as I
import paper_2604_24708_amd as H
from harness import check_state, library_config, oracle_config, rel_err
from oracle import hdet_oracle as O

pytestmark = pytest.mark.gpu


def test_sampled_columns_at_full_size():
    n, P, T = 8, 1_000_000_000, 3
    need = 4 * n * P * 4
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < need + (8 << 30):
        pytest.skip(f"needs {need / 2**30:.0f} GiB of free HBM")
    dev = torch.device("cuda:0")
    theta = torch.empty((n, P), dtype=torch.float32, device=dev)
    g = torch.empty_like(theta)
    m = torch.zeros_like(theta)
    v = torch.zeros_like(theta)
    I.device_normal_(theta[0], I.SEED_INIT, 0.02)
    for r in range(1, n):
        theta[r].copy_(theta[0])
    I.device_normal_(g, I.SEED_GRADS, 1e-3)

    rng = np.random.default_rng(11)
    idx = np.unique(np.concatenate([rng.integers(0, P, size=1 << 16), np.arange(0, 1024),
                                    np.arange(P - 1024, P), np.arange(P // 2 - 300, P // 2 + 300)]))
    idx_dev = torch.from_numpy(idx).to(dev)

    d = dict(n_replicas=n, total_steps=7, sync_interval=T, warm_steps=3, lr_max=1e-3, alpha=0.1,
             autolr_enabled=True, optimizer=O.ADAMW, weight_decay=0.01, grad_mode=O.GRAD_PER_REPLICA,
             seed=I.SEED_PERM)
    orc = O.HDETOracle(oracle_config(d), theta[:, idx_dev].cpu().numpy())
    g_s = g[:, idx_dev].cpu().numpy()
    h = H.hdet_create(library_config(d, n_params=P, model_kind=H.HDET_FLAT), theta, m, v, plane_stride=P)
    untouched = theta[:, 5].clone()
    for t in range(1, 8):
        losses = I.flat_losses(n, t)
        H.hdet_fanout_step(h, g, H.HDET_FUSE_CONVERGE if t == 3 else 0)
        orc.fanout_step(g_s, losses)
        if t % T == 0:
            H.hdet_converge(h)
            orc.converge()
            H.hdet_autolr_update(h, (orc.l_acc / T).tolist())
            orc.autolr_update()
        tol = min(t * 1e-5, 1e-4)
        assert rel_err(theta[:, idx_dev].cpu().numpy(), orc.theta) <= tol
        assert rel_err(m[:, idx_dev].cpu().numpy(), orc.m) <= tol
        assert rel_err(v[:, idx_dev].cpu().numpy(), orc.v) <= tol
        check_state(H.hdet_get_state(h), orc)
    assert not torch.equal(untouched, theta[:, 5])
    # after the sync step t = 6 and one more update the planes differ again; a final converge
    # makes all replicas identical over the whole 1e9 columns (Algorithm 1, return)
    H.hdet_converge(h)
    for r in range(1, n):
        assert torch.equal(theta[0], theta[r])
    H.hdet_destroy(h)
    del theta, g, m, v
    torch.cuda.empty_cache()
