"""Benchmark of the HDET hot path on one MI355X.

Workload (default): the flat-buffer fan-out + converge case -- N = 8 replicas x P = 1e9
fp32 parameters, AdamW state per replica, per-replica synthetic gradients ~N(0, (1e-3)^2),
alpha = 0.1, converge every T = 16 steps fused into the sync-step update, auto-LR controller
on with injected losses.  A step is one pass of the whole path: hdet_fanout_step, and on
sync steps hdet_converge + hdet_autolr_update.  All buffers are resident in HBM before the
timed region starts.

Prints ONE JSON line (see the keys below).  `roofline` is for the update kernel:
algorithmic bytes (28 B per replica-element: theta, g, m, v read, theta, m, v written)
divided by the kernel's average duration measured with HIP events on the library's stream.
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ADAMW_BYTES = 28          # per replica-element per update
CONVERGE_BYTES = 8        # standalone converge: 4 read + 4 written

# HBM bytes per launch of the update kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE (scaled by
# what the same counters read for a plain 4e9-byte copy: x2.000 and x1.000), measured on the
# default workload; valid only for the kernel source it was taken with.
TRAFFIC_KERNEL_SHA = "86fe73c12446da6d"
TRAFFIC_BYTES_PER_REPLICA_ELEMENT = 223.998e9 / 8e9
TRAFFIC_SOURCE = "profiles/update_kernels_flat_N8_P1e9_hbm_counters.txt"


def measured_traffic(n, p):
    import hashlib
    h = hashlib.sha256()
    try:
        for name in ("hdet_update.hip", "hdet_update_math.h"):      # the kernels and their arithmetic
            h.update(open(os.path.join(ROOT, "paper_2604_24708_amd", "csrc", name), "rb").read())
    except OSError:
        return None
    sha = h.hexdigest()[:16]
    if sha != TRAFFIC_KERNEL_SHA or (n, p) != (8, 1_000_000_000):
        return None      # kernel or workload changed since the counters were taken
    return TRAFFIC_BYTES_PER_REPLICA_ELEMENT * n * p


def oracle_baseline(n, t_sync, p_sample, steps):
    """The CPU oracle as it stands on a bounded sample: same N, T, optimizer; P = p_sample.  Its flat path is
    element-wise numpy, which runs on one thread whatever the size of the BLAS pool.  Returns seconds."""
    import numpy as np
    import hdet_inputs as I
    from oracle import hdet_oracle as O
    cfg = O.Config(n_replicas=n, total_steps=steps, sync_interval=t_sync, warm_steps=0, lr_max=1e-3,
                   alpha=0.1, autolr_enabled=True, optimizer=O.ADAMW, weight_decay=0.01,
                   grad_mode=O.GRAD_PER_REPLICA, seed=7)
    orc = O.HDETOracle(cfg, I.flat_theta0(n, p_sample, 5))
    g = I.flat_grads(n, p_sample, 99, 1)
    t0 = time.perf_counter()
    for t in range(1, steps + 1):
        orc.step(g, 1.0 + 0.01 * np.arange(n))
    return time.perf_counter() - t0


def _oracle_chunk(job):
    n, t_sync, p_chunk, steps = job
    if p_chunk == 0:
        return 0.0          # start-up call: the process has imported what it needs
    return oracle_baseline(n, t_sync, p_chunk, steps)


def oracle_baseline_all_cores(n, t_sync, p_sample, steps):
    """The same oracle run on every host core at once: the update and the converge are element-wise in P, so
    each process takes a slice of the parameter axis (the controller's N scalars are recomputed by each).
    Returns (wall seconds, processes)."""
    import concurrent.futures
    import multiprocessing
    procs = max(1, min(os.cpu_count() or 1, 16))
    chunk = p_sample // procs
    with concurrent.futures.ProcessPoolExecutor(procs, mp_context=multiprocessing.get_context("spawn")) as ex:
        list(ex.map(_oracle_chunk, [(n, t_sync, 0, steps)] * procs))          # spin the processes up
        t0 = time.perf_counter()
        list(ex.map(_oracle_chunk, [(n, t_sync, chunk, steps)] * procs))
        return time.perf_counter() - t0, procs


MFMA_BF16_PEAK_TFLOPS = 2500.0


def mlp_workload(args, shared=False, one_call=False):
    """N = 8 replicas of the 4-layer MLP 1024-4096-4096-4096-1000, batch 256 per replica, bf16
    GEMMs with fp32 master weights, AdamW, one-cycle 1000 steps peak 3e-4, alpha 0.1, T = 16,
    auto-LR on.  A step = forward/backward + fan-out update (+ converge + controller on sync
    steps).  shared: the paper's own mode -- every replica applies the replica mean of the gradients
    (formed as one gradient plane by the model path) and AdamW's moments are kept once.
    one_call: hdet_train_step instead of hdet_forward_backward + hdet_fanout_step (the weight matrices' updates are
    then applied inside the products that form their gradients).  Returns a dict of measurements."""
    import numpy as np
    import torch
    import hdet_inputs as I
    import paper_2604_24708_amd as H
    dev = torch.device("cuda:0")
    n, B, T = 8, 256, 16
    widths = [1024, 4096, 4096, 4096, 1000]
    P = I.mlp_param_count(widths)
    stride = (P + 63) // 64 * 64          # planes start on 256-byte boundaries
    total = max(1000, args.warmup + args.steps)
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(I.mlp_init(1, widths, I.SEED_INIT)).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.zeros_like(theta)
    if shared:
        m, v = m[:1], v[:1]
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    x = torch.empty((n, B, widths[0]), dtype=torch.float32, device=dev)
    I.device_normal_(x, I.SEED_DATA, 1.0)
    y = torch.randint(0, widths[-1], (n, B), dtype=torch.int32, device=dev,
                      generator=torch.Generator(device=dev).manual_seed(I.SEED_TEACHER))
    stream = torch.cuda.current_stream()
    cfg = H.make_config(n_replicas=n, sync_interval=T, total_steps=total, warm_steps=int(0.3 * total),
                        lr_max=3e-4, alpha=0.1, autolr_enabled=1, optimizer=H.HDET_ADAMW, weight_decay=0.01,
                        grad_mode=H.HDET_GRAD_SHARED if shared else H.HDET_GRAD_PER_REPLICA, shared_opt_state=int(shared),
                        precision=H.HDET_BF16_GEMM_FP32_MASTER,
                        model_kind=H.HDET_MLP, widths=widths, batch=B, seed=I.SEED_PERM,
                        stream=stream.cuda_stream)
    _, _, ws_bytes = H.hdet_workspace_bytes(cfg, stride)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    h = H.hdet_create(cfg, theta, m, v, grads=g, params_bf16=shadow, workspace=ws, plane_stride=stride)
    ev = []

    def step(t, timed):
        if timed:
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(stream)
        if one_call:
            H.hdet_train_step(h, x, y, H.HDET_FUSE_CONVERGE)
        else:
            H.hdet_forward_backward(h, x, y)
        if timed:
            e[1].record(stream)
        if not one_call:
            H.hdet_fanout_step(h, None, H.HDET_FUSE_CONVERGE)
        if timed:
            e[2].record(stream)
            ev.append(e)
        if t % T == 0:
            H.hdet_converge(h)
            H.hdet_autolr_update(h, None)

    for t in range(1, args.warmup + 1):
        step(t, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup + 1, args.warmup + args.steps + 1):
        step(t, True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fb_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev)
    up_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / len(ev)
    st = H.hdet_get_state(h)
    H.hdet_destroy(h)
    fwd_flop = sum(2.0 * B * widths[i] * widths[i + 1] for i in range(len(widths) - 1))
    dgrad_flop = sum(2.0 * B * widths[i] * widths[i + 1] for i in range(1, len(widths) - 1))
    gemm_flop = n * (2 * fwd_flop + dgrad_flop)          # forward + wgrad + dgrad (none for layer 1)
    tflops = gemm_flop / (fb_ms * 1e-3) / 1e12
    # update bytes per parameter: theta read + written and the bf16 copy written per replica; then either g, m, v per
    # replica (30 N), or one gradient plane and one set of moments (10 N + 20)
    upd_bytes = (10.0 * n + 20.0) * P if shared else 30.0 * n * P
    return {"workload": "N=8 x MLP 1024-4096-4096-4096-1000, batch 256/replica, bf16 GEMM + fp32 master, AdamW, T=16"
                        + (", shared gradients (one gradient plane, one set of moments)" if shared else "")
                        + (", one call per step (weight updates inside the weight-gradient products)" if one_call else ""),
            "replica_steps_per_s": n * args.steps / dt, "ms_per_step": dt / args.steps * 1e3,
            # one call per step: the update is part of the first figure
            "forward_backward_ms": fb_ms, "update_ms": up_ms, "update_algorithmic_bytes": upd_bytes,
            "update_GBps": None if one_call else upd_bytes / (up_ms * 1e-3) / 1e9,
            "gemm_flop_per_step": gemm_flop, "forward_backward_TFLOPs": tflops,
            "mfma_frac_of_bf16_peak": tflops / MFMA_BF16_PEAK_TFLOPS,
            "loss_first_replica": float(st.l_step[0])}


def transformer_workload(args):
    """N = 8 replicas of a decoder-only transformer: 6 layers, d_model 512, 8 heads, FFN 2048,
    seq 256, vocab 32000, 16 sequences per replica, Zipf(1.1) token ids, bf16 GEMMs with fp32
    master weights, AdamW, one-cycle 2000 steps peak 6e-4, alpha 0.15, T = 32, auto-LR on."""
    import torch
    import hdet_inputs as I
    import paper_2604_24708_amd as H
    dev = torch.device("cuda:0")
    n, B, T = 8, 16, 32
    cfg = dict(n_blocks=6, d_model=512, n_heads=8, d_ff=2048, seq_len=256, vocab=32000)
    lr_max, alpha, extra = 6e-4, 0.15, []
    if getattr(args, "tf_config", "6L") == "12L":
        # the larger configuration: 12 layers, d_model 1024, 16 heads, FFN 4096, seq 512, T = 64, and three
        # explored scalars (rate; dropout base 0.1 spread 1.0; weight decay base 0.05 spread 0.5)
        T = 64
        cfg = dict(n_blocks=12, d_model=1024, n_heads=16, d_ff=4096, seq_len=512, vocab=32000)
        lr_max = 3e-4
        extra = [(H.HDET_CH_DROPOUT, 0.1, 1.0, 0.5, 0.0, 0.45), (H.HDET_CH_WD, 0.05, 0.5, 0.5, 0.0, float("inf"))]
    P = I.transformer_param_count(cfg)
    stride = (P + 63) // 64 * 64          # planes start on 256-byte boundaries
    total = max(2000, args.warmup + args.steps)
    theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
    theta[:, :P] = torch.from_numpy(I.transformer_init(1, cfg, I.SEED_INIT)).to(dev)
    m, v, g = torch.zeros_like(theta), torch.zeros_like(theta), torch.zeros_like(theta)
    shared = getattr(args, "model_grad_mode", "per_replica") == "shared"
    one_call = bool(getattr(args, "one_call", False))
    if shared:
        m, v = m[:1], v[:1]
    shadow = torch.zeros((n, stride), dtype=torch.bfloat16, device=dev)
    ids, tgt = I.zipf_tokens(n, B, cfg["seq_len"], cfg["vocab"], I.SEED_DATA, 0)
    ids, tgt = torch.from_numpy(ids).to(dev), torch.from_numpy(tgt).to(dev)
    stream = torch.cuda.current_stream()
    lc = H.make_config(n_replicas=n, sync_interval=T, total_steps=total, warm_steps=int(0.3 * total),
                       lr_max=lr_max, alpha=alpha, autolr_enabled=1, optimizer=H.HDET_ADAMW, weight_decay=0.01,
                       grad_mode=H.HDET_GRAD_SHARED if shared else H.HDET_GRAD_PER_REPLICA, shared_opt_state=int(shared),
                       precision=H.HDET_BF16_GEMM_FP32_MASTER,
                       model_kind=H.HDET_TRANSFORMER, batch=B, seed=I.SEED_PERM, stream=stream.cuda_stream,
                       extra=extra, **cfg)
    _, _, ws_bytes = H.hdet_workspace_bytes(lc, stride)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    h = H.hdet_create(lc, theta, m, v, grads=g, params_bf16=shadow, workspace=ws, plane_stride=stride)
    ev = []

    def step(t, timed):
        if timed:
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(stream)
        if one_call:
            H.hdet_train_step(h, ids, tgt, H.HDET_FUSE_CONVERGE)
        else:
            H.hdet_forward_backward(h, ids, tgt)
        if timed:
            e[1].record(stream)
        if not one_call:
            H.hdet_fanout_step(h, None, H.HDET_FUSE_CONVERGE)
        if timed:
            e[2].record(stream)
            ev.append(e)
        if t % T == 0:
            H.hdet_converge(h)
            H.hdet_autolr_update(h, None)

    for t in range(1, args.warmup + 1):
        step(t, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup + 1, args.warmup + args.steps + 1):
        step(t, True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    fb_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / len(ev)
    up_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / len(ev)
    st = H.hdet_get_state(h)
    H.hdet_destroy(h)
    M, d, ff, V, S, L, nh = B * cfg["seq_len"], cfg["d_model"], cfg["d_ff"], cfg["vocab"], cfg["seq_len"], cfg["n_blocks"], cfg["n_heads"]
    lin = L * (2.0 * M * d * 3 * d + 2.0 * M * d * d + 2 * 2.0 * M * d * ff) + 2.0 * M * d * V
    attn = L * 2 * 2.0 * B * nh * S * S * (d // nh)          # scores and P V, full (unmasked) squares
    gemm_flop = n * 3 * (lin + attn)                          # forward + dgrad + wgrad
    tflops = gemm_flop / (fb_ms * 1e-3) / 1e12
    return {"workload": f"N=8 x decoder-only transformer {L}L d{d} h{nh} ffn{ff} seq{S} vocab{V}, {B} seq/replica, "
                        f"bf16 GEMM + fp32 master, AdamW, T={T}, {1 + len(extra)} channel(s)"
                        + (", shared gradients (one gradient plane, one set of moments)" if shared else "")
                        + (", one call per step (weight updates inside the weight-gradient products)" if one_call else ""),
            "n_params": P, "replica_steps_per_s": n * args.steps / dt, "tokens_per_s": n * M * args.steps / dt,
            "ms_per_step": dt / args.steps * 1e3, "forward_backward_ms": fb_ms, "update_ms": up_ms,
            "update_GBps": None if one_call else ((10.0 * n + 20.0) if shared else 30.0 * n) * P / (up_ms * 1e-3) / 1e9,
            "gemm_flop_per_step": gemm_flop,
            "forward_backward_TFLOPs": tflops, "mfma_frac_of_bf16_peak": tflops / MFMA_BF16_PEAK_TFLOPS,
            "loss_first_replica": float(st.l_step[0])}


def cfg0_leg():
    """The small parity configuration as a latency figure: N = 4 replicas of the MLP 64-128-10 in fp32, batch 32,
    SGD momentum 0.9, one-cycle peak 0.05 over 40 steps, alpha 0.2, T = 4, auto-LR on; the full 40-step run on the
    device (second run timed, kernels warm) and in the oracle."""
    import numpy as np
    import torch
    import hdet_inputs as I
    import paper_2604_24708_amd as H
    from oracle import hdet_oracle as O
    from oracle import mlp_oracle as M
    dev = torch.device("cuda:0")
    n, B, T, S = 4, 32, 4, 40
    widths = [64, 128, 10]
    P = I.mlp_param_count(widths)
    stride = (P + 3) // 4 * 4
    th0 = I.mlp_init(n, widths, I.SEED_INIT)
    batches = [I.mlp_batch(n, B, widths[0], I.SEED_DATA, t, widths, I.SEED_TEACHER) for t in range(1, S + 1)]
    dev_batches = [(torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev)) for x, y in batches]
    stream = torch.cuda.current_stream()

    def run_device():
        theta = torch.zeros((n, stride), dtype=torch.float32, device=dev)
        theta[:, :P] = torch.from_numpy(th0).to(dev)
        m, g = torch.zeros_like(theta), torch.zeros_like(theta)
        cfg = H.make_config(n_replicas=n, sync_interval=T, total_steps=S, warm_steps=12, lr_max=0.05, alpha=0.2,
                            autolr_enabled=1, optimizer=H.HDET_SGDM, momentum=0.9, weight_decay=0.0,
                            grad_mode=H.HDET_GRAD_PER_REPLICA, precision=H.HDET_FP32, model_kind=H.HDET_MLP,
                            widths=widths, batch=B, seed=I.SEED_PERM, stream=stream.cuda_stream)
        _, _, ws_bytes = H.hdet_workspace_bytes(cfg, stride)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        h = H.hdet_create(cfg, theta, m, None, grads=g, workspace=ws, plane_stride=stride)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(1, S + 1):
            H.hdet_forward_backward(h, *dev_batches[t - 1])
            H.hdet_fanout_step(h, None, H.HDET_FUSE_CONVERGE)
            if t % T == 0:
                H.hdet_converge(h)
                H.hdet_autolr_update(h, None)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        H.hdet_destroy(h)
        return dt

    run_device()
    gpu_s = run_device()
    ocfg = O.Config(n_replicas=n, total_steps=S, sync_interval=T, warm_steps=12, lr_max=0.05, alpha=0.2,
                    autolr_enabled=True, optimizer=O.SGDM, momentum=0.9, weight_decay=0.0,
                    grad_mode=O.GRAD_PER_REPLICA, seed=I.SEED_PERM)
    orc = O.HDETOracle(ocfg, th0)
    t0 = time.perf_counter()
    for t in range(1, S + 1):
        x, y = batches[t - 1]
        out = [M.mlp_loss_and_grad(orc.theta[r], x[r], y[r], widths) for r in range(n)]
        orc.step(np.stack([o[1] for o in out]), [o[0] for o in out])
    cpu_s = time.perf_counter() - t0
    return {"workload": "N=4 x MLP 64-128-10 fp32, batch 32/replica, SGD momentum 0.9, 40 steps, T=4, auto-LR on",
            "gpu_run_ms": gpu_s * 1e3, "gpu_ms_per_step": gpu_s * 1e3 / S, "gpu_replica_steps_per_s": n * S / gpu_s,
            "oracle_run_ms": cpu_s * 1e3, "oracle_replica_steps_per_s": n * S / cpu_s, "oracle_cores": 1,
            "note": "launch-latency bound (9 610 parameters per replica); the oracle runs it on one thread"}


def warm_init_leg(H, theta, theta0, n, P, stride, stream):
    """Eq. 10 at the headline size: theta0 [P] read, N perturbed planes written (4 (N + 1) P algorithmic bytes)."""
    import torch
    ms = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        H.hdet_warm_init_noalloc(theta0, theta, None, P, stride, n, 0.01, 4242, stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    best = min(ms)
    nbytes = 4.0 * (n + 1) * P
    return {"ms": best, "algorithmic_bytes": nbytes, "achieved": nbytes / (best * 1e-3) / 1e9, "unit": "GB/s",
            "frac_of_hbm_peak": nbytes / (best * 1e-3) / 1e9 / HBM_PEAK_GBS}


def stream_reference(a, b):
    """What the memory system gives plain streams of the headline size on this machine, same buffers: a device copy
    (1 read + 1 write per element) and a three-stream add (2 reads + 1 write), by the tensor library's kernels."""
    import torch
    out = {}
    for name, fn, streams in (("copy_1r1w", lambda: b.copy_(a), 2), ("add_2r1w", lambda: torch.add(a, b, out=b), 3)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        out[name] = {"ms": ms, "GBps": streams * a.numel() * 4 / (ms * 1e-3) / 1e9}
    return out


def shared_state_leg(H, I, theta, g, m, v, n, P, T, stride, stream, args):
    """2 T steps of shared-gradient AdamW with one plane of each moment, timed like the main leg."""
    import torch
    steps, warm = 2 * T, 4
    m1, v1 = m[:1], v[:1]
    m1.zero_(); v1.zero_()
    cfg = H.make_config(n_replicas=n, sync_interval=T, total_steps=steps + warm, warm_steps=int(0.3 * (steps + warm)),
                        lr_max=1e-3, alpha=0.1, autolr_enabled=1, optimizer=H.HDET_ADAMW, weight_decay=0.01,
                        grad_mode=H.HDET_GRAD_SHARED, shared_opt_state=1, model_kind=H.HDET_FLAT, n_params=P,
                        seed=I.SEED_PERM, stream=stream.cuda_stream)
    h = H.hdet_create(cfg, theta, m1, v1, plane_stride=stride)
    losses = [1.0 + 0.01 * r for r in range(n)]
    ev = []
    t0 = None
    for t in range(1, steps + warm + 1):
        if t == warm + 1:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        if t > warm:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
        H.hdet_fanout_step(h, g, H.HDET_FUSE_CONVERGE)
        if t > warm:
            e1.record(stream)
            ev.append((e0, e1))
        if t % T == 0:
            H.hdet_converge(h)
            H.hdet_autolr_update(h, losses)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    H.hdet_destroy(h)
    ms = sum(a.elapsed_time(b) for a, b in ev) / len(ev)
    nbytes = (12 * n + 16) * P
    return {"replica_steps_per_s": n * steps / dt, "ms_per_step": dt / steps * 1e3, "kernel_ms": ms,
            "algorithmic_bytes_per_launch": nbytes, "achieved": nbytes / (ms * 1e-3) / 1e9, "unit": "GB/s",
            "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--params", type=float, default=1e9, help="P per replica (default: the benchmark's 1e9)")
    ap.add_argument("--replicas", type=int, default=8)
    ap.add_argument("--sync-interval", type=int, default=16)
    ap.add_argument("--grad-mode", choices=["per_replica", "shared"], default="per_replica")
    ap.add_argument("--shared-state", action="store_true",
                    help="with --grad-mode shared: one set of AdamW moments for all replicas (12N+16 B per element)")
    ap.add_argument("--unfused", action="store_true", help="standalone converge kernel on sync steps")
    ap.add_argument("--variant", type=int, default=0, help="update kernel selection (0 = default)")
    ap.add_argument("--blocks", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", choices=["flat", "mlp", "transformer", "both"], default="both",
                    help="flat: the headline flat-buffer case only; mlp: only the bf16 MLP case (printed as its own "
                         "JSON line); transformer: only the bf16 transformer case; both: the headline line with the "
                         "MLP and transformer figures attached as `mlp_bf16` and `transformer_bf16`")
    ap.add_argument("--model-grad-mode", choices=["per_replica", "shared"], default="per_replica",
                    help="--workload mlp / transformer: shared = the replica mean of the gradients as one plane, one set of moments")
    ap.add_argument("--one-call", action="store_true",
                    help="--workload mlp / transformer: hdet_train_step (forward, backward and update in one call)")
    ap.add_argument("--tf-config", choices=["6L", "12L"], default="6L",
                    help="transformer workload: 6 layers d512 seq256 (default) or 12 layers d1024 seq512 with 3 channels")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of known size (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the replicas are an axis in one GPU's memory); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    # The CPU oracle first, before this process touches the GPU: its all-cores figure starts worker processes.
    cpu_baseline = None
    if args.workload in ("both", "flat") and not args.no_cpu_baseline:
        n, P, T = args.replicas, int(args.params), args.sync_interval
        p_sample, o_steps = 12_000_000, T + 1
        odt = oracle_baseline(n, T, p_sample, o_steps)
        cpu_baseline = {"value": n * o_steps / odt * (p_sample / P), "unit": "replica-steps/s",
                        "cores": 1, "kind": "oracle",
                        "sample": f"oracle (numpy, fp64 arithmetic, element-wise: one thread) on N={n} x P={p_sample} for "
                                  f"{o_steps} steps incl. one converge+controller, {odt:.1f} s; scaled linearly in P to P={P:.3g}"}
        p_all = 64_000_000
        adt, procs = oracle_baseline_all_cores(n, T, p_all, o_steps)
        cpu_baseline["all_cores"] = {"value": n * o_steps / adt * (p_all / P), "unit": "replica-steps/s", "cores": procs,
                                     "sample": f"the same oracle in {procs} processes, each on a slice of P={p_all} "
                                               f"(element-wise in P), {adt:.1f} s wall; scaled linearly in P to P={P:.3g}"}

    import torch
    import hdet_inputs as I
    import paper_2604_24708_amd as H

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "mlp":
        print(json.dumps(mlp_workload(args, shared=args.model_grad_mode == "shared", one_call=args.one_call)))
        return
    if args.workload == "transformer":
        print(json.dumps(transformer_workload(args)))
        return
    n, P, T = args.replicas, int(args.params), args.sync_interval
    stride = (P + 63) // 64 * 64          # planes start on 256-byte boundaries
    total = args.warmup + args.steps

    if args.shared_state and args.grad_mode != "shared":
        print("bench.py: --shared-state needs --grad-mode shared", file=sys.stderr)
        sys.exit(2)
    theta = torch.empty((n, stride), dtype=torch.float32, device=dev)
    g = torch.empty_like(theta)
    m = torch.zeros((1 if args.shared_state else n, stride), dtype=torch.float32, device=dev)
    v = torch.zeros_like(m)
    I.device_normal_(theta[0], I.SEED_INIT, 0.02)          # identical replicas at t = 0
    for r in range(1, n):
        theta[r].copy_(theta[0])
    I.device_normal_(g, I.SEED_GRADS, 1e-3)                # per-replica gradients, fixed over the run
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    cfg = H.make_config(n_replicas=n, sync_interval=T, total_steps=total, warm_steps=int(0.3 * total),
                        lr_max=1e-3, alpha=0.1, autolr_enabled=1, optimizer=H.HDET_ADAMW,
                        weight_decay=0.01,
                        grad_mode=H.HDET_GRAD_SHARED if args.grad_mode == "shared" else H.HDET_GRAD_PER_REPLICA,
                        shared_opt_state=int(args.shared_state),
                        model_kind=H.HDET_FLAT, n_params=P, seed=I.SEED_PERM, stream=stream.cuda_stream)
    h = H.hdet_create(cfg, theta, m, v, plane_stride=stride)
    if args.variant or args.blocks:
        H.hdet_set_launch_shape(h, args.variant, args.blocks)
    losses = [1.0 + 0.01 * r for r in range(n)]
    flags = 0 if args.unfused else H.HDET_FUSE_CONVERGE

    upd_ev, conv_ev = [], []

    def step(t, timed):
        if timed:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
        H.hdet_fanout_step(h, g, flags)
        if timed:
            e1.record(stream)
            upd_ev.append((e0, e1))
        if t % T == 0:
            if timed and args.unfused:
                c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                c0.record(stream)
            H.hdet_converge(h)
            if timed and args.unfused:
                c1.record(stream)
                conv_ev.append((c0, c1))
            H.hdet_autolr_update(h, losses)

    if args.copy_calibration:
        # 3 x (one plane read + one plane written) by the runtime's plain device copy
        src, dst = g[0].view(-1)[:P], m[0].view(-1)[:P]
        for _ in range(3):
            dst.copy_(src)
        dst.zero_()
    for t in range(1, args.warmup + 1):
        step(t, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup + 1, total + 1):
        step(t, True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    upd_all = sorted(a.elapsed_time(b) for a, b in upd_ev)
    upd_ms = sum(upd_all) / len(upd_all)
    bytes_per_launch = (12 * n + 16) * P if args.shared_state else ADAMW_BYTES * n * P
    achieved = bytes_per_launch / (upd_ms * 1e-3) / 1e9
    st = H.hdet_get_state(h)
    H.hdet_destroy(h)

    out = {
        "metric": "replica-steps/s at N=8 (fused update+converge, flat buffers)",
        "value": n * args.steps / dt,
        "unit": "replica-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"flat fan-out+converge: N={n} replicas x P={P:.3g} fp32, AdamW(0.9,0.999,wd 0.01), "
                               f"alpha=0.1, T={T}, grads ~N(0,1e-3^2) per replica, {args.grad_mode} gradients"
                               f"{' with one set of moments' if args.shared_state else ''}, "
                               f"converge {'standalone' if args.unfused else 'fused into the sync-step update'}, auto-LR on",
                   "n_replicas": n, "n_params": P, "sync_interval": T, "grad_mode": args.grad_mode,
                   "controller_updates": int(st.k)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(n, P),
                     # not a reading of this run: the stored counter figure of the summary named here, null once the
                     # kernel source or the workload differs from what the counters were taken on
                     "traffic_source": TRAFFIC_SOURCE if measured_traffic(n, P) is not None else None,
                     "kernel": "hdet_update_kernel", "kernel_ms": upd_ms,
                     "kernel_ms_median": upd_all[len(upd_all) // 2], "kernel_ms_min": upd_all[0],
                     "algorithmic_bytes_per_launch": bytes_per_launch},
    }
    if conv_ev:
        cms = sum(a.elapsed_time(b) for a, b in conv_ev) / len(conv_ev)
        out["converge_standalone"] = {"kernel_ms": cms, "achieved": CONVERGE_BYTES * n * P / (cms * 1e-3) / 1e9,
                                      "unit": "GB/s"}
    if not args.shared_state:
        out["stream_reference"] = stream_reference(g.view(-1)[:n * P], m.view(-1)[:n * P])
        m.zero_()
        out["warm_init"] = warm_init_leg(H, theta, g[0, :P], n, P, stride, stream)
        # the paper's own mode on the same buffers: every replica applies the mean gradient, and
        # AdamW's moments, which then do not depend on the replica, are kept once
        out["shared_gradient_one_set_of_moments"] = shared_state_leg(H, I, theta, g, m, v, n, P, T, stride, stream, args)
    del theta, g, m, v
    torch.cuda.empty_cache()
    if args.workload == "both":
        out["mlp_bf16"] = mlp_workload(args)
        torch.cuda.empty_cache()
        out["mlp_bf16_shared_gradient"] = mlp_workload(args, shared=True)
        torch.cuda.empty_cache()
        out["mlp_bf16_one_call"] = mlp_workload(args, one_call=True)
        torch.cuda.empty_cache()
        targs = argparse.Namespace(**vars(args))
        targs.steps, targs.warmup = min(args.steps, 16), min(args.warmup, 4)
        out["transformer_bf16"] = transformer_workload(targs)
        torch.cuda.empty_cache()
        targs.model_grad_mode = "shared"
        out["transformer_bf16_shared_gradient"] = transformer_workload(targs)
        targs.model_grad_mode = "per_replica"
        torch.cuda.empty_cache()
        targs.one_call = True
        out["transformer_bf16_one_call"] = transformer_workload(targs)
        targs.one_call = False
        torch.cuda.empty_cache()
        targs.tf_config, targs.steps, targs.warmup = "12L", min(args.steps, 8), min(args.warmup, 2)
        out["transformer_12L_bf16"] = transformer_workload(targs)
        torch.cuda.empty_cache()
        targs.one_call = True
        out["transformer_12L_bf16_one_call"] = transformer_workload(targs)
        targs.one_call = False
        torch.cuda.empty_cache()
        out["mlp_fp32_small"] = cfg0_leg()
    if cpu_baseline is not None:
        out["cpu_baseline"] = cpu_baseline
    print(json.dumps(out))


if __name__ == "__main__":
    main()
