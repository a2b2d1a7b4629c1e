#!/usr/bin/env python3
"""Throughput of the DQN training step on one MI355X.

A "step" is one pass of the whole hot path over one minibatch drawn from a device-resident
1,000,000-frame replay ring: prioritized sampling, frame-stack gather, three forward passes
(online on s and s', target on s'), dueling head, Double-DQN target, Huber loss, backward,
RMSProp, priority update.  Inputs are synthetic (seeded i.i.d. uniform bytes with Atari's
shapes) and already resident in HBM when the timed region starts.

Prints ONE JSON line.  `value` is train steps/s of the headline workload; `roofline` describes
the kernel that takes the most time in that workload (timed live with HIP events on the
launch stream); `cpu_baseline` is the CPU oracle timed on a bounded sample of the same
workload; `also` carries the batch-32 fp32 configuration of the same metric.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

F_CONV1, F_CONV2, F_CONV3, F_FC1 = 6553600, 5308416, 3612672, 3211264
PEAK = {"fp32": 157.3e12, "bf16": 2.5e15}
HBM_PEAK = 8.0e12


def flops_per_launch(B, R):
    """Algorithmic flop (2*MAC) of each GEMM kernel for one training step of batch B."""
    head = 2 * 512 * R
    return {
        "conv1_fwd": 3 * B * F_CONV1, "conv2_fwd": 3 * B * F_CONV2, "conv3_fwd": 3 * B * F_CONV3,
        "fc1_fwd": 3 * B * F_FC1, "head_train": 4 * B * head, "head_wgrad": B * head,
        "fc1_dgrad": B * F_FC1, "fc1_wgrad": B * F_FC1, "conv3_dgrad": B * F_CONV3,
        "conv3_wgrad": B * F_CONV3, "conv2_dgrad": B * F_CONV2, "conv2_wgrad": B * F_CONV2,
        "conv1_wgrad": B * F_CONV1,
    }


def bytes_per_launch(B, n_params, bf16):
    """Algorithmic HBM bytes of the bandwidth-bound kernels."""
    return {
        "gather": B * 5 * 7056 * 2,                       # read 5 ring frames, write the 5-stack
        "rmsprop": n_params * (22 if bf16 else 20),       # r/w theta, v; read g (+ bf16 copy)
    }


def step_flops(B, R):
    fwd = F_CONV1 + F_CONV2 + F_CONV3 + F_FC1 + 2 * 512 * R
    return B * (3 * fwd + 2 * fwd - F_CONV1)


def build_model(dqn, synth, torch, B, precision, capacity, K=18):
    cfg = dqn.make_config(num_actions=K, dueling=1, double_q=1, precision=precision, loss_kind=1,
                          huber_delta=1.0, gamma=0.99, lr=2.5e-4, rms_decay=0.95, rms_eps=0.01,
                          max_batch=B, max_act_batch=32, replay_capacity=capacity, per_alpha=0.6,
                          per_eps=1e-6, seed=1804, target_seed=5834)
    m = dqn.Dqn(cfg)
    chunk = 25000
    for s0 in range(0, capacity, chunk):
        n = min(chunk, capacity - s0)
        fr = synth.frames(21, torch.arange(s0, s0 + n, device="cuda"), device="cuda")
        m.replay_write(s0, fr, synth.actions(40, n, K, "cuda", first=s0),
                       synth.rewards(41, n, "cuda", first=s0), synth.dones(42, n, 0.01, "cuda", first=s0))
        torch.cuda.synchronize()
        del fr
    m.per_fill(synth.exp_priorities(9, capacity, "cuda"))
    torch.cuda.synchronize()
    return m


def time_steps(m, torch, B, steps, warmup, seed0=0):
    for i in range(warmup):
        m.train_step(B, None, beta=0.4, draw_seed=seed0 + i, outputs=False)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        m.train_step(B, None, beta=0.4, draw_seed=seed0 + warmup + i, outputs=False)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) / 1e3


def profile_kernels(m, torch, B, steps, seed0):
    m.profile_begin()
    for i in range(steps):
        m.train_step(B, None, beta=0.4, draw_seed=seed0 + i, outputs=False)
    return m.profile_end()


def check_health(m, torch, B):
    """The throughput run must leave a finite loss and a self-consistent tree."""
    out = m.train_step(B, None, beta=0.4, draw_seed=123456)
    loss = float(out["loss"][0])
    tree = m.tree
    root = float(tree[1])
    leaves = float(tree[m.L:2 * m.L].double().sum())
    assert loss == loss and abs(loss) < 1e6, loss
    assert abs(root - leaves) <= 1e-4 * leaves, (root, leaves)
    return loss


def cpu_baseline(torch, synth, B, sample_rows):
    """The CPU oracle on `sample_rows` rows of the same workload, scaled to a B-row step."""
    import numpy as np
    import oracle
    K = 18
    p = synth.he_uniform_params(1804, K, 1)
    pt = synth.he_uniform_params(5834, K, 1)
    s, sn, a, r, d = synth.batch(11, sample_rows, K)
    cfg = oracle.make_config(K, 1, 1, 1)
    theta = p.copy(); v = np.zeros_like(p)
    args = (s.numpy(), sn.numpy(), a.numpy(), r.numpy(), d.numpy())
    t0 = time.perf_counter()
    reps = 0
    while True:
        oracle.train_step(cfg, theta, pt, v, *args)
        reps += 1
        el = time.perf_counter() - t0
        if el > 10.0 or reps >= 20:
            break
    per_step = el / reps * (B / sample_rows)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count()))
    return {"value": 1.0 / per_step, "unit": "train steps/s", "cores": cores, "kind": "oracle",
            "sample": "%d full oracle steps (fp64, explicit batch) on %d of the %d rows, time scaled by %d/%d"
                      % (reps, sample_rows, B, B, sample_rows)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--batch", type=int, default=512)
    ap.add_argument("--precision", choices=["fp32", "bf16"], default="bf16")
    ap.add_argument("--capacity", type=int, default=1_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the batch-32 fp32 side measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a one-GPU training step (no collectives, no sharding); "
                 "run it with --gpus 1")

    import torch
    from paper_1804_05834_amd import dqn, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    dqn.lib()

    B, K, R = args.batch, 18, 19
    prec = 1 if args.precision == "bf16" else 0
    m = build_model(dqn, synth, torch, B, prec, args.capacity)
    wall, dev_s = time_steps(m, torch, B, args.steps, args.warmup)
    ms_per_step = wall / args.steps * 1e3
    value = args.steps / wall

    prof = profile_kernels(m, torch, B, min(args.steps, 100), seed0=10_000_000)
    loss = check_health(m, torch, B)
    fl = flops_per_launch(B, R)
    by = bytes_per_launch(B, m.n, prec == 1)
    name = max(prof, key=lambda k: prof[k][1])
    cnt, tot_ms = prof[name]
    avg_s = tot_ms / cnt / 1e3
    if name in fl:
        roof = {"kernel": name, "bound": "mfma", "achieved": fl[name] / avg_s / 1e12,
                "peak": PEAK[args.precision] / 1e12, "unit": "TFLOP/s"}
    else:
        roof = {"kernel": name, "bound": "hbm", "achieved": by.get(name, 0) / avg_s / 1e9,
                "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None
    roof["avg_us"] = avg_s * 1e6
    kernels = {k: round(v[1] / v[0] * 1e3, 2) for k, v in sorted(prof.items(), key=lambda kv: -kv[1][1])}

    res = {
        "metric": "DQN train steps/s (84x84x4, dueling Double-DQN + PER, 1M-frame replay)",
        "value": value, "unit": "train steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.precision, "data": "synthetic",
        "config": {"workload": "dueling Double-DQN + prioritized replay train step, K=18, batch %d, %s, "
                               "%d-frame device replay ring, %d consecutive steps"
                               % (B, args.precision, args.capacity, args.steps),
                   "batch": B, "num_actions": K},
        "mfma_frac_step": step_flops(B, R) * value / PEAK[args.precision],
        "device_ms_per_step": dev_s / args.steps * 1e3,
        "final_loss": loss,
        "kernel_avg_us": kernels,
        "roofline": roof,
    }
    m.close()
    del m
    torch.cuda.empty_cache()

    if not args.no_also and not (B == 32 and prec == 0):
        m32 = build_model(dqn, synth, torch, 32, 0, args.capacity)
        w32, d32 = time_steps(m32, torch, 32, args.steps, args.warmup)
        res["also"] = {"workload": "same step, batch 32, fp32", "value": args.steps / w32,
                       "unit": "train steps/s", "ms_per_step": w32 / args.steps * 1e3,
                       "device_ms_per_step": d32 / args.steps * 1e3,
                       "mfma_frac_step": step_flops(32, R) * args.steps / w32 / PEAK["fp32"]}
        m32.close()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(torch, synth, B, min(B, 64))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
