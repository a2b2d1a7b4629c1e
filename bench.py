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
workload; `kernels` lists every kernel of the step against its own roofline; `also` carries
the batch-32 fp32 configuration of the same metric, the acting + training loop and the
single-stream agent loop (act, store with maximal priority, train every fourth step).
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
        "conv12_fwd": 3 * B * (F_CONV1 + F_CONV2),   # bf16, larger batches: conv1 + conv2 in one launch
        "fc1_fwd": 3 * B * F_FC1, "head_train": 4 * B * head, "head_wgrad": B * head,
        "fc1_dgrad": B * F_FC1, "fc1_wgrad": B * F_FC1, "conv3_dgrad": B * F_CONV3,
        "conv3_wgrad": B * F_CONV3, "conv2_dgrad": B * F_CONV2, "conv2_wgrad": B * F_CONV2,
        "conv1_wgrad": B * F_CONV1,
        # bf16: a layer's input gradient and weight gradient share one launch
        "fc1_bwd": 2 * B * F_FC1, "conv3_bwd": 2 * B * F_CONV3, "conv2_bwd": 2 * B * F_CONV2,
        # bf16: conv2's two gradients and conv1's weight gradient in one launch
        "conv21_bwd": 2 * B * F_CONV2 + B * F_CONV1,
    }


def bytes_per_launch(B, n_params, bf16, levels=20):
    """Algorithmic HBM bytes of the kernels that move data rather than multiply."""
    return {
        "gather": B * 5 * 7056 * 2,                       # read 5 ring frames, write the 5-stack
        "sample_gather": B * 5 * 7056 * 2,                # the same, with the draw in front (fp32 path)
        "rmsprop": n_params * (22 if bf16 else 20),       # r/w theta, v; read g (+ bf16 copy)
        "per_sample": B * levels * 4,                     # one useful node per level and draw
        "per_update": B * levels * 12,                    # read sibling, write node (+ leaf) per level
    }


def gemm_bytes_per_launch(B, R, bf16):
    """Algorithmic HBM bytes (read + write) of each GEMM kernel: every operand once, no split
    partial sums, the five distinct ring frames of a transition once for the three forward passes."""
    e = 2 if bf16 else 4                       # activation / shadow-weight element
    a1, a2, a3, hid = 400 * 32 * e, 81 * 64 * e, 49 * 64 * e, 512 * 4
    w1, w2, w3, wf = 32 * 256 * e, 64 * 512 * e, 64 * 576 * e, 512 * 3136 * e
    frames = B * 5 * 7056 * (1 if bf16 else 2)   # fp32 path: conv1 also writes the gathered 5-frame stacks
    return {
        "conv1_fwd": frames + w1 + 3 * B * a1,
        "conv2_fwd": 3 * B * (a1 + a2) + w2,
        # the fused launch keeps conv1's output on the CU; only the training rows' copy goes to memory
        "conv12_fwd": frames + w1 + w2 + B * a1 + 3 * B * a2,
        "conv3_fwd": 3 * B * (a2 + a3) + w3,
        "fc1_fwd": 3 * B * (a3 + hid) + wf,
        "fc1_dgrad": B * (512 * e + 2 * a3) + wf,           # dH, ReLU mask, dX
        "conv3_dgrad": B * (a3 + 2 * a2) + w3,
        "conv2_dgrad": B * (a2 + 2 * a1) + w2,
        "conv1_wgrad": B * (4 * 7056 + a1) + 32 * 256 * 4,
        "conv2_wgrad": B * (a1 + a2) + 64 * 512 * 4,
        "conv3_wgrad": B * (a2 + a3) + 64 * 576 * 4,
        "fc1_wgrad": B * (a3 + 512 * e) + 512 * 3136 * 4,
        # the merged launches read dY and the layer input once for both gradients
        "fc1_bwd": B * (512 * e + 2 * a3) + wf + 512 * 3136 * 4,
        "conv3_bwd": B * (a3 + 2 * a2) + w3 + 64 * 576 * 4,
        "conv2_bwd": B * (a2 + 2 * a1) + w2 + 64 * 512 * 4,
        # conv1's dY stays on the CU: dY of conv2, conv1's activations (mask and conv2's weight-gradient operand),
        # the four frames; the weights and the two weight gradients
        "conv21_bwd": B * (a2 + a1 + 4 * 7056) + w2 + 64 * 512 * 4 + 32 * 256 * 4,
    }


# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs), each
# scaled by what the same counter shows for the ring-fill copy kernel of known size in the same
# run (fetch x1.949, write x0.9875).  Keyed by (kernel, batch, precision); the figures and the
# commands are in profiles/train_step_b512_bf16_hbm_traffic.md.
MEASURED_TRAFFIC = {
    ("conv12_fwd", 512, "bf16"): 46.2e6 + 28.7e6,
    ("conv3_fwd", 512, "bf16"): 16.8e6 + 9.5e6,
    ("fc1_fwd", 512, "bf16"): 19.6e6 + 12.4e6,
    ("head_train", 512, "bf16"): 13.2e6 + 1.7e6,
    ("fc1_bwd", 512, "bf16"): 13.5e6 + 9.6e6,
    ("conv3_bwd", 512, "bf16"): 10.0e6 + 11.2e6,
    ("conv21_bwd", 512, "bf16"): 50.3e6 + 16.0e6,
    ("rmsprop", 512, "bf16"): 41.1e6 + 17.1e6,
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
    fill_ring(m, synth, torch, capacity, K)
    return m


def fill_ring(m, synth, torch, capacity, K):
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


SPIN_UP_STEPS = 300   # untimed, before the counted warm-up: clocks and caches reach their steady state


def time_steps(m, torch, B, steps, warmup, seed0=0):
    """Returns (wall seconds, device seconds, host seconds spent enqueueing) for `steps` steps.
    A fixed spin-up runs first, so that a short run (--steps 20 --warmup 5) measures the same steady
    state as a long one."""
    for i in range(SPIN_UP_STEPS):
        m.train_step(B, None, beta=0.4, draw_seed=seed0 + 5_000_000 + i, outputs=False)
    torch.cuda.synchronize()
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
    # host cost of enqueueing a step, over a burst short enough that the queues never fill
    # (inside the long loop the host is held back by the device)
    burst = 20
    t1 = time.perf_counter()
    for i in range(burst):
        m.train_step(B, None, beta=0.4, draw_seed=seed0 + warmup + steps + i, outputs=False)
    t_enq = (time.perf_counter() - t1) / burst * steps
    torch.cuda.synchronize()
    return wall, e0.elapsed_time(e1) / 1e3, t_enq


def time_act_train(dqn, synth, torch, capacity, iters, warmup, E=2048, B=256, K=18):
    """The fifth configuration as a closed loop: act on E environments (epsilon 0.05), store the E
    new time steps with the maximal priority (one sub-ring of capacity / E slots per environment
    stream), train on a batch of B drawn from what the streams stored (bf16).  The observations and
    the frames that are stored rotate among pre-generated sets so they are not cache-resident; the
    ring is filled through the same store path before the clock starts."""
    cfg = dqn.make_config(num_actions=K, dueling=1, double_q=1, precision=1, loss_kind=1,
                          huber_delta=1.0, gamma=0.99, lr=2.5e-4, rms_decay=0.95, rms_eps=0.01,
                          max_batch=B, max_act_batch=E, replay_capacity=capacity, per_alpha=0.6,
                          per_eps=1e-6, seed=1804, target_seed=5834)
    m = dqn.Dqn(cfg)
    obs = [synth.states(31 + i, E, device="cuda") for i in range(4)]
    rew = [synth.rewards(41 + i, E, "cuda") for i in range(4)]
    don = [synth.dones(45 + i, E, 0.01, "cuda") for i in range(4)]
    sub = capacity // E
    for t in range(sub + 8):                       # every sub-ring full, written through the store path
        k = t % 4
        m.replay_store_envs(obs[k][:, 3].contiguous() if t < 4 else obs[k][:, t % 4].contiguous(),
                            synth.actions(40, E, K, "cuda", first=t * E), rew[k], don[k])
    torch.cuda.synchronize()
    newest = [o[:, 3].contiguous() for o in obs]   # the newest frame of every observation: what gets stored

    def loop(n, first, store, train):
        for i in range(n):
            k = i % 4
            act = m.act(obs[k], 0.05, first + i)
            if store:
                m.replay_store_envs(newest[k], act, rew[k], don[k])
            if train:
                m.train_step(B, None, beta=0.4, draw_seed=first + i, outputs=False)
        torch.cuda.synchronize()

    loop(warmup, 0, True, True)
    t0 = time.perf_counter()
    loop(iters, warmup, True, True)
    wall = time.perf_counter() - t0
    t0 = time.perf_counter()
    loop(iters, warmup + iters, False, True)
    no_store = time.perf_counter() - t0
    t0 = time.perf_counter()
    loop(iters, warmup + 2 * iters, False, False)
    act_only = time.perf_counter() - t0
    m.close()
    act_flops = E * (F_CONV1 + F_CONV2 + F_CONV3 + F_FC1 + 2 * 512 * 19)
    return {"workload": "act on %d environments (epsilon 0.05) + store their %d time steps (one sub-ring per "
                        "environment, maximal priority) + train step batch %d, bf16" % (E, E, B),
            "value": iters / wall, "unit": "act+store+train iterations/s", "ms_per_iteration": wall / iters * 1e3,
            "env_steps_per_s": E * iters / wall, "ms_per_iteration_without_store": no_store / iters * 1e3,
            "act_only_ms": act_only / iters * 1e3,
            "act_only_mfma_frac": act_flops * iters / act_only / PEAK["bf16"]}


def profile_kernels(m, torch, B, steps, seed0):
    m.profile_begin()
    for i in range(steps):
        m.train_step(B, None, beta=0.4, draw_seed=seed0 + i, outputs=False)
    return m.profile_end()


def time_variants(dqn, synth, torch, capacity, steps, warmup, K=18, B=32):
    """The four model settings of the paper's performance figure (Double DQN with a plain or a
    dueling head, uniform replay = priority exponent 0, or prioritized replay with exponent 0.6),
    each as the batch-32 fp32 step over the same ring."""
    out = []
    for name, dueling, alpha in (("double DQN", 0, 0.0), ("dueling double DQN", 1, 0.0),
                                 ("double DQN with prioritized replay", 0, 0.6),
                                 ("dueling double DQN with prioritized replay", 1, 0.6)):
        cfg = dqn.make_config(num_actions=K, dueling=dueling, double_q=1, precision=0, loss_kind=1,
                              huber_delta=1.0, gamma=0.99, lr=2.5e-4, rms_decay=0.95, rms_eps=0.01,
                              max_batch=B, max_act_batch=32, replay_capacity=capacity, per_alpha=alpha,
                              per_eps=1e-6, seed=1804, target_seed=5834)
        m = dqn.Dqn(cfg)
        fill_ring(m, synth, torch, capacity, K)
        wall, _, _ = time_steps(m, torch, B, steps, warmup)
        out.append({"setting": name, "value": steps / wall, "unit": "train steps/s"})
        m.close()
        del m
        torch.cuda.empty_cache()
    return {"workload": "the four model settings of the paper's performance figure, batch %d fp32" % B, "settings": out}


def time_agent_loop(dqn, synth, torch, capacity, env_steps, K=18, B=32):
    """The loop of Alg.1 / Alg.2 around a synthetic emulator (one environment stream, as in the
    paper): every environment step acts on one observation and stores one time step with the
    maximal priority; every fourth step trains on a batch of 32 (fp32); the target network is
    copied on Table 1's period; epsilon and beta follow Table 1's ramps.  The ring starts
    full (learning start already passed)."""
    cfg = dqn.make_config(num_actions=K, dueling=1, double_q=1, precision=0, loss_kind=1,
                          huber_delta=1.0, gamma=0.99, lr=2.5e-4, rms_decay=0.95, rms_eps=0.01,
                          max_batch=B, max_act_batch=32, replay_capacity=capacity, per_alpha=0.6,
                          per_eps=1e-6, seed=1804, target_seed=5834)
    m = dqn.Dqn(cfg)
    fill_ring(m, synth, torch, capacity, K)
    sc = dqn.schedule_default()
    pool = 256
    obs = synth.states(31, pool, device="cuda")
    frames = synth.frames(23, torch.arange(pool, device="cuda"), device="cuda")
    rew = synth.rewards(41, pool, "cuda")
    don = synth.dones(42, pool, 0.01, "cuda")
    t0 = None
    first = sc.learning_start + 1
    trains = 0
    for i in range(-40, env_steps):
        if i == 0:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        t = first + max(i, 0)
        eps, beta, train, sync = dqn.schedule_at(sc, t)
        k = i % pool
        act = m.act(obs[k:k + 1], eps, t)
        m.replay_store(frames[k:k + 1], act, rew[k:k + 1], don[k:k + 1])
        if train:
            m.train_step(B, None, beta=beta, draw_seed=t, outputs=False)
            trains += i >= 0
        if sync:
            m.sync_target()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    m.close()
    return {"workload": "agent loop (Alg.1/Alg.2, Table 1 schedules): act on 1 observation + store 1 time step "
                        "per environment step, train batch %d fp32 every 4th step, synthetic emulator" % B,
            "value": env_steps / wall, "unit": "environment steps/s", "us_per_env_step": wall / env_steps * 1e6,
            "train_steps": trains}


def kernel_table(prof, B, R, n_params, precision, step_s=None):
    """Per kernel: live HIP-event average duration, the roofline that bounds it, what it achieves.
    An event pair around a kernel adds a fixed cost to what it measures (the events themselves are
    commands on the stream).  step_s, the duration of a step timed WITHOUT per-kernel events, gives
    that cost: the kernels of a step run back to back on one stream, so the event-timed durations
    exceed the step by (launches per step) x (cost per pair).  It is subtracted (`avg_us`; the raw
    event time stays in `avg_us_events`), so that the kernel times add up to the step."""
    fl = flops_per_launch(B, R)
    by = bytes_per_launch(B, n_params, precision == "bf16")
    gb = gemm_bytes_per_launch(B, R, precision == "bf16")
    out = {}
    overhead_s = 0.0
    if step_s is not None and prof:
        per_step = sum(tot_ms / cnt for cnt, tot_ms in prof.values()) / 1e3
        overhead_s = max(0.0, (per_step - step_s) / len(prof))
    for k, (cnt, tot_ms) in prof.items():
        raw_s = tot_ms / cnt / 1e3
        avg_s = max(raw_s - overhead_s, 0.25 * raw_s)
        if k in fl and k in gb and gb[k] / HBM_PEAK > fl[k] / PEAK[precision]:
            # a GEMM kernel whose operands take longer to stream at the HBM peak than its flops
            # take at the MFMA peak: HBM is the roof that binds
            e = {"bound": "hbm", "achieved": gb[k] / avg_s / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
        elif k in fl:
            e = {"bound": "mfma", "achieved": fl[k] / avg_s / 1e12, "peak": PEAK[precision] / 1e12, "unit": "TFLOP/s"}
        else:
            e = {"bound": "hbm", "achieved": by.get(k, 0) / avg_s / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
        e["frac"] = e["achieved"] / e["peak"]
        e["avg_us"] = round(avg_s * 1e6, 2)
        e["avg_us_events"] = round(raw_s * 1e6, 2)
        e["achieved"] = round(e["achieved"], 3)
        e["frac"] = round(e["frac"], 5)
        out[k] = e
    return dict(sorted(out.items(), key=lambda kv: -kv[1]["avg_us"]))


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


def time_replay_calls(m, torch, synth, capacity, reps=200):
    """The replay calls of the boundary on their own, over the same ring: microseconds per call and
    the algorithmic bytes they move against the HBM peak.  (Inside the training step the draws ride in
    the first forward kernel and the priority update in the backward launches; the tree walks are
    chains of dependent loads, so the time per call is the figure that matters.)"""
    out = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, n):
        for _ in range(10):
            fn(0)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    levels = max(1, (m.L - 1).bit_length())
    for B in (32, 512):
        t = timed(lambda i: m.per_sample(B, 0.4, 1000 + i), reps)
        out.append({"call": "per_sample", "batch": B, "us_per_call": t * 1e6, "algorithmic_bytes": B * levels * 4,
                    "achieved_GBps": B * levels * 4 / t / 1e9, "frac_of_hbm_peak": B * levels * 4 / t / HBM_PEAK})
        idx, _ = m.per_sample(B, 0.4, 7)
        td = synth.u24(5, torch.arange(B)).cuda()
        t = timed(lambda i: m.per_update(idx, td), reps)
        out.append({"call": "per_update", "batch": B, "us_per_call": t * 1e6, "algorithmic_bytes": B * levels * 12,
                    "achieved_GBps": B * levels * 12 / t / 1e9, "frac_of_hbm_peak": B * levels * 12 / t / HBM_PEAK})
        # rotate over distinct index sets so the frames are not cache-resident
        sets = [m.per_sample(B, 0.4, 50 + k)[0] for k in range(16)]
        from paper_1804_05834_amd import dqn as _d
        s = torch.empty(B, 4, 84, 84, dtype=torch.uint8, device="cuda")
        sn = torch.empty_like(s)
        a = torch.empty(B, dtype=torch.int32, device="cuda")
        r = torch.empty(B, device="cuda")
        d = torch.empty(B, dtype=torch.uint8, device="cuda")

        def gather(i):
            ix = sets[i % 16]
            m._check(_d.lib().dqn_replay_gather(m._h, _d._ptr(ix), B, _d._ptr(s), _d._ptr(sn), _d._ptr(a), _d._ptr(r),
                                                _d._ptr(d), _d._stream()))
        t = timed(gather, reps)
        nb = B * (5 * 7056 + 2 * 4 * 7056)     # five ring frames read, two four-frame stacks written
        out.append({"call": "dqn_replay_gather", "batch": B, "us_per_call": t * 1e6, "algorithmic_bytes": nb,
                    "achieved_GBps": nb / t / 1e9, "frac_of_hbm_peak": nb / t / HBM_PEAK})
    pri = synth.exp_priorities(9, capacity, "cuda")
    t = timed(lambda i: m.per_fill(pri), 20)
    nb = capacity * 4 + 2 * m.L * 4          # priorities read, every node of the tree written
    out.append({"call": "per_fill", "slots": capacity, "us_per_call": t * 1e6, "algorithmic_bytes": nb,
                "achieved_GBps": nb / t / 1e9, "frac_of_hbm_peak": nb / t / HBM_PEAK,
                "launches": 1 + (levels + 11) // 12})   # the leaves, then twelve tree levels per launch
    return {"workload": "the replay calls of the boundary on their own, %d-slot ring" % capacity, "calls": out}


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
        if el > 12.0 or reps >= 200:   # about 12 s of CPU work
            break
    per_step = el / reps * (B / sample_rows)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count()))
    sample = ("%d full oracle steps (fp64, explicit batch) on all %d rows" % (reps, B) if sample_rows == B else
              "%d full oracle steps (fp64, explicit batch) on %d of the %d rows, time scaled by %d/%d"
              % (reps, sample_rows, B, B, sample_rows))
    return {"value": 1.0 / per_step, "unit": "train steps/s", "cores": cores, "kind": "oracle", "sample": sample}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--batch", type=int, default=512)
    ap.add_argument("--precision", choices=["fp32", "bf16"], default="bf16")
    ap.add_argument("--capacity", type=int, default=1_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="skip the batch-32 fp32 and the act+train side measurements")
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
    wall, dev_s, enq_s = time_steps(m, torch, B, args.steps, args.warmup)
    ms_per_step = wall / args.steps * 1e3
    value = args.steps / wall

    prof = profile_kernels(m, torch, B, min(args.steps, 100), seed0=10_000_000)
    loss = check_health(m, torch, B)
    table = kernel_table(prof, B, R, m.n, args.precision, step_s=dev_s / args.steps)
    # the dominant kernel: the largest total time among the kernels of the step (the tree
    # kernels are listed in the table too; they are bound by dependent-load latency, not by a
    # throughput roofline; in the bf16 step per_update rides inside the backward launches)
    ranked = [k for k in sorted(table, key=lambda k: -table[k]["avg_us"]) if k not in ("per_update", "per_sample")]
    name = ranked[0]
    roof = {"kernel": name, "bound": table[name]["bound"], "achieved": table[name]["achieved"],
            "peak": table[name]["peak"], "unit": table[name]["unit"], "frac": table[name]["frac"],
            "traffic": MEASURED_TRAFFIC.get((name, B, args.precision)), "avg_us": table[name]["avg_us"]}

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
        "host_enqueue_ms_per_step": enq_s / args.steps * 1e3,
        "spin_up_steps": SPIN_UP_STEPS,
        "final_loss": loss,
        "roofline": roof,
        "kernels": table,
    }
    replay_calls = None if args.no_also else time_replay_calls(m, torch, synth, args.capacity)
    m.close()
    del m
    torch.cuda.empty_cache()

    if not args.no_also:
        also = [replay_calls]
        if not (B == 32 and prec == 0):
            m32 = build_model(dqn, synth, torch, 32, 0, args.capacity)
            w32, d32, _ = time_steps(m32, torch, 32, args.steps, args.warmup)
            also.append({"workload": "same step, batch 32, fp32", "value": args.steps / w32,
                         "unit": "train steps/s", "ms_per_step": w32 / args.steps * 1e3,
                         "device_ms_per_step": d32 / args.steps * 1e3,
                         "mfma_frac_step": step_flops(32, R) * args.steps / w32 / PEAK["fp32"]})
            m32.close()
            del m32
            torch.cuda.empty_cache()
        also.append(time_act_train(dqn, synth, torch, args.capacity, max(50, args.steps // 5), 10))
        also.append(time_agent_loop(dqn, synth, torch, args.capacity, max(200, 2 * args.steps)))
        also.append(time_variants(dqn, synth, torch, args.capacity, max(100, args.steps // 2), args.warmup))
        if not (B == 32 and prec == 1):
            m32 = build_model(dqn, synth, torch, 32, 1, args.capacity)
            w32, d32, _ = time_steps(m32, torch, 32, args.steps, args.warmup)
            also.append({"workload": "same step, batch 32, bf16", "value": args.steps / w32,
                         "unit": "train steps/s", "ms_per_step": w32 / args.steps * 1e3,
                         "device_ms_per_step": d32 / args.steps * 1e3,
                         "mfma_frac_step": step_flops(32, R) * args.steps / w32 / PEAK["bf16"]})
            m32.close()
            del m32
            torch.cuda.empty_cache()
        res["also"] = also
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(torch, synth, B, B)   # whole steps on all rows, about 12 s of CPU work
    print(json.dumps(res))


if __name__ == "__main__":
    main()
