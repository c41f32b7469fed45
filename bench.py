#!/usr/bin/env python3
"""Throughput of the population TD3 update step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..6] [--no-cpu] [--no-secondary]

A "step" is one update step of the whole population (every kernel of the hot
path: replay sample + gather, target chain, critic chain, critic weight
gradients + Adam, and on delayed steps the actor chain and actor weight
gradients + Adam + Polyak).  The replay buffers are filled with seeded
synthetic transitions and are resident in HBM before the timed region starts
(the paper's protocol, Sec. 4.1: batches already in accelerator memory, data
loading excluded, parameters not returned to the host between steps).

Prints ONE JSON line: agent-updates/s = P * steps / seconds.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

import workloads

MFMA_FP32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
H = 256


def kernel_flops(P, B, O, A, algo="td3"):
    """Algorithmic FLOPs of one launch of each kernel (2 per multiply-add), whole population."""
    D = O + A
    if algo == "sac":
        return sac_kernel_flops(P, B, O, A)
    fwd_actor = 2 * B * (O * H + H * H + H * A)
    fwd_critic = 2 * B * (D * H + H * H + H)
    per_agent = {
        "gather": 0,
        "target": fwd_actor + 2 * fwd_critic,
        "critic": 2 * (fwd_critic + 2 * B * H * H + 2 * B * H),
        "wgrad_critic": 2 * (2 * B * H * H + 2 * B * D * H),
        "actor": fwd_actor + 2 * B * (D * H + H * H) + 2 * B * H * H + 3 * (2 * B * A * H) + 2 * B * H * H,
        "wgrad_actor": 2 * B * H * H + 2 * B * O * H,
    }
    per_agent["target_critic"] = per_agent["target"] + per_agent["critic"]
    # the whole step as one launch: average over launches with and without the delayed actor part (delay 2)
    per_agent["step_tail"] = per_agent["wgrad_critic"] + per_agent["actor"] + per_agent["wgrad_actor"]
    per_agent["step"] = (per_agent["target_critic"] + per_agent["wgrad_critic"]
                         + (per_agent["actor"] + per_agent["wgrad_actor"]) / 2)
    return {k: v * P for k, v in per_agent.items()}


def sac_kernel_flops(P, B, O, A):
    """SAC: the actor head has 2A outputs, the actor step runs both critics forward and backward."""
    D = O + A
    fwd_actor = 2 * B * (O * H + H * H + H * 2 * A)
    fwd_critic = 2 * B * (D * H + H * H + H)
    critic_to_action = 2 * B * H + 2 * B * H * H + 2 * B * A * H          # dz2, dz1, da
    per_agent = {
        "gather": 0,
        "target": fwd_actor + 2 * fwd_critic,
        "critic": 2 * (fwd_critic + 2 * B * H * H + 2 * B * H),
        "wgrad_critic": 2 * (2 * B * H * H + 2 * B * D * H),
        "actor": fwd_actor + 2 * fwd_critic + 2 * critic_to_action + 2 * (2 * B * 2 * A * H) + 2 * B * H * H,
        "wgrad_actor": 2 * B * H * H + 2 * B * O * H,
    }
    per_agent["target_critic"] = per_agent["target"] + per_agent["critic"]
    for k in ("step", "step_tail"):
        per_agent[k] = 0
    return {k: v * P for k, v in per_agent.items()}


def step_flops_per_agent(B, O, A, delay=2, algo="td3"):
    f = kernel_flops(1, B, O, A, algo)
    if algo == "sac":
        delay = 1
    return f["target"] + f["critic"] + f["wgrad_critic"] + (f["actor"] + f["wgrad_actor"]) / delay


def build_population(config_id, torch, fill=None):
    import paper_2206_08888_amd as pp
    c = workloads.CONFIGS[config_id]
    P, O, A, cap = c["P"], c["obs_dim"], c["act_dim"], c["capacity"]
    algo = {"sac": pp.POP_ALGO_SAC, "td3": pp.POP_ALGO_TD3, "td3_shared": pp.POP_ALGO_TD3_SHARED}[c["algo"]]
    cfg = pp.make_config(P, O, A, c["hidden"], c["batch"], cap, algo=algo)
    pop = pp.Population(cfg, workloads.hparams(config_id))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(workloads.DATA_SEED + config_id)
    fill = cap if fill is None else fill
    piece = max(1, min(fill, (64 << 20) // max(1, P * (2 * O + A + 2))))
    done_rows = 0
    while done_rows < fill:
        n = min(piece, fill - done_rows)
        tr = dict(
            obs=torch.randn((P, n, O), generator=gen, device="cuda"),
            act=torch.rand((P, n, A), generator=gen, device="cuda") * 2 - 1,
            rew=torch.randn((P, n), generator=gen, device="cuda"),
            done=(torch.rand((P, n), generator=gen, device="cuda") < 0.01).float(),
            next_obs=torch.randn((P, n, O), generator=gen, device="cuda"),
        )
        pop.insert(-1, **tr)
        done_rows += n
    pop.sync()
    return pop, c


def time_config(config_id, steps, warmup, torch, with_kernels=True):
    pop, c = build_population(config_id, torch)
    P = c["P"]
    pop.update(warmup)
    pop.sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pop.update(steps)
    pop.sync()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out = dict(P=P, seconds=dt, ms_per_step=1e3 * dt / steps, value=P * steps / dt)
    if with_kernels:
        ms, cnt = pop.update_timed(steps)
        out["kernel_us"] = {k: (1e3 * ms[k] / cnt[k] if cnt[k] else None) for k in ms}
        out["kernel_launches"] = cnt
    pop.close()
    return out, c


def cpu_baseline(config_id, budget_s=12.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import sac, td3, td3_shared
    c = workloads.CONFIGS[config_id]
    n_agents, rows = 2, 50_000
    hps = workloads.hparams(config_id)[:n_agents]
    orc = {"sac": sac, "td3": td3, "td3_shared": td3_shared}[c["algo"]].Population(hps, c["obs_dim"], c["act_dim"], list(c["hidden"]), c["batch"], rows)
    for i in range(n_agents):
        orc.insert(i, **workloads.transitions(config_id, i, rows))
    orc.update(1)
    t0 = time.perf_counter()
    steps = 0
    while time.perf_counter() - t0 < budget_s and steps < 2000:
        orc.update(10)
        steps += 10
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return dict(value=n_agents * steps / dt, unit="agent-updates/s", cores=int(cores), kind="oracle",
                sample="agents 0-%d of the workload, %d-row buffers, %d steps each (numpy fp64, BLAS threads)"
                       % (n_agents - 1, rows, steps))


def read_traffic(kernel, P):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    key = "%s P=%d bytes_per_launch" % (kernel, P)
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line.split("=")[-1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=1, choices=(0, 1, 2, 3, 4, 5, 6))
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-secondary", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: populations shard by agent with no traffic inside the step, "
              "and this build runs on a single MI355X; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2206_08888_amd as pp
    pp.load_library()                       # fails loudly when the HIP library is missing

    if args.calibrate_copy:                 # known traffic: 1 GiB read + 1 GiB written per copy
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    res, c = time_config(args.config, args.steps, args.warmup, torch)
    P, B, O, A = c["P"], c["batch"], c["obs_dim"], c["act_dim"]
    flops = kernel_flops(P, B, O, A, c["algo"])
    kus = res["kernel_us"]
    per_step_us = {k: (kus[k] or 0.0) * res["kernel_launches"][k] / args.steps for k in kus}
    dominant = max((k for k in kus if flops[k] > 0 and kus[k]), key=lambda k: per_step_us[k])
    achieved = flops[dominant] / (kus[dominant] * 1e-6) / 1e12
    roofline = dict(bound="mfma", kernel=dominant, achieved=achieved, peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=achieved / MFMA_FP32_PEAK_TFLOPS, traffic=read_traffic(dominant, P),
                    avg_launch_us=kus[dominant], flops_per_launch=flops[dominant])
    step_frac = res["value"] * step_flops_per_agent(B, O, A, algo=c["algo"]) / (MFMA_FP32_PEAK_TFLOPS * 1e12)
    line = {
        "metric": "agent-updates/sec (P x SGD steps/s), %s population" % c["algo"].upper(),
        "value": res["value"], "unit": "agent-updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s population P=%d, obs %d, act %d, MLP 256x256, batch %d, "
                               "%d-row replay buffer per agent, per-agent hyperparameters"
                               % (args.config, c["algo"].upper(), P, O, A, B, c["capacity"]),
                   "P": P, "batch": B, "obs_dim": O, "act_dim": A, "capacity": c["capacity"]},
        "roofline": roofline,
        "step_frac_of_fp32_mfma_peak": step_frac,
        "kernel_avg_us": kus,
        "kernel_us_per_step": per_step_us,
    }
    if not args.no_secondary and args.config == 1:
        sec, c2 = time_config(2, args.steps, args.warmup, torch, with_kernels=True)
        line["p80"] = {"workload": "config 2: TD3 population P=80 hyperparameter sweep",
                       "value": sec["value"], "unit": "agent-updates/s", "ms_per_step": sec["ms_per_step"],
                       "step_frac_of_fp32_mfma_peak": sec["value"] * step_flops_per_agent(
                           c2["batch"], c2["obs_dim"], c2["act_dim"]) / (MFMA_FP32_PEAK_TFLOPS * 1e12),
                       "kernel_avg_us": sec["kernel_us"]}
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.config)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
