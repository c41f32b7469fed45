#!/usr/bin/env python3
"""Throughput of the population TD3 update step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..6] [--repeats R] [--no-cpu] [--no-secondary]
    python bench.py --sweep [--steps K]        # config 4: saturation of the chip as P grows 1 -> 256

A "step" is one update step of the whole population (every kernel of the hot
path: replay sample + gather, target chain, critic chain, critic weight
gradients + Adam, and on delayed steps the actor chain and actor weight
gradients + Adam + Polyak).  The replay buffers are filled with seeded
synthetic transitions and are resident in HBM before the timed region starts
(the paper's protocol, Sec. 4.1: batches already in accelerator memory, data
loading excluded, parameters not returned to the host between steps).

Timing: max(W, 20) untimed warm-up steps, then R (default 5) repeats of exactly K steps, each repeat one
pop_update(K) call bracketed by a synchronisation on both sides; the line reports the MEDIAN repeat.

Prints ONE JSON line: agent-updates/s = P * K / seconds, with
  roofline      the dominant kernel against the fp32 MFMA peak (launch time from HIP events on the library's stream);
  hbm           achieved GB/s of the memory-bound parts (replay gather, weight-gradient tiles with Adam / Polyak)
                against the 8 TB/s HBM peak: algorithmic bytes / launch time;
  counters      what rocprofv3 counter runs recorded for the same kernels (profiles/*.txt: HBM bytes per launch,
                MFMA busy share), with a flag telling whether the kernel sources have changed since;
  cpu_baseline  the CPU oracle on the machine's host cores, one process per agent, one BLAS thread each.
"""
import argparse
import hashlib
import json
import os
import statistics
import sys
import time

import numpy as np

import workloads

MFMA_FP32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
HBM_PEAK_GBPS = 8000.0             # MI355X HBM3E
H = 256
ROOT = os.path.dirname(os.path.abspath(__file__))


def kernel_flops(P, B, O, A, algo="td3", actor_ahead=False):
    """Algorithmic FLOPs of one launch of each kernel (2 per multiply-add), whole population.  actor_ahead: the
    actor's forward pass runs inside the target / critic launch on steps with a policy update (every second one)."""
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
    if actor_ahead:
        per_agent["target_critic"] += fwd_actor / 2
        per_agent["actor"] -= fwd_actor
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


def kernel_bytes(P, B, O, A, algo="td3", delay=2):
    """Algorithmic HBM bytes of one launch of the memory-bound parts, whole population.

    gather: B rows of (2 O + A + 2) floats read from the replay buffer and written to the batch (+ 4 B per index).
    wgrad_critic: both critics' parameters, first and second moments read and written (24 B per parameter), on
      delayed steps also their targets (8 B per parameter; averaged over the delay), the three activation tensors
      of each critic ([B, 256] floats: h1, dz2, dz1) and the batch rows read.
    wgrad_actor: the same for the actor, whose launch always carries Polyak (32 B per parameter), with its
      activations h1, h2, dz2, dz1 (h2 only as far as the head's weight gradient needs it).
    The shared critics keep ONE critic pair: their Adam traffic does not grow with P.
    The chain launches, for the ratio of measured to necessary traffic (they are bound by the matrix units, not by
    HBM): every network a chain runs read once (4 B per parameter), its columns of the batch rows read, and what
    it leaves for the weight-gradient tiles written (target: y; critic: h1, dz2, dz1 of both critics; actor: h1, h2,
    dz2, dz1 and the head's gradient).  target_critic and step are the sums of the parts one launch carries (step:
    averaged over steps with and without the actor part)."""
    D, out_a = O + A, (2 * A if algo == "sac" else A)
    row = 2 * O + A + 2
    n_actor = O * H + H + H * H + H + H * out_a + out_a
    n_critic = D * H + H + H * H + H + H + 1
    polyak = 1.0 if algo == "sac" else 1.0 / delay
    act_critic = 2 * 3 * B * H * 4 + B * row * 4
    crit_state = 2 * n_critic * (24 + 8 * polyak)
    shared = algo == "td3_shared"
    nets_target = 0 if shared else 2 * n_critic             # critics beside the actor in each chain, per agent
    nets_critic = 0 if shared else 2 * n_critic
    nets_actor = 0 if shared else (2 if algo == "sac" else 1) * n_critic
    per = {
        "gather": 2 * B * row * 4 + B * 4,
        "wgrad_critic": act_critic + crit_state,
        "wgrad_actor": 4 * B * H * 4 + B * row * 4 + n_actor * (24 + (0 if algo == "sac" else 8)),
        "target": 4 * (n_actor + nets_target) + B * (O + 2) * 4 + B * 4,
        "critic": 4 * nets_critic + B * (D + 1) * 4 + 2 * 3 * B * H * 4,
        "actor": 4 * (n_actor + nets_actor) + B * O * 4 + 4 * B * H * 4 + B * out_a * 4,
    }
    out = {k: v * P for k, v in per.items()}
    if shared:                                              # one critic pair and its targets, read once per launch
        out["wgrad_critic"] = act_critic * P + crit_state
        out["target"] += 4 * 2 * n_critic
        out["critic"] += 4 * 2 * n_critic
        out["actor"] += 4 * n_critic
    out["target_critic"] = out["target"] + out["critic"]
    out["step"] = out["target_critic"] + out["wgrad_critic"] + (out["actor"] + out["wgrad_actor"]) / delay + out["gather"]
    return out


def sources_sha():
    """Fingerprint of the kernel sources, to tell whether committed counter summaries still describe them."""
    h = hashlib.sha1()
    d = os.path.join(ROOT, "paper_2206_08888_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h")):
            h.update(f.encode()); h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def read_counters(config_id):
    """Machine-readable lines of the committed rocprofv3 counter summaries: 'config=<id> kernel=<name> key=value ...'
    (profiles/hbm_traffic.txt, profiles/mfma_utilisation.txt) -> {kernel: {key: value}}, and whether they were
    recorded on the kernel sources as they are now."""
    out, shas = {}, set()
    for name in ("hbm_traffic.txt", "mfma_utilisation.txt"):
        try:
            lines = open(os.path.join(ROOT, "profiles", name)).read().splitlines()
        except OSError:
            continue
        for line in lines:
            if line.startswith("kernel_sources_sha="):
                shas.add(line.split("=", 1)[1].strip())
            if not line.startswith("config=%d " % config_id):
                continue
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            k = kv.pop("kernel")
            out.setdefault(k, {}).update({a: float(b) for a, b in kv.items()})
    return out, (shas == {sources_sha()} if shas else None)


def build_population(config_id, torch, P=None, **tuning):
    import paper_2206_08888_amd as pp
    c = dict(workloads.CONFIGS[config_id])
    if P is not None:
        c["P"] = P
    P, O, A, cap = c["P"], c["obs_dim"], c["act_dim"], c["capacity"]
    algo = {"sac": pp.POP_ALGO_SAC, "td3": pp.POP_ALGO_TD3, "td3_shared": pp.POP_ALGO_TD3_SHARED}[c["algo"]]
    cfg = pp.make_config(P, O, A, c["hidden"], c["batch"], cap, algo=algo, **tuning)
    pop = pp.Population(cfg, workloads.hparams(config_id, P))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(workloads.DATA_SEED + config_id)
    piece = max(1, min(cap, (64 << 20) // max(1, P * (2 * O + A + 2))))
    done_rows = 0
    while done_rows < cap:
        n = min(piece, cap - done_rows)
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


def time_steps(pop, steps, warmup, repeats, torch):
    """Seconds of each of `repeats` pop_update(steps) calls, after max(warmup, 20) untimed steps -- and as many more
    as it takes to fill 100 ms, so that a short run is timed at the clocks a long one settles at."""
    pop.update(max(warmup, 20))
    pop.sync()
    t_end = time.perf_counter() + 0.1
    while time.perf_counter() < t_end:
        pop.update(20)
        pop.sync()
    out = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pop.update(steps)
        pop.sync()
        torch.cuda.synchronize()
        out.append(time.perf_counter() - t0)
    return out


def time_gather(pop, torch, calls=24):
    """Average duration (us) of the stand-alone replay gather: a one-row insert makes the rows gathered ahead
    stale, so the next update has to draw and gather its batch in a launch of its own."""
    P, c = pop.cfg.P, pop.cfg
    one = dict(obs=torch.zeros((P, 1, c.obs_dim), device="cuda"), act=torch.zeros((P, 1, c.act_dim), device="cuda"),
               rew=torch.zeros((P, 1), device="cuda"), done=torch.zeros((P, 1), device="cuda"),
               next_obs=torch.zeros((P, 1, c.obs_dim), device="cuda"))
    total, n = 0.0, 0
    for i in range(calls):
        pop.insert(-1, **one)
        ms, cnt = pop.update_timed(1)
        if i >= 4 and cnt["gather"]:
            total += ms["gather"]; n += cnt["gather"]
    return 1e3 * total / n if n else None


def time_config(config_id, steps, warmup, repeats, torch, with_kernels=True, P=None, **tuning):
    pop, c = build_population(config_id, torch, P=P, **tuning)
    P = c["P"]
    secs = time_steps(pop, steps, warmup, repeats, torch)
    dt = statistics.median(secs)
    out = dict(P=P, seconds=dt, ms_per_step=1e3 * dt / steps, value=P * steps / dt,
               repeat_ms_per_step=[1e3 * s / steps for s in secs], tuning=pop.tuning())
    if with_kernels:
        n = max(steps, 100)
        ms, cnt = pop.update_timed(n)
        out["kernel_us"] = {k: (1e3 * ms[k] / cnt[k] if cnt[k] else None) for k in ms}
        out["kernel_launches_per_step"] = {k: cnt[k] / n for k in cnt}
        out["kernel_us"]["gather"] = time_gather(pop, torch)
    pop.close()
    return out, c


# ---------------------------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, one process per agent, one BLAS thread each (the paper's own CPU reference
# is one core per agent, Sec. 4.1).  Runs before anything touches the GPU: the worker processes are started from a
# process that holds no device.

CPU_MAX_BUFFER_FLOATS = 64 << 20      # rows of a worker's buffer are capped so that it stays within 256 MB


def _cpu_rows(c):
    return min(c["capacity"], CPU_MAX_BUFFER_FLOATS // (2 * c["obs_dim"] + c["act_dim"] + 2))


def _cpu_worker(args):
    config_id, agents, budget_s = args
    from threadpoolctl import threadpool_limits
    from oracle import sac, td3, td3_shared
    c = workloads.CONFIGS[config_id]
    rows = _cpu_rows(c)
    with threadpool_limits(limits=1):
        mod = {"sac": sac, "td3": td3, "td3_shared": td3_shared}[c["algo"]]
        hps = [workloads.hparams(config_id)[a] for a in agents]
        orc = mod.Population(hps, c["obs_dim"], c["act_dim"], list(c["hidden"]), c["batch"], rows)
        for j, a in enumerate(agents):
            for tr in workloads.transition_chunks(config_id, a, rows):
                orc.insert(j, **tr)
        orc.update(1)                                     # warm-up step
        t0 = time.perf_counter()
        steps = 0
        while steps < 3 or time.perf_counter() - t0 < budget_s:
            orc.update(1)
            steps += 1
        return steps * len(agents), time.perf_counter() - t0


def cpu_baseline(config_id, budget_s=12.0):
    import multiprocessing as mp
    c = workloads.CONFIGS[config_id]
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))     # the machine's CPU share
    except ValueError:
        pass
    n = max(1, min(c["P"], cores))
    if c["algo"] == "td3_shared":       # the step couples the agents through the one critic pair: one process steps a
        jobs = [(config_id, list(range(min(c["P"], 4))), budget_s)]           # population of four
    else:
        jobs = [(config_id, [i], budget_s) for i in range(n)]
    saved = {k: os.environ.get(k) for k in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS")}
    for k in saved:
        os.environ[k] = "1"
    try:
        with mp.get_context("spawn").Pool(len(jobs)) as pool:
            res = pool.map(_cpu_worker, jobs)
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
    value = sum(u / t for u, t in res)
    rows = _cpu_rows(c)
    return dict(value=value, unit="agent-updates/s", cores=len(jobs), kind="oracle",
                sample="%s, one process and one BLAS thread each, %d-row buffers%s, %d agent-updates in %.0f s after one warm-up "
                       "step each (numpy fp64)"
                       % ("agents 0-%d of the workload" % (len(jobs) - 1) if c["algo"] != "td3_shared"
                          else "a shared-critic population of the workload's first %d agents" % len(jobs[0][1]),
                          rows, "" if rows == c["capacity"] else " (the workload's: %d)" % c["capacity"],
                          sum(u for u, _ in res), max(t for _, t in res)))


def analyse(res, c, steps, config_id):
    P, B, O, A = c["P"], c["batch"], c["obs_dim"], c["act_dim"]
    flops = kernel_flops(P, B, O, A, c["algo"], actor_ahead=res["tuning"]["actor_ahead"] == 2)
    nbytes = kernel_bytes(P, B, O, A, c["algo"])
    kus, per = res["kernel_us"], res["kernel_launches_per_step"]
    per_step_us = {k: (kus[k] or 0.0) * per[k] for k in kus}
    dominant = max((k for k in kus if flops[k] > 0 and kus[k]), key=lambda k: per_step_us[k])
    achieved = flops[dominant] / (kus[dominant] * 1e-6) / 1e12
    counters, fresh = read_counters(config_id)
    roofline = dict(bound="mfma", kernel=dominant, achieved=achieved, peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=achieved / MFMA_FP32_PEAK_TFLOPS, traffic=counters.get(dominant, {}).get("hbm_bytes_per_launch"),
                    avg_launch_us=kus[dominant], flops_per_launch=flops[dominant])
    hbm = {}
    for k in ("gather", "wgrad_critic", "wgrad_actor"):
        if kus.get(k):
            gbps = nbytes[k] / (kus[k] * 1e-6) / 1e9
            hbm[k] = dict(algorithmic_bytes_per_launch=nbytes[k], avg_launch_us=kus[k], gbps=gbps, frac_of_hbm_peak=gbps / HBM_PEAK_GBPS,
                          measured_bytes_per_launch=counters.get(k, {}).get("hbm_bytes_per_launch"))
    if kus.get("step"):                                     # the parts run inside one launch: the launch as a whole
        tot = nbytes["wgrad_critic"] + nbytes["wgrad_actor"] / 2 + nbytes["gather"]
        gbps = (counters.get("step", {}).get("hbm_bytes_per_launch") or tot) / (kus["step"] * 1e-6) / 1e9
        hbm["step"] = dict(algorithmic_bytes_per_launch_of_its_memory_bound_parts=tot, algorithmic_bytes_per_launch=nbytes["step"],
                           avg_launch_us=kus["step"],
                           measured_bytes_per_launch=counters.get("step", {}).get("hbm_bytes_per_launch"),
                           gbps=gbps, frac_of_hbm_peak=gbps / HBM_PEAK_GBPS)
    step_frac = res["value"] * step_flops_per_agent(B, O, A, algo=c["algo"]) / (MFMA_FP32_PEAK_TFLOPS * 1e12)
    return dict(roofline=roofline, hbm=hbm, step_frac=step_frac, per_step_us=per_step_us,
                counters=dict(per_kernel=counters, recorded_on_current_kernel_sources=fresh,
                              source="profiles/hbm_traffic.txt, profiles/mfma_utilisation.txt (rocprofv3 --pmc runs of this file)"))


def sweep(args, torch):
    """Config 4: the same shapes, buffers (50,000 rows) and hyperparameter draws at P = 1 .. 256."""
    c = workloads.CONFIGS[4]
    rows = []
    for P in (1, 2, 4, 8, 10, 16, 32, 64, 80, 128, 192, 256):
        res, _ = time_config(4, args.steps, args.warmup, max(3, args.repeats), torch, with_kernels=False, P=P)
        frac = res["value"] * step_flops_per_agent(c["batch"], c["obs_dim"], c["act_dim"]) / (MFMA_FP32_PEAK_TFLOPS * 1e12)
        rows.append(dict(P=P, value=res["value"], us_per_step=1e3 * res["ms_per_step"], us_per_agent_update=1e6 / res["value"],
                         step_frac_of_fp32_mfma_peak=frac))
        print("P = %3d: %9.0f agent-updates/s, %8.1f us/step, %.3f of the fp32 MFMA step ceiling" % (P, res["value"], 1e3 * res["ms_per_step"], frac),
              file=sys.stderr, flush=True)
    full = rows[-1]
    print(json.dumps({
        "metric": "agent-updates/sec (P x SGD steps/s), TD3 population, saturation sweep", "value": full["value"],
        "unit": "agent-updates/s", "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 20),
        "ms_per_step": full["us_per_step"] / 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config 4: TD3 population P = 1 .. 256, obs 17, act 6, MLP 256x256, batch 256, 50000-row replay "
                               "buffer per agent, per-agent lr, tau and policy noise (value: P = 256)"},
        "repeats": max(3, args.repeats), "sweep": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--repeats", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, choices=(0, 1, 2, 3, 4, 5, 6))
    ap.add_argument("--sweep", action="store_true", help="config 4: P = 1 .. 256")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-secondary", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 200 if args.sweep else 1000
    if args.gpus != 1:
        print("bench.py measures one GPU: populations shard by agent with no traffic inside the step, "
              "and this build runs on a single MI355X; --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.repeats < 1:
        print("--steps and --repeats must be positive", file=sys.stderr)
        sys.exit(2)
    cpu = None
    if not args.no_cpu and not args.sweep:                  # first: its worker processes start before the GPU is in use
        cpu = cpu_baseline(args.config)
    import torch
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2206_08888_amd as pp
    pp.load_library()                       # fails loudly when the HIP library is missing

    if args.sweep:
        sweep(args, torch)
        return
    if args.calibrate_copy:                 # known traffic: 1 GiB read + 1 GiB written per copy
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    res, c = time_config(args.config, args.steps, args.warmup, args.repeats, torch)
    P, B, O, A = c["P"], c["batch"], c["obs_dim"], c["act_dim"]
    an = analyse(res, c, args.steps, args.config)
    line = {
        "metric": "agent-updates/sec (P x SGD steps/s), %s population" % c["algo"].upper(),
        "value": res["value"], "unit": "agent-updates/s", "n_gpus": 1, "steps": args.steps, "warmup": max(args.warmup, 20),
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s population P=%d, obs %d, act %d, MLP 256x256, batch %d, "
                               "%d-row replay buffer per agent, per-agent hyperparameters"
                               % (args.config, c["algo"].upper(), P, O, A, B, c["capacity"]),
                   "P": P, "batch": B, "obs_dim": O, "act_dim": A, "capacity": c["capacity"]},
        "repeats": args.repeats, "repeat_ms_per_step": res["repeat_ms_per_step"],
        "roofline": an["roofline"],
        "step_frac_of_fp32_mfma_peak": an["step_frac"],
        "hbm": an["hbm"],
        "counters": an["counters"],
        "tuning_in_force": res["tuning"],
        "kernel_avg_us": res["kernel_us"],
        "kernel_us_per_step": an["per_step_us"],
    }
    if not args.no_secondary and args.config == 1:
        sec, c2 = time_config(2, args.steps, args.warmup, args.repeats, torch, with_kernels=True)
        an2 = analyse(sec, c2, args.steps, 2)
        line["p80"] = {"workload": "config 2: TD3 population P=80 hyperparameter sweep",
                       "value": sec["value"], "unit": "agent-updates/s", "ms_per_step": sec["ms_per_step"],
                       "repeat_ms_per_step": sec["repeat_ms_per_step"],
                       "step_frac_of_fp32_mfma_peak": an2["step_frac"], "roofline": an2["roofline"], "hbm": an2["hbm"],
                       "counters": an2["counters"], "tuning_in_force": sec["tuning"], "kernel_avg_us": sec["kernel_us"]}
    if cpu is not None:
        line["cpu_baseline"] = cpu
    print(json.dumps(line))


if __name__ == "__main__":
    main()
