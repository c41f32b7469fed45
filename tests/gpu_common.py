"""Helpers for the GPU parity tests: build the HIP population and the oracle on
identical seeded inputs."""
import os

import numpy as np

import paper_2206_08888_amd as pp
import workloads
from oracle import td3 as oracle_td3

NETS = ("actor", "critic1", "critic2")


def ensure_built():
    if not os.path.exists(pp.lib_path()):
        from paper_2206_08888_amd import build
        build.build()
    return pp.load_library()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def make_pair(config_id=0, P=None, capacity=None, fill=None, batch=None, hps=None, agents=None, oracle=True,
              obs_dim=None, act_dim=None, **tuning):
    """HIP population + oracle population fed with the same hyperparameters and
    transitions.  `agents` selects which population members the oracle holds; `tuning`: launch structure, rows
    per workgroup and tile width (see paper_2206_08888_amd.make_config)."""
    cfgd = workloads.CONFIGS[config_id]
    P = cfgd["P"] if P is None else P
    capacity = cfgd["capacity"] if capacity is None else capacity
    fill = capacity if fill is None else fill
    batch = cfgd["batch"] if batch is None else batch
    O = cfgd["obs_dim"] if obs_dim is None else obs_dim
    A = cfgd["act_dim"] if act_dim is None else act_dim
    hps = workloads.hparams(config_id, P) if hps is None else hps
    cfg = pp.make_config(P, O, A, cfgd["hidden"], batch, capacity, **tuning)
    gpu = pp.Population(cfg, hps)
    agents = list(range(P)) if agents is None else list(agents)
    orc = None
    if oracle:
        orc = oracle_td3.Population([hps[i] for i in agents], O, A, list(cfgd["hidden"]), batch, capacity)
    custom = obs_dim is not None or act_dim is not None     # the config's stream drawn at the given shapes
    for i in range(P):
        chunks = [workloads.transitions(config_id, i, fill, obs_dim=O, act_dim=A, salt=1)] if custom else workloads.transition_chunks(config_id, i, fill)
        for tr in chunks:
            gpu.insert(i, **tr)
            if oracle and i in agents:
                orc.insert(agents.index(i), **tr)
    return gpu, orc, agents


def make_full_size_pair(config_id, verify_agents, **tuning):
    """HIP population of a config at its full size and an oracle population holding
    only `verify_agents`.  The verified agents get host-generated transitions
    (identical bytes on both sides); the other agents' buffers are filled on the
    device with the same distributions (torch generator, seeded) -- they only have
    to keep the GPU busy at the real shape, nothing is compared on them."""
    import torch
    cfgd = workloads.CONFIGS[config_id]
    P, O, A, cap, B = cfgd["P"], cfgd["obs_dim"], cfgd["act_dim"], cfgd["capacity"], cfgd["batch"]
    hps = workloads.hparams(config_id)
    cfg = pp.make_config(P, O, A, cfgd["hidden"], B, cap, **tuning)
    gpu = pp.Population(cfg, hps)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(workloads.DATA_SEED + 77 * config_id)
    piece = max(1, min(cap, (48 << 20) // (P * (2 * O + A + 2))))
    done = 0
    while done < cap:
        n = min(piece, cap - done)
        gpu.insert(-1, obs=torch.randn((P, n, O), generator=gen, device="cuda"),
                   act=torch.rand((P, n, A), generator=gen, device="cuda") * 2 - 1,
                   rew=torch.randn((P, n), generator=gen, device="cuda"),
                   done=(torch.rand((P, n), generator=gen, device="cuda") < 0.01).float(),
                   next_obs=torch.randn((P, n, O), generator=gen, device="cuda"))
        done += n
    orc = oracle_td3.Population([hps[i] for i in verify_agents], O, A, list(cfgd["hidden"]), B, cap)
    for j, i in enumerate(verify_agents):          # a full ring of host rows overwrites the device-made ones
        for tr in workloads.transition_chunks(config_id, i, cap):
            gpu.insert(i, **tr)
            orc.insert(j, **tr)
    return gpu, orc


PARAMS6 = ("actor", "critic1", "critic2", "t_actor", "t_critic1", "t_critic2")
MOM_M = ("m_actor", "m_critic1", "m_critic2")
MOM_V = ("v_actor", "v_critic1", "v_critic2")
STATE12 = PARAMS6 + MOM_M + MOM_V


def force_state(gpu, orc, pairs):
    """Set the GPU agents to the oracle agents' current state; pairs = [(gpu_agent, oracle_agent)]."""
    for i, j in pairs:
        for which in STATE12:
            gpu.set_params(i, which, orc.get_params(j, which))


# ------------------------------------------------------------------------------------------------------------
# Element-wise / per-tensor comparisons (tests/parity_checks.py holds the arithmetic and its derivation)
import parity_checks as pc

KIND_NETS = {"td3": ("actor", "critic1", "critic2"), "sac": ("actor", "critic1", "critic2"),
             "shared": ("actor", "critic1", "critic2")}


def _kind_of(orc):
    name = type(orc).__module__.rsplit(".", 1)[-1]
    return {"td3": "td3", "sac": "sac", "td3_shared": "shared"}[name]


def snapshot(orc, oracle_agents):
    """The oracle's parameters, targets and moments of the given agents (flat fp64 copies), keyed (agent, name)."""
    kind = _kind_of(orc)
    names = [n for n in STATE12 if not (kind == "sac" and n == "t_actor")]
    return {(j, n): orc.get_params(j, n).copy() for j in oracle_agents for n in names}


def _adam_info(orc, kind, j, net):
    """(lr, b1, b2, eps, Adam count of the update just taken, tau, updated?, targets moved?) of one network."""
    ag = orc.agents[j]
    hp = orc.agents[0].hp if (kind == "shared" and net != "actor") else ag.hp
    lr = hp["lr_actor"] if net == "actor" else hp["lr_critic"]
    if kind == "sac":
        return lr, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"], ag.t, (None if net == "actor" else hp["tau"]), True, net != "actor"
    actor_step = ag.last.get("actor_grads") is not None
    if net == "actor":
        return lr, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"], ag.actor_updates, hp["tau"], actor_step, actor_step
    if kind == "shared":
        moved = (orc.t - 1) % int(hp["policy_delay"]) == 0
    else:
        moved = actor_step
    return lr, hp["adam_b1"], hp["adam_b2"], hp["adam_eps"], ag.t, hp["tau"], True, moved


def check_step_elementwise(gpu, orc, pairs, before, label, grads=True, ties=None, eta=pc.ETA, tol=pc.TOL, report=None):
    """After ONE step that both sides took from the common state `before` (snapshot() of the oracle taken before
    the step; the GPU agents held the same values rounded to fp32): every network of every (gpu_agent,
    oracle_agent) pair tensor by tensor and element by element (parity_checks.check_adam_step), networks
    without an update in this step bit-unchanged.  grads: the GPU recorded its gradients (set_debug).

    ties: a list, or None.  With a list, a network whose device gradient differs from the oracle's by more than
    1e-5 (relative L2) must be the oracle's gradient with hidden units on their kink resolved the other way
    (relu_ties.explain: relative margin below relu_ties.RHO_TIE, gradient reproduced to 1e-5); the network is then
    compared, as strictly as any other, with the oracle's own Adam and Polyak applied to that gradient, networks
    downstream of it in the same step (the actor behind critic 1) with the oracle's pass through the flipped
    result; (gpu_agent, network, flips) is appended to the list.  With None such a step fails."""
    import relu_ties as rt
    kind = _kind_of(orc)
    O, A = gpu.cfg.obs_dim, gpu.cfg.act_dim
    sac = kind == "sac"
    rep = pc.StepReport() if report is None else report
    flipped = {}                                          # critic index -> flipped critic (list form) after its update
    for i, j in pairs:
        ag = orc.agents[j]
        if kind != "shared":
            flipped = {}
        for net in ("critic1", "critic2", "actor"):
            if kind == "shared" and net != "actor" and (i, j) != tuple(pairs[0]):
                continue                                  # the one critic pair is compared once
            lr, b1, b2, eps, count, tau, updated, moved = _adam_info(orc, kind, j, net)
            has_target = not (sac and net == "actor")
            shape = pc.net_shape(net, O, A, sac)
            got = {"theta": gpu.get_params(i, net), "m": gpu.get_params(i, "m_" + net), "v": gpu.get_params(i, "v_" + net)}
            bef = {"theta": before[j, net], "m": before[j, "m_" + net], "v": before[j, "v_" + net]}
            if has_target:
                got["target"] = gpu.get_params(i, "t_" + net)
                bef["target"] = before[j, "t_" + net]
            tag = "%s, agent %d" % (label, i)
            if not updated:
                pc.check_unchanged(tag, net, got, bef)
                continue
            ref = {"theta": orc.get_params(j, net), "m": orc.get_params(j, "m_" + net), "v": orc.get_params(j, "v_" + net),
                   "g": orc.get_params(j, "g_" + net)}
            if has_target:
                ref["target"] = orc.get_params(j, "t_" + net)
            if grads:
                got["g"] = gpu.get_params(i, "g_" + net)
            if has_target and not moved:
                pc.check_unchanged(tag, "t_" + net, {"target": got["target"]}, {"target": bef["target"]})
            tau_used = tau if (has_target and moved) else None
            # the oracle's pass for this network: scale of the gradient's rounding error, and the masks open to flips
            n_before = rt.unflatten(bef["theta"], *shape)
            if net != "actor":
                ps = rt.SharedCriticPass(orc.agents, n_before) if kind == "shared" else rt.CriticPass(ag, n_before)
            elif sac:
                ps = rt.SacActorPass(ag, n_before, [flipped.get(k, ag.critic[k]) for k in range(2)])
            else:
                ps = rt.ActorPass(ag, n_before, flipped.get(0))
            kept = []
            if ties is not None and grads:
                if net == "actor" and flipped:            # the actor's loss runs through a critic that took a flipped step
                    ref = rt.redo_adam(bef, ps.gradient(), shape, lr, b1, b2, eps, count, tau_used)
                ge = rel_l2(got["g"], ref["g"])
                if ge > 1e-5:
                    base, err, kept, rho0 = rt.explain(ps, got["g"])
                    assert kept and err <= 1e-5, ("%s: %s gradient differs by %.3e (rel-L2) and flipping the hidden units nearest "
                                                  "their kink (smallest relative margin %.2e) leaves %.3e" % (tag, net, base, rho0, err))
                    ref = rt.redo_adam(bef, ps.gradient(), shape, lr, b1, b2, eps, count, tau_used)
                    ties.append((i, net, [(c[0], c[1], c[2]) for c in kept], base, err))
                    if net != "actor":
                        flipped[int(net[-1]) - 1] = rt.unflatten(ref["theta"], *shape)
            env, n_env = (rt.tie_envelope(ps, skip=kept) if ties is not None else (None, 0))
            rep.tie_units += n_env
            # (the shared critics' gradient is a sum over P batches in agent groups: twice the single-batch bound)
            pc.check_adam_step(rep, tag, net, shape, got, ref, bef, lr, b1, b2, eps, count, tau=tau_used, tol=tol,
                               eta=2.0 * eta if (kind == "shared" and net != "actor") else eta,
                               g_scale=ps.noise_scale(), g_extra=env)
    return rep


def check_tensors_all(gpu, orc, pairs, names, tol, label, steps=0):
    """Per-tensor relative L2 (see parity_checks.check_tensors) of the named flat networks; returns the worst
    per-network relative L2 for the report.  steps > 0: the comparison follows that many free-running steps, and
    up to 8 entries per tensor whose first Adam update took the other sign may be 2 lr per step apart."""
    kind = _kind_of(orc)
    O, A = gpu.cfg.obs_dim, gpu.cfg.act_dim
    worst, left_out = 0.0, 0
    for i, j in pairs:
        lr = max(orc.agents[j].hp["lr_actor"], orc.agents[j].hp["lr_critic"], orc.agents[0].hp["lr_critic"])
        for n in names:
            got, ref = gpu.get_params(i, n), orc.get_params(j, n)
            _, k = pc.check_tensors(got, ref, n, O, A, tol, "%s, agent %d" % (label, i), sac=(kind == "sac"),
                                    outliers=8 if steps else 0, outlier_bound=2.02 * lr * max(steps, 1))
            left_out += k
            worst = max(worst, rel_l2(got, ref))
    if left_out:
        print("%s: %d entries left out of the per-tensor norms (first Adam update with the other sign)" % (label, left_out))
    return worst


def free_run_tie_aware(gpu, orc, pairs, steps, label, each_step=None, tight=1e-5):
    """Free run of `steps` steps, one at a time on both sides (TD3 oracle; the GPU records its gradients).

    As long as an agent's two trajectories have met no ReLU tie they must agree tightly: every gradient to `tight`
    (relative L2 per network) and every parameter tensor to `tight` after every step.  The first step at which a
    gradient differs by more must be a tie: the device's gradient is reproduced (to `tight`) by the oracle's with
    hidden units of relative margin < relu_ties.RHO_TIE resolved the other way.  From there the two are different,
    equally valid trajectories and only the caller's final bound applies.
    Returns {gpu_agent: dict(departed=(step, network, flips) or None, error=worst per-network rel-L2 at the end)}."""
    import relu_ties as rt
    assert _kind_of(orc) == "td3"
    O, A = gpu.cfg.obs_dim, gpu.cfg.act_dim
    gpu.set_debug(1)
    departed = {i: None for i, _ in pairs}
    for t in range(steps):
        live = [(i, j) for i, j in pairs if departed[i] is None]
        pre = {j: {n: orc.get_params(j, n) for n in NETS} for _, j in live}
        gpu.update(1); orc.update(1)
        if each_step is not None:
            each_step(t)
        for i, j in live:
            ag = orc.agents[j]
            for net in ("critic1", "critic2", "actor"):
                if net == "actor" and ag.last["actor_grads"] is None:
                    continue
                g = gpu.get_params(i, "g_" + net)
                ge = rel_l2(g, orc.get_params(j, "g_" + net))
                if ge <= tight:
                    continue
                shape = pc.net_shape(net, O, A)
                n_before = rt.unflatten(pre[j][net], *shape)
                ps = rt.ActorPass(ag, n_before) if net == "actor" else rt.CriticPass(ag, n_before)
                base, err, kept, rho0 = rt.explain(ps, g, goal=tight)
                assert kept and err <= tight, (
                    "%s: step %d, agent %d: %s gradient differs by %.3e (rel-L2) and flipping the hidden units nearest their "
                    "kink (smallest relative margin %.2e) leaves %.3e" % (label, t, i, net, base, rho0, err))
                departed[i] = (t, net, [(c[0], c[1], c[2]) for c in kept])
                break
            if departed[i] is None:
                check_tensors_all(gpu, orc, [(i, j)], PARAMS6, tight, "%s: step %d (no tie met so far)" % (label, t), steps=t + 1)
    out = {}
    for i, j in pairs:
        e = max(rel_l2(gpu.get_params(i, n), orc.get_params(j, n)) for n in PARAMS6)
        out[i] = dict(departed=departed[i], error=e)
    gpu.set_debug(0)
    return out


def describe_free_run(res):
    errs = sorted(r["error"] for r in res.values())
    parts = []
    for i, r in sorted(res.items()):
        if r["departed"] is None:
            parts.append("agent %d: no tie, %.2e" % (i, r["error"]))
        else:
            t, net, flips = r["departed"]
            parts.append("agent %d: %s tie at step %d (relative margin %.1e), %.2e at the end" % (i, net, t, flips[0][0], r["error"]))
    return "median %.2e, worst %.2e over %d agents; %s" % (errs[len(errs) // 2], errs[-1], len(errs), "; ".join(parts))
