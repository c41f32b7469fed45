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
              obs_dim=None, act_dim=None):
    """HIP population + oracle population fed with the same hyperparameters and
    transitions.  `agents` selects which population members the oracle holds."""
    cfgd = workloads.CONFIGS[config_id]
    P = cfgd["P"] if P is None else P
    capacity = cfgd["capacity"] if capacity is None else capacity
    fill = capacity if fill is None else fill
    batch = cfgd["batch"] if batch is None else batch
    O = cfgd["obs_dim"] if obs_dim is None else obs_dim
    A = cfgd["act_dim"] if act_dim is None else act_dim
    hps = workloads.hparams(config_id, P) if hps is None else hps
    cfg = pp.make_config(P, O, A, cfgd["hidden"], batch, capacity)
    gpu = pp.Population(cfg, hps)
    agents = list(range(P)) if agents is None else list(agents)
    orc = None
    if oracle:
        orc = oracle_td3.Population([hps[i] for i in agents], O, A, list(cfgd["hidden"]), batch, capacity)
    for i in range(P):
        for tr in workloads.transition_chunks(config_id, i, fill):
            if obs_dim is not None or act_dim is not None:
                raise NotImplementedError
            gpu.insert(i, **tr)
            if oracle and i in agents:
                orc.insert(agents.index(i), **tr)
    return gpu, orc, agents


def make_full_size_pair(config_id, verify_agents):
    """HIP population of a config at its full size and an oracle population holding
    only `verify_agents`.  The verified agents get host-generated transitions
    (identical bytes on both sides); the other agents' buffers are filled on the
    device with the same distributions (torch generator, seeded) -- they only have
    to keep the GPU busy at the real shape, nothing is compared on them."""
    import torch
    cfgd = workloads.CONFIGS[config_id]
    P, O, A, cap, B = cfgd["P"], cfgd["obs_dim"], cfgd["act_dim"], cfgd["capacity"], cfgd["batch"]
    hps = workloads.hparams(config_id)
    cfg = pp.make_config(P, O, A, cfgd["hidden"], B, cap)
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


def forced_step_errors(gpu, orc, pairs):
    """After one step from a common state: worst rel-L2 of (parameters and targets, second
    moments, first moments) over the given agents."""
    def worst(names):
        w = 0.0
        for i, j in pairs:
            for which in names:
                ref = orc.get_params(j, which)
                if ref.any():
                    w = max(w, rel_l2(gpu.get_params(i, which), ref))
        return w
    return worst(PARAMS6), worst(MOM_V), worst(MOM_M)


class ForcedStepStats:
    """Tolerances of a forced single step (GPU started from the oracle's state):
      parameters and targets  <= 1e-4 always (the one-step tolerance);
      second moments          <= 1e-3 always;
      first moments           <= 1e-4, except on steps where a ReLU pre-activation lies
                              within fp32 rounding error of zero and the two sides resolve
                              it differently: one (sample, unit) then enters or leaves the
                              gradient, which moves m by up to a few 1e-3 relative while
                              the parameters move by < 1e-5.  Such steps must stay rare
                              (<= 10 % of the steps) and bounded (<= 5e-2)."""

    def __init__(self):
        self.steps = 0
        self.flips = 0
        self.worst_p = self.worst_v = self.worst_m = 0.0

    def add(self, ep, ev, em, tag):
        self.steps += 1
        self.worst_p, self.worst_v, self.worst_m = max(self.worst_p, ep), max(self.worst_v, ev), max(self.worst_m, em)
        assert ep <= 1e-4, (tag, "parameters", ep)
        assert ev <= 1e-3, (tag, "second moments", ev)
        assert em <= 5e-2, (tag, "first moments", em)
        if em > 1e-4:
            self.flips += 1

    def finish(self):
        assert self.flips <= max(1, self.steps // 10), (self.flips, self.steps)
        return ("%d forced steps: parameters %.2e, v %.2e, m %.2e worst rel-L2; %d step(s) with a ReLU tie resolved "
                "differently" % (self.steps, self.worst_p, self.worst_v, self.worst_m, self.flips))
