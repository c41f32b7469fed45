"""The comparison used by the GPU parity tests, tested on the CPU: a stand-in for the device (a second oracle
whose results are rounded to fp32) must pass, and planted mistakes -- a head bias that is never updated, a
hidden bias vector left alone, a stale target, a wrong column of the head -- must fail, including the ones that
the relative L2 norm of the whole network does not see."""
import copy
import types

import numpy as np
import pytest

import parity_checks as pc
import workloads
from gpu_common import STATE12, check_step_elementwise, check_tensors_all, snapshot
from oracle import td3


class Rounded:
    """Looks like the HIP population to the checkers: get_params returns fp32."""

    def __init__(self, orc, O, A):
        self.orc = orc
        self.cfg = types.SimpleNamespace(obs_dim=O, act_dim=A)
        self.patch = {}

    def get_params(self, agent, which):
        a = self.orc.get_params(agent, which).astype(np.float32)
        if (agent, which) in self.patch:
            a = self.patch[agent, which](a)
        return a


def _pair(steps_before=0):
    hps = workloads.hparams(0, 2)
    def make():
        p = td3.Population(hps, 17, 6, [256, 256], 256, 600)
        for i in range(2):
            p.insert(i, **workloads.transitions(0, i, 600))
        return p
    ref, dev = make(), make()
    ref.update(steps_before); dev.update(steps_before)
    return ref, dev


@pytest.mark.parametrize("steps_before", [0, 1, 4])
def test_a_correct_fp32_result_passes(steps_before):
    ref, dev = _pair(steps_before)
    before = snapshot(ref, [0, 1])
    ref.update(1); dev.update(1)
    rep = check_step_elementwise(Rounded(dev, 17, 6), ref, [(0, 0), (1, 1)], before, "cpu stand-in")
    assert rep.entries > (250_000 if steps_before == 1 else 400_000) and rep.worst_ratio < 0.05
    assert check_tensors_all(Rounded(dev, 17, 6), ref, [(0, 0), (1, 1)], STATE12[:6], 1e-4, "cpu stand-in") < 1e-6


def _slices(net):
    return dict(pc.tensor_slices(*pc.net_shape(net, 17, 6))[0])


PLANTS = {
    # name: (tensor code, tensor left at its old value (None: all of them), does the whole-network norm at 1e-4 miss it?)
    "critic head bias never updated": ("critic1", "b3", True),
    "actor head bias never updated": ("actor", "b3", True),
    "actor hidden bias vector never updated": ("actor", "b1", False),
    "critic second bias never updated": ("critic2", "b2", False),
    "critic-2 target left where it was": ("t_critic2", None, True),
}


@pytest.mark.parametrize("plant", sorted(PLANTS))
def test_planted_mistakes_fail_although_the_network_norm_hides_them(plant):
    which, tensor, hidden_from_the_norm = PLANTS[plant]
    ref, dev = _pair(0)
    before = snapshot(ref, [0, 1])
    ref.update(1); dev.update(1)
    fake = Rounded(dev, 17, 6)
    old = before[0, which].astype(np.float32)
    if tensor is None:
        fake.patch[0, which] = lambda a: old.copy()
    else:
        s = _slices(which)[tensor]
        def stale(a, s=s):
            a = a.copy(); a[s] = old[s]; return a
        fake.patch[0, which] = stale
    # the old criterion (one relative L2 norm per network at 1e-4) does not notice
    if hidden_from_the_norm:
        assert pc.rel_l2(fake.get_params(0, which), ref.get_params(0, which)) < 1e-4
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, plant)
    if tensor is not None:                                  # the per-tensor norm sees it as well
        with pytest.raises(AssertionError):
            check_tensors_all(fake, ref, [(0, 0)], [which], 1e-4, plant)


def test_wrong_head_column_and_wrong_moment_fail():
    ref, dev = _pair(2)
    before = snapshot(ref, [0, 1])
    ref.update(1); dev.update(1)
    fake = Rounded(dev, 17, 6)
    s = _slices("actor")["W3"]
    def wrong_column(a):
        a = a.copy(); w = a[s].reshape(256, 6); w[:, 4] += np.float32(3e-4) * np.sign(w[:, 4]); return a
    fake.patch[1, "actor"] = wrong_column
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "wrong head column")
    fake.patch.clear()
    sb = _slices("critic1")["b1"]
    def wrong_m(a):
        a = a.copy(); a[sb][7] *= np.float32(1.01); return a
    fake.patch[0, "m_critic1"] = wrong_m
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "wrong first moment")


def test_sign_of_an_undetermined_gradient_entry_may_differ_but_only_there():
    """First step: an entry whose gradient is below the rounding error of the fp32 path (ETA times the sum of the
    absolute values of its terms) may come out with the other sign (2 lr apart) and is masked; the same 2 lr on a
    well-determined entry fails."""
    ref, dev = _pair(0)
    before = snapshot(ref, [0, 1])
    ref.update(1); dev.update(1)
    import relu_ties as rt
    g = ref.get_params(0, "g_critic1")
    s = _slices("critic1")["W2"]
    scale = rt.CriticPass(ref.agents[0], rt.unflatten(before[0, "critic1"], 23, 1)).noise_scale()   # sum of |terms| per entry
    eta = 1e-4          # in this batch no entry is below the real ETA; the test widens it to have masked entries
    small = np.flatnonzero((np.abs(g[s]) < eta * scale[s]) & (g[s] != 0.0))
    big = np.flatnonzero(np.abs(g[s]) > 0.1 * scale[s])
    assert small.size and big.size
    lr = ref.agents[0].hp["lr_critic"]
    fake = Rounded(dev, 17, 6)
    def flip(at):
        def f(a):
            a = a.copy(); w = a[s]; w[at] += np.float32(2 * lr) * np.sign(g[s][at]).astype(np.float32); return a
        return f
    fake.patch[0, "critic1"] = flip(small[0])
    rep = check_step_elementwise(fake, ref, [(0, 0)], before, "masked entry", eta=eta)
    assert rep.masked >= small.size
    with pytest.raises(AssertionError):                      # at the real ETA the same entry is determined
        check_step_elementwise(fake, ref, [(0, 0)], before, "masked entry")
    fake.patch[0, "critic1"] = flip(big[0])
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0)], before, "determined entry", eta=eta)


def test_delayed_step_requires_bit_unchanged_actor_and_targets():
    ref, dev = _pair(1)                                      # step 1 is a critic-only step (delay 2)
    before = snapshot(ref, [0, 1])
    ref.update(1); dev.update(1)
    fake = Rounded(dev, 17, 6)
    check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "critic-only step")
    fake.patch[1, "t_critic1"] = lambda a: a * np.float32(1.0 + 1e-6)
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "target moved on a critic-only step")


def _plant_tie(pop, agent, unit, z):
    """Move bias `unit` of critic 1's first layer so that the unit's pre-activation on the first sampled row of
    step 0 is exactly z."""
    from oracle import philox
    ag = pop.agents[agent]
    idx = philox.sample_indices(ag.seed, 0, ag.B, ag.buffer.count)
    s, a = (x.astype(np.float64) for x in ag.buffer.gather(idx[:1])[:2])
    W, b = ag.critic[0][0]
    b[unit] = z - float(np.concatenate([s, a], axis=1)[0] @ W[:, unit])


def test_a_relu_resolved_the_other_way_is_accepted_only_as_such():
    """The oracle has one hidden unit of critic 1 at +1e-9, the stand-in for the device has it at -1e-9 (a bias that
    differs by 2e-9): the unit's mask differs, the critic-1 gradient by that sample's share, and the actor's step
    runs through a critic that moved differently.  With the tie allowance the step passes and names the flip;
    without it, or when the difference is not a tie, it fails."""
    ref, dev = _pair(0)
    _plant_tie(ref, 0, 11, +1e-9)
    _plant_tie(dev, 0, 11, -1e-9)
    before = snapshot(ref, [0, 1])
    ref.update(1); dev.update(1)
    fake = Rounded(dev, 17, 6)
    assert pc.rel_l2(fake.get_params(0, "g_critic1"), ref.get_params(0, "g_critic1")) > 1e-4
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "no allowance")
    ties = []
    rep = check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "tie allowance", ties=ties)
    assert len(ties) == 1 and ties[0][0] == 0 and ties[0][1] == "critic1"
    (rho, p, layer), = ties[0][2]
    assert rho < 1e-8 and layer == 0 and ties[0][4] < 1e-6
    assert rep.worst_ratio < 0.2
    # a gradient that is wrong in another way is not explained away
    s = _slices("critic1")["W2"]
    def wrong(a):
        a = a.copy(); a[s][::7] *= np.float32(1.01); return a
    fake.patch[0, "g_critic1"] = wrong
    with pytest.raises(AssertionError):
        check_step_elementwise(fake, ref, [(0, 0), (1, 1)], before, "not a tie", ties=[])


def test_explain_finds_planted_flips_in_the_actor_phase():
    import relu_ties as rt
    from oracle import mlp
    ref, _ = _pair(0)
    actor_before = mlp.copy_net(ref.agents[1].actor)
    ref.update(1)
    ag = ref.agents[1]
    clean = rt.ActorPass(ag, actor_before)
    assert pc.rel_l2(clean.gradient(), ref.get_params(1, "g_actor")) < 1e-12      # the pass is the oracle's computation
    cands = rt.candidates(clean.passes, np.inf, 3)
    dev = rt.ActorPass(ag, actor_before)
    for _, p, l, r, u in (cands[0], cands[2]):
        dev.flip(p, l, r, u)
    g_dev = dev.gradient()
    base, err, kept, rho0 = rt.explain(clean, g_dev, rho_max=np.inf, limit=8, goal=1e-9)
    assert base > 1e-6 and err < 1e-12 and len(kept) == 2      # (a row drawn twice gives two equivalent candidates)
