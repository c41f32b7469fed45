"""pop_act_explore_noalloc, the entry point for callers that cannot allocate: through the C boundary against
pop_act_explore (same kernels, so the results must be equal bit for bit), on two calls in a row, the second on a
smaller population with fewer rows -- both use the one static scratch array of the GPU, which keeps the first
call's contents."""
import numpy as np
import pytest
import torch

import paper_2206_08888_amd as pp
import workloads
from gpu_common import ensure_built

pytestmark = pytest.mark.gpu


def _population(P, seed_config):
    cfg = pp.make_config(P, 17, 6, (256, 256), 256, 600)
    pop = pp.Population(cfg, workloads.hparams(seed_config, P))
    for i in range(P):
        pop.insert(i, **workloads.transitions(seed_config, i, 600))
    pop.update(2)                                        # actors that differ from their initial state
    return pop


def test_noalloc_entry_point_equals_pop_act_explore_on_two_calls_in_a_row():
    ensure_built()
    big, small = _population(6, 2), _population(3, 1)
    rng = np.random.default_rng(11)
    calls = [(big, 70, [0.3, 0.0, 0.1, 0.25, 0.2, 0.05], 7),
             (small, 20, [0.15, 0.4, 0.0], 123456)]         # second call: smaller population, fewer rows
    outs = []
    for pop, n, sigma, step in calls:                       # both calls back to back, nothing in between
        obs = torch.from_numpy(rng.standard_normal((pop.cfg.P, n, 17)).astype(np.float32)).cuda()
        out = torch.full((pop.cfg.P, n, 6), float("nan"), dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        pp.pop_act_explore_noalloc(pop.ctx, obs, n, out, sigma, step)
        assert torch.cuda.memory_allocated() == before
        outs.append((pop, obs, n, sigma, step, out))
    for pop, obs, n, sigma, step, out in outs:
        pop.sync()
        want = pop.act(obs, sigma=sigma, step=step)         # pop_act_explore, device pointers
        assert torch.equal(out, want), float((out - want).abs().max())
        assert torch.equal(out[[i for i, s in enumerate(sigma) if s == 0.0]],
                           pop.act(obs)[[i for i, s in enumerate(sigma) if s == 0.0]])   # sigma 0: the noiseless path
        assert bool(torch.all(out.abs() <= 1.0))
    # a call with n = 0 is a no-op; bad arguments are refused before anything is launched
    pp.pop_act_explore_noalloc(big.ctx, outs[0][1], 0, outs[0][5], outs[0][3], 0)
    with pytest.raises(pp.PopError) as e:
        pp.pop_act_explore_noalloc(big.ctx, outs[0][1], 70, outs[0][5], [0.1, -1.0, 0.1, 0.1, 0.1, 0.1], 0)
    assert e.value.code == pp.POP_EINVAL
    big.close(); small.close()


def test_noalloc_entry_point_refuses_populations_beyond_its_scratch():
    ensure_built()
    P = 257
    cfg = pp.make_config(P, 17, 6, (256, 256), 256, 256)
    pop = pp.Population(cfg, workloads.hparams(4, P))
    obs = torch.zeros((P, 1, 17), device="cuda"); out = torch.zeros((P, 1, 6), device="cuda")
    with pytest.raises(pp.PopError) as e:
        pp.pop_act_explore_noalloc(pop.ctx, obs, 1, out, [0.1] * P, 0)
    assert e.value.code == pp.POP_EUNSUPPORTED and "256" in str(e.value)
    pop.act(obs, sigma=[0.1] * P, step=0)                   # the allocating-free limit does not bind pop_act_explore
    pop.close()
