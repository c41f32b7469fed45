"""CPU oracle for the population TD3 (td3.py), SAC (sac.py) and shared-critic TD3 (td3_shared.py) update steps.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, fp64 definition of
what the HIP path computes: every agent of the population is stepped on its
own, one after another, with hand-derived backprop.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product path
never does.  It shares no code with the HIP library.

Paper passages followed (Flajolet et al., "Fast Population-Based Reinforcement
Learning on a Single Machine"):
  * Sec. 4.1 "Training Independent Replicas of the Same Agent": N replicas,
    different initial weights and hyperparameters, updated independently; MLP
    actor and critics; TD3 and SAC with the standard hyperparametrization.
  * Sec. 4.2 "Training Agents Sharing Parameters": one critic pair for the
    whole population, every batch through the policy networks in parallel,
    the critic loss averaged over the population (td3_shared.py).
  * App. C: a population layer is y[p] = x[p] W[p] + b[p] with W of shape
    [P, in, out] and b of shape [P, 1, out].
  * App. A: one bounded first-in-first-out replay buffer per agent, batches of
    all agents stacked on a new leading axis.
The paper does not print the TD3 or SAC equations (it cites Fujimoto et al. 2018
and Haarnoja et al. 2018);
the reading taken for every point it leaves open is listed in the design notes
of the repository and restated in the docstrings below.

Pin status: every function is pinned by tests that do not retype its formula
(finite differences, torch.autograd in float64, torch.optim.Adam, closed
forms, brute force).  The one exception is the bit pattern of the counter RNG
stream (philox.py): no known-answer vectors are available offline, so it is
pinned by structure and statistics only -- "parity unpinned" for conformance
to the published Philox test vectors; the contract is only that both sides
draw the same words.
"""
