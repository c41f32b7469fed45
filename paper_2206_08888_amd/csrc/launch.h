// Host-side launch wrappers implemented in the kernel source files.
#pragma once
#include <hip/hip_runtime.h>
#include "pop_dev.h"

namespace pop {

// parameter initialisation: Glorot-uniform weights of the three online networks
// of every agent, copied into the targets; limits are computed by the host.
struct InitLimits { float actor[3], critic[3]; };
hipError_t launch_init(const PopDev& d, const InitLimits& lim, hipStream_t s);

// replay ring: write n rows per agent starting at cursor (agent < 0: all agents,
// sources carry a leading population axis), then advance cursor and count.
hipError_t launch_insert(const PopDev& d, int agent, int64_t n, const float* obs, const float* act,
                         const float* rew, const float* done, const float* next_obs, hipStream_t s);

// one update step
hipError_t launch_sample_gather(const PopDev& d, uint32_t t, hipStream_t s);
hipError_t launch_target(const PopDev& d, uint32_t t, hipStream_t s);
hipError_t launch_critic(const PopDev& d, uint32_t t, hipStream_t s);
hipError_t launch_target_critic(const PopDev& d, uint32_t t, hipStream_t s);   // both of the above in one launch
hipError_t launch_actor(const PopDev& d, uint32_t t, hipStream_t s);
// prefetch_next != 0: extra workgroups also gather the replay rows of step t + 1
hipError_t launch_wgrad_adam(const PopDev& d, uint32_t t, int actor_phase, int prefetch_next, hipStream_t s);

// shared critics: partial gradient sums per agent group, then Adam on the one critic pair (k_wgrad_shared.hip)
hipError_t launch_wgrad_shared(const PopDev& d, uint32_t t, int prefetch_next, hipStream_t s);

// SAC: target chain (online actor, soft clipped double-Q target) and actor chain (k_sac.hip); the critic chain
// and the weight-gradient launches are shared with TD3
hipError_t launch_sac_target(const PopDev& d, uint32_t t, hipStream_t s);
hipError_t launch_sac_actor(const PopDev& d, uint32_t t, hipStream_t s);
hipError_t launch_sac_target_critic(const PopDev& d, uint32_t t, hipStream_t s);   // target + critic chains in one launch
hipError_t setup_sac_kernels();
size_t td3_lds_bytes(const PopDev& d);   // the same for the TD3 step's chains
size_t sac_lds_bytes(const PopDev& d);   // largest dynamic LDS request of the SAC step's and the acting kernels

// the step as one launch (k_step.hip); with_chains = 0: without the target and critic chains (launched
// before); with_actor: some agent has its delayed actor step at t; launch_seq: 0, 1, 2, ... over the
// launches of this kernel on this population (alternates the two sets of hand-over counters)
hipError_t launch_step(const PopDev& d, uint32_t t, uint32_t launch_seq, int with_chains, int with_actor,
                       int prefetch_next, hipStream_t s);
hipError_t setup_step_kernel();
int wgrad_role_count(const PopDev& d, int actor_phase);

// acting: obs[P][n][O] -> act[P][n][A] through the online actors; sigma (device, [P]) != nullptr adds
// exploration noise drawn at counter `step`, rows numbered from row_base
hipError_t launch_act(const PopDev& d, const float* obs, int n, float* act, const float* sigma, uint32_t step,
                      uint32_t row_base, hipStream_t s);

// one-time per-process kernel attribute setup (large dynamic LDS)
hipError_t setup_kernels();

}  // namespace pop
