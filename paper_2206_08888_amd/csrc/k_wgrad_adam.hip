// Weight gradients + Adam + Polyak as a launch of its own (wgrad.h has the work); extra
// blocks past the last network gather the replay rows of step t + 1 into the other half of
// the double-buffered batch (App. A of the paper: the next batches are fetched while the
// current update runs).
#include "gather.h"
#include "wgrad.h"

namespace pop {

// HALF: tiles of half the width, for populations whose full tiles would leave CUs with one or two of them.
template <bool HALF>
__global__ __launch_bounds__(kThreads, 3) void k_wgrad_adam(PopDev d, uint32_t t, int actor_phase, int main_blocks,
                                                          int roles, int prefetch) {
  __shared__ Adam sh_adam;
  __shared__ __attribute__((aligned(16))) float xt_lds[32 * kLda];
  POP_MARK(49);
  POP_BLOCK_TIME(actor_phase ? kTraceWgradActor : kTraceWgradCritic, 0);
  if ((int)blockIdx.x >= main_blocks) {              // gather role: rows of the next step
    if (prefetch) {
      const int g = blockIdx.x - main_blocks, per = gather_blocks_per_agent(d);
      gather_block(d, t + 1u, g / per, g % per, threadIdx.x);
    }
    POP_BLOCK_TIME(actor_phase ? kTraceWgradActor : kTraceWgradCritic, 1);
    return;
  }
  int unit, role;
  if (decode_block(blockIdx.x, actor_phase ? d.P : 2 * d.P, roles, unit, role))
    wgrad_roles<false, true, HALF>(d, t, actor_phase, unit, role, xt_lds, &sh_adam);
  POP_BLOCK_TIME(actor_phase ? kTraceWgradActor : kTraceWgradCritic, 1);
}

// Roles of one network: its 32 x 128 weight tiles, then the small tensors (wgrad.h): one role, and for an actor one
// more per kSmallHeadBlock head columns.
static int small_roles(const PopDev& d, int actor_phase) {
  return actor_phase ? 1 + (d.actor.out + kSmallHeadBlock - 1) / kSmallHeadBlock : 1;
}
int wgrad_role_count(const PopDev& d, int actor_phase) {
  const NetLayout& L = actor_phase ? d.actor : d.critic;
  return 16 + 2 * ((L.in + 31) / 32) + small_roles(d, actor_phase);
}

hipError_t launch_wgrad_adam(const PopDev& d, uint32_t t, int actor_phase, int prefetch_next, hipStream_t s) {
  const int full = wgrad_role_count(d, actor_phase), small = small_roles(d, actor_phase);
  const int roles = d.half_tiles ? 2 * (full - small) + small : full;   // every tile role twice; the small-tensor roles once
  const int main_blocks = xcd_grid(actor_phase ? d.P : 2 * d.P, roles);
  const int extra = prefetch_next ? d.P * gather_blocks_per_agent(d) : 0;
  const dim3 grid(main_blocks + extra), block(kThreads);
  if (d.half_tiles) k_wgrad_adam<true><<<grid, block, 0, s>>>(d, t, actor_phase, main_blocks, roles, prefetch_next);
  else k_wgrad_adam<false><<<grid, block, 0, s>>>(d, t, actor_phase, main_blocks, roles, prefetch_next);
  return hipGetLastError();
}

}  // namespace pop
