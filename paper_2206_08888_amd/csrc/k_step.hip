// One update step of the whole population as a single launch (Sec. 4.1 of the paper: the
// update steps of all population members are issued together and chained on the device).
//
// (with_chains = 0: the target and critic chains ran as a launch of their own and only the
// rest of the step is here.)  Blocks, in index order:
//   target chains | critic chains | critic weight-gradient tiles | actor chains |
//   actor weight-gradient tiles | gather of the next step's replay rows
// Each part depends on the one before it only per agent or per network, never globally:
// a critic chunk needs the Bellman targets of its own rows, a weight-gradient tile the 8
// chunks of its own network, an actor chunk the updated critic 1 of its own agent.  Those
// hand-overs happen inside the launch (tagged words and release/acquire counters, see
// chains.h), so nothing waits for the slowest workgroup of a whole phase, memory-bound
// Adam tiles run beside matrix-bound chains of other agents, and work that has no
// dependency yet (the critics' forward pass, the actor's forward pass, the Adam operand
// loads) starts at once.  Workgroups are dispatched in block order, so a workgroup only
// ever waits for workgroups that were dispatched before it.
#include "gather.h"
#include "wgrad.h"

namespace pop {

#ifdef POP_TRACE
int g_trace_step_parts[6];           // blocks of the parts of the last k_step launch: target, critic, critic tiles, actor, actor tiles, gather
#endif

struct StepGrid {
  int t, c, wc, a, wa, g;          // blocks of each part (0: the part is not in this launch)
  int roles_c, roles_a;            // weight-gradient roles per critic / actor network
};

// GT, GC, GA: tile geometries of the target, critic and actor chains.
template <class GT, class GC, class GA>
__global__ __launch_bounds__(kThreads, 2) void k_step(PopDev d, uint32_t t, StepGrid g) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  int b = blockIdx.x;
  POP_MARK(63);
  POP_BLOCK_TIME(kTraceStep, 0);
  if (b == 0) {                                      // zero the counters the next step will count in
                                                     // (whichever part block 0 belongs to)
    const int other = d.sync_half ^ 1;
    for (int i = threadIdx.x; i < 2 * d.P; i += kThreads) {
      d.done_c[other * 2 * d.P + i] = 0u;
      d.done_wc[other * 2 * d.P + i] = 0u;
      if (i < d.P) d.done_a[other * d.P + i] = 0u;
    }
  }
  int unit, sub;
  if (b < g.t) {
    if (decode_block(b, d.P, d.B / GT::R, unit, sub)) target_chain<GT>(d, t, unit, sub, lds);
    POP_BLOCK_TIME(kTraceStep, 1);
    return;
  }
  b -= g.t;
  if (b < g.c) {
    if (decode_block(b, 2 * d.P, d.B / GC::R, unit, sub)) critic_chain<GC, true, true>(d, t, unit, sub, lds);
    POP_BLOCK_TIME(kTraceStep, 1);
    return;
  }
  b -= g.c;
  Adam* sh_adam = reinterpret_cast<Adam*>(lds + 32 * kLda);
  if (GA::R == 16 && b < g.wc + g.a) {
    // Small populations (the 16-row class), measured 97.6 against 99.2 us/step at P = 10 (and 448 against 439 at
    // P = 80, hence not there): per agent the tiles of its two critics, then its actor chains; an actor chain
    // still finds what it waits for -- the tiles of its own critic 1 -- at lower block indices.  With one
    // workgroup per CU the actor chains of the first agents then start while later agents' tiles still run.
    const int tiles = 2 * g.roles_c, chunks = g.a / d.P;
    if (decode_block<true>(b, d.P, tiles + chunks, unit, sub)) {    // an agent's actor chains wait for its own tiles
      if (sub < tiles) wgrad_roles<true>(d, t, 0, 2 * unit + sub / g.roles_c, sub % g.roles_c, lds, sh_adam, g.c != 0);
      else actor_chain<GA, true>(d, t, unit, sub - tiles, lds, g.roles_c);
    }
    POP_BLOCK_TIME(kTraceStep, 1);
    return;
  }
  if (b < g.wc) {
    if (decode_block(b, 2 * d.P, g.roles_c, unit, sub)) wgrad_roles<true>(d, t, 0, unit, sub, lds, sh_adam, g.c != 0);
    POP_BLOCK_TIME(kTraceStep, 1);
    return;
  }
  b -= g.wc;
  if (b < g.a) {
    if (decode_block(b, d.P, d.B / GA::R, unit, sub)) actor_chain<GA, true>(d, t, unit, sub, lds, g.roles_c);
    POP_BLOCK_TIME(kTraceStep, 1);
    return;
  }
  b -= g.a;
  if (b < g.wa) {
    if (decode_block(b, d.P, g.roles_a, unit, sub)) wgrad_roles<true>(d, t, 1, unit, sub, lds, sh_adam);
    POP_BLOCK_TIME(kTraceStep, 1);
    return;
  }
  b -= g.wa;
  if (b < g.g) {
    const int per = gather_blocks_per_agent(d);
    gather_block(d, t + 1u, b / per, b % per, threadIdx.x);
  }
}

#define POP_STEP_SMALL k_step<Rows16, Rows32<2>, Rows16>
#define POP_STEP_MID k_step<Rows32<1, true>, Rows32<1, true>, Rows32<1, true>>
#define POP_STEP_LARGE k_step<Rows32<2>, Rows32<2>, Rows32<2>>

hipError_t setup_step_kernel() {
  hipError_t e;
  if ((e = hipFuncSetAttribute((const void*)POP_STEP_SMALL, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute((const void*)POP_STEP_MID, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)) != hipSuccess) return e;
  return hipFuncSetAttribute((const void*)POP_STEP_LARGE, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

hipError_t launch_step(const PopDev& dev, uint32_t t, uint32_t launch_seq, int with_chains, int with_actor,
                       int prefetch_next, hipStream_t s) {
  PopDev d = dev;
  const bool small = d.rows_t == 16 && d.rows_c == 64 && d.rows_a == 16;
  if (!small && !(d.rows_t == d.rows_c && d.rows_c == d.rows_a && (d.rows_a == 32 || d.rows_a == 64)))
    return hipErrorInvalidValue;                     // the kernel exists for these three row classes only
  d.sync_half = (int)(launch_seq & 1u);              // the previous launch of this kernel cleared this half
  StepGrid g;
  g.roles_c = wgrad_role_count(d, 0);
  g.roles_a = wgrad_role_count(d, 1);
  g.t = with_chains ? xcd_grid(d.P, d.B / d.rows_t) : 0;       // else: target and critic chains ran in an earlier launch
  g.c = with_chains ? xcd_grid(2 * d.P, d.B / d.rows_c) : 0;
  g.wc = xcd_grid(2 * d.P, g.roles_c);
  g.a = with_actor ? xcd_grid(d.P, d.B / d.rows_a) : 0;
  g.wa = with_actor ? xcd_grid(d.P, g.roles_a) : 0;
  g.g = prefetch_next ? d.P * gather_blocks_per_agent(d) : 0;
  const int vec_ta = vec_target(d) > vec_actor(d) ? vec_target(d) : vec_actor(d);
  const int vec = vec_ta > vec_critic(d) ? vec_ta : vec_critic(d);
  const size_t tiles = (size_t)(32 * kLda) * sizeof(float) + sizeof(Adam);
  const dim3 grid(g.t + g.c + g.wc + g.a + g.wa + g.g), block(kThreads);
#ifdef POP_TRACE
  g_trace_step_parts[0] = g.t; g_trace_step_parts[1] = g.c; g_trace_step_parts[2] = g.wc; g_trace_step_parts[3] = g.a;
  g_trace_step_parts[4] = g.wa; g_trace_step_parts[5] = g.g;
#endif
  size_t bytes = tiles;
  auto need = [&](size_t b) { if (b > bytes) bytes = b; };
  if (d.rows_a == 16) {
    need(LdsMap<16, 16>(d.D).bytes(vec_ta) + kStage16 * sizeof(float));   // with the weight stage of the 16-row actor chain
    need(Lds<2>(d.D).bytes(vec_critic(d)));
    // One workgroup per CU for small populations: the request is kept above half of a CU's LDS (the 64-row
    // critic chain alone needs 80,928 of the 81,920 bytes that would let two share).  With two per CU the actor
    // chains start earlier but every chain then shares its matrix pipe: 118 against 100 us/step at P = 10.
    need((size_t)kLdsPerCU / 2 + 64);
    POP_STEP_SMALL<<<grid, block, bytes, s>>>(d, t, g);
  } else if (d.rows_a == 32) {
    need(Lds<1>(d.D).bytes(vec));
    POP_STEP_MID<<<grid, block, bytes, s>>>(d, t, g);
  } else {
    need(Lds<2>(d.D).bytes(vec));
    POP_STEP_LARGE<<<grid, block, bytes, s>>>(d, t, g);
  }
  return hipGetLastError();
}

}  // namespace pop
