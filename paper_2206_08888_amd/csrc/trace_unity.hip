// Traced build of the library: every source as ONE translation unit with the timeline instrumentation of
// pop_dev.h compiled in (the instrumented kernels write to __device__ arrays defined here, which separate
// translation units could not share without relocatable device code).  Built as libpop_trace.so by
// `python -m paper_2206_08888_amd.build --trace`; same C boundary as libpop.so plus the trace_* calls below.
// Not for timing runs of the product: the marks cost a few clock reads per block.
#define POP_TRACE 1
#include <hip/hip_runtime.h>
#include "pop_dev.h"

__device__ unsigned long long g_pop_trace[64];
__device__ int g_pop_trace_block = 0;
__device__ unsigned long long g_pop_block_time[kTraceKinds][2][kTraceBlocks];

#include "k_replay.hip"
#include "k_init.hip"
#include "k_chain.hip"
#include "k_wgrad_adam.hip"
#include "k_step.hip"
#include "k_sac.hip"
#include "k_wgrad_shared.hip"
#include "pop_api.hip"

extern "C" {

// Number of kernel kinds and of blocks per kind the block-time array holds.
int pop_trace_dims(int32_t* kinds, int32_t* blocks) {
  if (kinds) *kinds = kTraceKinds;
  if (blocks) *blocks = kTraceBlocks;
  return POP_OK;
}

// Zero the block times and the phase marks (synchronises the device).
int pop_trace_reset(void) {
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_pop_block_time)) != hipSuccess) return POP_EHIP;
  if (hipMemset(p, 0, sizeof(unsigned long long) * kTraceKinds * 2 * kTraceBlocks) != hipSuccess) return POP_EHIP;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_pop_trace)) != hipSuccess) return POP_EHIP;
  if (hipMemset(p, 0, sizeof(unsigned long long) * 64) != hipSuccess) return POP_EHIP;
  return hipDeviceSynchronize() == hipSuccess ? POP_OK : POP_EHIP;
}

// Copy the block times out: out[kind][0 = start, 1 = end][block], ticks of the 100 MHz constant-rate clock
// (0 = that block did not run since the last reset).  Synchronises the device.
int pop_trace_block_times(uint64_t* out) {
  if (!out) return POP_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return POP_EHIP;
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_pop_block_time), sizeof(unsigned long long) * kTraceKinds * 2 * kTraceBlocks) == hipSuccess
             ? POP_OK : POP_EHIP;
}

// Choose the block whose phase marks are recorded, and read the 64 marks back.
int pop_trace_select_block(int32_t block) {
  return hipMemcpyToSymbol(HIP_SYMBOL(g_pop_trace_block), &block, sizeof block) == hipSuccess ? POP_OK : POP_EHIP;
}
int pop_trace_marks(uint64_t* out) {
  if (!out) return POP_EINVAL;
  if (hipDeviceSynchronize() != hipSuccess) return POP_EHIP;
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_pop_trace), sizeof(unsigned long long) * 64) == hipSuccess ? POP_OK : POP_EHIP;
}

// Blocks of the parts of the last single-launch step: target, critic, critic tiles, actor, actor tiles, gather.
int pop_trace_step_parts(int32_t* out) {
  if (!out) return POP_EINVAL;
  for (int i = 0; i < 6; ++i) out[i] = pop::g_trace_step_parts[i];
  return POP_OK;
}

}  // extern "C"
