// Kernels around the SAC chains of chains_sac.h (one launch per chain; the critic chain and
// the weight-gradient tiles are the TD3 ones).
#include <algorithm>
#include "chains_sac.h"

namespace pop {

template <class G>
__global__ __launch_bounds__(kThreads, 1) void k_sac_target(PopDev d, uint32_t t) {
  extern __shared__ float lds[];
  int agent, chunk;
  POP_BLOCK_TIME(kTraceTarget, 0);
  if (decode_block(blockIdx.x, d.P, d.B / G::R, agent, chunk)) sac_target_chain<G>(d, t, agent, chunk, lds);
  POP_BLOCK_TIME(kTraceTarget, 1);
}

template <class G>
__global__ __launch_bounds__(kThreads, 1) void k_sac_actor(PopDev d, uint32_t t) {
  extern __shared__ float lds[];
  int agent, chunk;
  POP_BLOCK_TIME(kTraceActor, 0);
  if (decode_block(blockIdx.x, d.P, d.B / G::R, agent, chunk)) sac_actor_chain<G>(d, t, agent, chunk, lds);
  POP_BLOCK_TIME(kTraceActor, 1);
}

// Target and critic chains in one launch, as for TD3 (k_chain.hip): the critics' forward pass runs beside
// the target workgroups and only the loss waits for the targets of its own rows.
template <class GT, class GC>
__global__ __launch_bounds__(kThreads, 1) void k_sac_target_critic(PopDev d, uint32_t t, int target_blocks) {
  extern __shared__ float lds[];
  int unit, chunk;
  POP_BLOCK_TIME(kTraceTargetCritic, 0);
  if ((int)blockIdx.x < target_blocks) {
    if (decode_block(blockIdx.x, d.P, d.B / GT::R, unit, chunk)) sac_target_chain<GT>(d, t, unit, chunk, lds);
  } else if (decode_block(blockIdx.x - target_blocks, 2 * d.P, d.B / GC::R, unit, chunk)) {
    critic_chain<GC, true, false>(d, t, unit, chunk, lds);
  }
  POP_BLOCK_TIME(kTraceTargetCritic, 1);
}

hipError_t setup_sac_kernels() {
  hipError_t e;
  const int most = 160 * 1024;
#define POP_SET_LDS(...)                                                                                   \
  if ((e = hipFuncSetAttribute((const void*)__VA_ARGS__, hipFuncAttributeMaxDynamicSharedMemorySize, most)) != hipSuccess) return e
  POP_SET_LDS(k_sac_target<Rows16>);
  POP_SET_LDS(k_sac_target<Rows32<1>>);
  POP_SET_LDS(k_sac_target<Rows32<2>>);
  POP_SET_LDS(k_sac_target<Rows16Deep>);
  POP_SET_LDS(k_sac_target<Rows32Deep<1>>);
  POP_SET_LDS(k_sac_actor<Rows16>);
  POP_SET_LDS(k_sac_actor<Rows32<1>>);
  POP_SET_LDS(k_sac_actor<Rows32<2>>);
  POP_SET_LDS(k_sac_actor<Rows16Deep>);
  POP_SET_LDS(k_sac_actor<Rows32Deep<1>>);
  POP_SET_LDS(k_sac_target_critic<Rows16, Rows32<2>>);
  POP_SET_LDS(k_sac_target_critic<Rows16, Rows32<1>>);
  POP_SET_LDS(k_sac_target_critic<Rows32<1>, Rows32<1>>);
#undef POP_SET_LDS
  return hipSuccess;
}

namespace {
size_t chain_lds(const PopDev& d, int rows, int regions, int vec) {
  return rows == 16 ? LdsMap<16, 16>(d.D, regions).bytes(vec)
         : rows == 32 ? LdsMap<32, 8>(d.D, regions).bytes(vec)
                      : LdsMap<64, 8>(d.D, regions).bytes(vec);
}
}  // namespace

size_t sac_lds_bytes(const PopDev& d) {
  size_t m = chain_lds(d, d.rows_t, kSacScratch, vec_sac_target(d));
  m = std::max(m, chain_lds(d, d.rows_a, kSacScratch, vec_sac_actor(d)) + (d.rows_a == 16 ? kStage16 * sizeof(float) : 0));   // weight stage
  m = std::max(m, chain_lds(d, d.rows_c, 3, vec_critic(d)));
  m = std::max(m, Lds<1>(d.O, kActScratch).bytes(vec_act(d)));
  return m;
}

hipError_t launch_sac_target(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(d.P, d.B / d.rows_t)), block(kThreads);
  const int vec = vec_sac_target(d);
  if (d.D > kMaxIn) {                                // wide inputs: 16 rows, pipelined first layers
    if (d.rows_t == 16) k_sac_target<Rows16Deep><<<grid, block, LdsMap<16, 16>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
    else if (d.rows_t == 32) k_sac_target<Rows32Deep<1>><<<grid, block, LdsMap<32, 8>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
    else return hipErrorInvalidValue;
  } else if (d.rows_t == 16) k_sac_target<Rows16><<<grid, block, LdsMap<16, 16>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
  else if (d.rows_t == 32) k_sac_target<Rows32<1>><<<grid, block, LdsMap<32, 8>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
  else k_sac_target<Rows32<2>><<<grid, block, LdsMap<64, 8>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
  return hipGetLastError();
}

hipError_t launch_sac_target_critic(const PopDev& d, uint32_t t, hipStream_t s) {
  const int nt = xcd_grid(d.P, d.B / d.rows_t), nc = xcd_grid(2 * d.P, d.B / d.rows_c);
  const dim3 grid(nt + nc), block(kThreads);
  const int vec = vec_sac_target(d);                 // larger than the critic chain's
  if (d.D > kMaxIn) return hipErrorInvalidValue;     // wide inputs run the two chains as separate launches
  if (d.rows_t == 16 && d.rows_c == 64) {
    const size_t a = LdsMap<16, 16>(d.D, kSacScratch).bytes(vec), b = Lds<2>(d.D).bytes(vec_critic(d));
    k_sac_target_critic<Rows16, Rows32<2>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
  } else if (d.rows_t == 16 && d.rows_c == 32) {
    const size_t a = LdsMap<16, 16>(d.D, kSacScratch).bytes(vec), b = Lds<1>(d.D).bytes(vec_critic(d));
    k_sac_target_critic<Rows16, Rows32<1>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
  } else if (d.rows_t == 32 && d.rows_c == 32) {
    const size_t a = LdsMap<32, 8>(d.D, kSacScratch).bytes(vec), b = Lds<1>(d.D).bytes(vec_critic(d));
    k_sac_target_critic<Rows32<1>, Rows32<1>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_sac_actor(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(d.P, d.B / d.rows_a)), block(kThreads);
  const int vec = vec_sac_actor(d);
  if (d.D > kMaxIn) {
    if (d.rows_a == 16) k_sac_actor<Rows16Deep><<<grid, block, LdsMap<16, 16>(d.D, kSacScratch).bytes(vec) + kStage16 * sizeof(float), s>>>(d, t);
    else if (d.rows_a == 32) k_sac_actor<Rows32Deep<1>><<<grid, block, LdsMap<32, 8>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
    else return hipErrorInvalidValue;
  } else if (d.rows_a == 16) k_sac_actor<Rows16><<<grid, block, LdsMap<16, 16>(d.D, kSacScratch).bytes(vec) + kStage16 * sizeof(float), s>>>(d, t);
  else if (d.rows_a == 32) k_sac_actor<Rows32<1>><<<grid, block, LdsMap<32, 8>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
  else k_sac_actor<Rows32<2>><<<grid, block, LdsMap<64, 8>(d.D, kSacScratch).bytes(vec), s>>>(d, t);
  return hipGetLastError();
}

}  // namespace pop
