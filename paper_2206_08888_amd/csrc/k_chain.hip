// Kernels around the layer chains of chains.h, one launch per chain:
//   k_target, k_critic, k_actor : the three chains of an update step
//   k_target_critic             : target and critic chains in one launch
//   k_act                       : obs -> actor (acting, no gradient)
#include <algorithm>
#include "chains.h"

namespace pop {

template <class G, int AS = kMaxAct>
__global__ __launch_bounds__(kThreads, 1) void k_target(PopDev d, uint32_t t) {
  extern __shared__ float lds[];
  int agent, chunk;
  POP_BLOCK_TIME(kTraceTarget, 0);
  if (decode_block(blockIdx.x, d.P, d.B / G::R, agent, chunk)) target_chain<G, AS>(d, t, agent, chunk, lds);
  POP_BLOCK_TIME(kTraceTarget, 1);
}

template <class G>
__global__ __launch_bounds__(kThreads, 1) void k_critic(PopDev d, uint32_t t) {
  extern __shared__ float lds[];
  int net, chunk;
  POP_BLOCK_TIME(kTraceCritic, 0);
  if (decode_block(blockIdx.x, 2 * d.P, d.B / G::R, net, chunk)) critic_chain<G, false, false>(d, t, net, chunk, lds);
  POP_BLOCK_TIME(kTraceCritic, 1);
}

// Target and critic chains of one step in a single launch.  The critic's forward pass does
// not need the Bellman targets, so its workgroups run beside the target workgroups and
// only wait, before the loss, for the targets of their own rows.  Target workgroups have the
// lower block indices: workgroups are dispatched in index order, so whatever a critic
// workgroup waits for has already been dispatched and the wait always ends.
// GT, GC: tile geometries of the two chains.  AHEAD: critic_chain's.
template <class GT, class GC, bool AHEAD = false>
__global__ __launch_bounds__(kThreads, 1) void k_target_critic(PopDev d, uint32_t t, int target_blocks) {
  extern __shared__ float lds[];
  int unit, chunk;
  POP_BLOCK_TIME(kTraceTargetCritic, 0);
  if ((int)blockIdx.x < target_blocks) {
    if (decode_block(blockIdx.x, d.P, d.B / GT::R, unit, chunk)) target_chain<GT>(d, t, unit, chunk, lds);
  } else if (decode_block(blockIdx.x - target_blocks, 2 * d.P, d.B / GC::R, unit, chunk)) {
    critic_chain<GC, true, false, AHEAD>(d, t, unit, chunk, lds);
  }
  POP_BLOCK_TIME(kTraceTargetCritic, 1);
}

// The same for populations whose 16-row target workgroups and 32-row critic workgroups do not all get a CU at
// once: a target workgroup goes on into critic 1 for its own 16 rows (its targets are its own, nothing waits),
// and only critic 2 has workgroups of its own.
template <class GC, bool AHEAD = false>
__global__ __launch_bounds__(kThreads, 1) void k_target_critic1(PopDev d, uint32_t t, int target_blocks) {
  extern __shared__ float lds[];
  int agent, chunk;
  POP_BLOCK_TIME(kTraceTargetCritic, 0);
  if ((int)blockIdx.x < target_blocks) {
    if (decode_block(blockIdx.x, d.P, d.B / 16, agent, chunk)) {
      target_chain<Rows16>(d, t, agent, chunk, lds);
      __syncthreads();                               // the chain is done with its LDS; a lane reads back the targets it wrote
      critic_chain<Rows16, false, false>(d, t, 2 * agent, chunk, lds);
    }
  } else if (decode_block(blockIdx.x - target_blocks, d.P, d.B / GC::R, agent, chunk)) {
    critic_chain<GC, true, false, AHEAD>(d, t, 2 * agent + 1, chunk, lds);
  }
  POP_BLOCK_TIME(kTraceTargetCritic, 1);
}

// PER_CU: workgroups per CU the register budget is set for; AHEAD, AS: actor_chain's
template <class G, int PER_CU = 1, bool AHEAD = false, int AS = kMaxAct>
__global__ __launch_bounds__(kThreads, PER_CU) void k_actor(PopDev d, uint32_t t) {
  extern __shared__ float lds[];
  int agent, chunk;
  POP_BLOCK_TIME(kTraceActor, 0);
  if (decode_block(blockIdx.x, d.P, d.B / G::R, agent, chunk)) actor_chain<G, false, AHEAD, AS>(d, t, agent, chunk, lds, 0);
  POP_BLOCK_TIME(kTraceActor, 1);
}

// ---------------------------------------------------------------------------------------------
// Acting: act[agent][r] = pi_agent(obs[agent][r]).  grid (ceil(n / 32), P).
// sigma != nullptr: Gaussian exploration noise, a = clip(pi + sigma[agent] eps, -1, 1) with eps =
// unit normal number (row_base + r) A + j of the agent's exploration stream at counter `step`
// (row_base: index of row 0 of this call within the caller's whole request).
__global__ __launch_bounds__(kThreads) void k_act(PopDev d, const float* __restrict__ obs, int n,
                                                  float* __restrict__ act, const float* __restrict__ sigma,
                                                  uint32_t step, uint32_t row_base) {
  constexpr int R = 32;
  extern __shared__ float lds[];
  constexpr int kHs = kSacMaxAct;                    // row stride of the head blocks: three [R][8] regions each
  const Lds<1> L(d.O, kActScratch);
  float* Xs = lds;
  float* buf = lds + L.buf;
  float* head = lds + L.s(0);
  float* head_ls = lds + L.s(kHs / kMaxAct);         // SAC: log-std head
  float* v_aw3 = lds + L.vec;
  float* v_ab3 = v_aw3 + kH * d.actor.out;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = blockIdx.y, r0 = blockIdx.x * R;
  const int valid = n - r0 < R ? n - r0 : R;
  const float* an = net_ptr(d, d.theta, agent, 0);
  LayerPre<1> pre;
  pre.load(an, d.actor, wave, lane);
  stage_head(v_aw3, an + d.actor.w3, d.actor.out, tid);      // SAC: 2A outputs, the means come first
  stage_vector(v_ab3, an + d.actor.b3, d.actor.out, tid);
  load_input<R>(Xs, L.xld, obs + ((size_t)agent * n + r0) * d.O, d.O, 0, d.O, valid, tid);
  __syncthreads();
  first_layer<1>(Xs, L.xld, an, d.actor, pre, buf, nullptr, wave, lane);
  __syncthreads();
  hidden_layer<1>(buf, an, d.actor, pre, nullptr, wave, lane, NoTail());
  __syncthreads();
  thin_wide<Rows32<1>>(buf, v_aw3, d.A, head, kHs, tid);
  const float sg = sigma ? sigma[agent] : 0.0f;
  const bool sac = d.algo == 1;
  if (sac && sg > 0.0f) thin_wide<Rows32<1>>(buf, v_aw3 + d.A * kH, d.A, head_ls, kHs, tid);
  __syncthreads();
  const HpDev hp = d.hp[agent];
  for (int e = tid; e < valid * d.A; e += kThreads) {
    const int r = e / d.A, j = e - r * d.A;
    const float pre_act = head[r * kHs + j] + v_ab3[j];
    float a = tanhf(pre_act);
    if (sg > 0.0f) {
      const uint32_t el = (row_base + (uint32_t)(r0 + r)) * (uint32_t)d.A + (uint32_t)j;
      const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, el >> 2, step, kStreamExplore, 0u);
      float n4[4];
      normals4(blk, n4);
      const float nz = (el & 2u) ? ((el & 1u) ? n4[3] : n4[2]) : ((el & 1u) ? n4[1] : n4[0]);
      if (sac) {                                     // a sample of the policy itself, its std scaled by sigma
        const float ls = fminf(fmaxf(head_ls[r * kHs + j] + v_ab3[d.A + j], -20.0f), 2.0f);
        a = tanhf(pre_act + sg * expf(ls) * nz);
      } else {
        a = fminf(fmaxf(a + sg * nz, -1.0f), 1.0f);
      }
    }
    act[((size_t)agent * n + r0 + r) * d.A + j] = a;
  }
}

hipError_t setup_kernels() {
  hipError_t e;
  const int most = 160 * 1024;                        // whole LDS of a CU; the launches ask for what they need
#define POP_SET_LDS(...)                                                                                   \
  if ((e = hipFuncSetAttribute((const void*)__VA_ARGS__, hipFuncAttributeMaxDynamicSharedMemorySize, most)) != hipSuccess) return e
  POP_SET_LDS(k_target<Rows16Deep, kSacMaxAct>);
  POP_SET_LDS(k_target<Rows32Deep<1>, kSacMaxAct>);
  POP_SET_LDS(k_actor<Rows16Deep, 1, false, kSacMaxAct>);
  POP_SET_LDS(k_actor<Rows32Deep<1>, 1, false, kSacMaxAct>);
  POP_SET_LDS(k_target<Rows16Deep>);
  POP_SET_LDS(k_target<Rows32Deep<1>>);
  POP_SET_LDS(k_actor<Rows16Deep>);
  POP_SET_LDS(k_actor<Rows32Deep<1>>);
  POP_SET_LDS(k_target<Rows16>);
  POP_SET_LDS(k_target<Rows32<1>>);
  POP_SET_LDS(k_target<Rows32<2>>);
  POP_SET_LDS(k_critic<Rows32<1>>);
  POP_SET_LDS(k_critic<Rows32<2>>);
  POP_SET_LDS(k_critic<Rows32Deep<1, 8>>);
  POP_SET_LDS(k_actor<Rows16>);
  POP_SET_LDS(k_actor<Rows32<1>>);
  POP_SET_LDS(k_actor<Rows32<1, true>, 2>);
  POP_SET_LDS(k_target_critic<Rows32<1, true>, Rows32<1, true>>);
  POP_SET_LDS(k_actor<Rows32<2>>);
  POP_SET_LDS(k_target_critic<Rows16, Rows32<2>>);
  POP_SET_LDS(k_target_critic<Rows16, Rows32<1>>);
  POP_SET_LDS(k_target_critic1<Rows32<1>>);
  POP_SET_LDS(k_target_critic1<Rows32<2>>);
  POP_SET_LDS(k_target_critic1<Rows32<1>, true>);
  POP_SET_LDS(k_target_critic<Rows16, Rows32<1>, true>);
  POP_SET_LDS(k_actor<Rows16, 1, true>);
  POP_SET_LDS(k_target_critic<Rows32<1>, Rows32<1>>);
  POP_SET_LDS(k_target_critic<Rows32<2>, Rows32<2>>);
  POP_SET_LDS(k_act);
#undef POP_SET_LDS
  return hipSuccess;
}

// Rows per workgroup (pop_dev.h): (target, critic, actor) = (16, 32 or 64, 16) for small
// populations, else (32, 32, 32); (64, 64, 64) on request.
// LDS of the largest chain workgroup of a TD3 step at these shapes (the launches below ask for what each needs)
size_t td3_lds_bytes(const PopDev& d) {
  auto chain = [&](int rows, int vec, bool staged, int regions) {
    return rows == 16 ? LdsMap<16, 16>(d.D, regions).bytes(vec) + (staged ? kStage16 * sizeof(float) : 0)
           : rows == 32 ? LdsMap<32, 8>(d.D, regions).bytes(vec) : LdsMap<64, 8>(d.D, regions).bytes(vec);
  };
  const int regions = d.A > kMaxAct ? kWideScratch : 3;
  size_t m = chain(d.rows_t, vec_target(d), false, regions);
  m = std::max(m, chain(d.rows_c, vec_critic(d), false, 3));
  m = std::max(m, chain(d.rows_a, vec_actor(d), true, regions));
  return std::max(m, Lds<1>(d.O, kActScratch).bytes(vec_act(d)));
}

hipError_t launch_target(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(d.P, d.B / d.rows_t)), block(kThreads);
  if (d.A > kMaxAct) {                               // wide actions: scratch rows of kSacMaxAct floats, first layers as for wide inputs
    if (d.rows_t == 16) k_target<Rows16Deep, kSacMaxAct><<<grid, block, LdsMap<16, 16>(d.D, kWideScratch).bytes(vec_target(d)), s>>>(d, t);
    else if (d.rows_t == 32) k_target<Rows32Deep<1>, kSacMaxAct><<<grid, block, LdsMap<32, 8>(d.D, kWideScratch).bytes(vec_target(d)), s>>>(d, t);
    else return hipErrorInvalidValue;
  } else if (d.D > kMaxIn) {                         // wide inputs: pipelined first layers, 16 or 32 rows
    if (d.rows_t == 16) k_target<Rows16Deep><<<grid, block, LdsMap<16, 16>(d.D).bytes(vec_target(d)), s>>>(d, t);
    else if (d.rows_t == 32) k_target<Rows32Deep<1>><<<grid, block, Lds<1>(d.D).bytes(vec_target(d)), s>>>(d, t);
    else return hipErrorInvalidValue;
  } else if (d.rows_t == 16) k_target<Rows16><<<grid, block, LdsMap<16, 16>(d.D).bytes(vec_target(d)), s>>>(d, t);
  else if (d.rows_t == 32) k_target<Rows32<1>><<<grid, block, Lds<1>(d.D).bytes(vec_target(d)), s>>>(d, t);
  else k_target<Rows32<2>><<<grid, block, Lds<2>(d.D).bytes(vec_target(d)), s>>>(d, t);
  return hipGetLastError();
}
hipError_t launch_critic(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(2 * d.P, d.B / d.rows_c)), block(kThreads);
  if (d.D > kMaxIn) {                                // wide inputs (SAC): 32 rows, pipelined first layer
    if (d.rows_c != 32) return hipErrorInvalidValue;
    k_critic<Rows32Deep<1, 8>><<<grid, block, Lds<1>(d.D).bytes(vec_critic(d)), s>>>(d, t);
  } else if (d.rows_c == 32) k_critic<Rows32<1>><<<grid, block, Lds<1>(d.D).bytes(vec_critic(d)), s>>>(d, t);
  else k_critic<Rows32<2>><<<grid, block, Lds<2>(d.D).bytes(vec_critic(d)), s>>>(d, t);
  return hipGetLastError();
}
hipError_t launch_target_critic(const PopDev& d, uint32_t t, hipStream_t s) {
  const int nt = xcd_grid(d.P, d.B / d.rows_t), nc = xcd_grid(2 * d.P, d.B / d.rows_c);
  const int vec = vec_target(d) > vec_critic(d) ? vec_target(d) : vec_critic(d);
  if (d.rows_c1 != d.rows_c) {                       // critic 1 inside the target workgroups
    if (d.rows_t != 16 || d.rows_c1 != 16 || (d.rows_c != 32 && d.rows_c != 64)) return hipErrorInvalidValue;
    // (the 16-row critic chain stages the weights of its transposed product in LDS)
    const size_t a = LdsMap<16, 16>(d.D).bytes(vec) + kStage16 * sizeof(float), b = d.rows_c == 32 ? Lds<1>(d.D).bytes(vec) : Lds<2>(d.D).bytes(vec);
    const dim3 grid(nt + xcd_grid(d.P, d.B / d.rows_c)), block(kThreads);
    if (d.actor_ahead) {
      if (d.rows_c != 32) return hipErrorInvalidValue;
      const size_t c = Lds<1>(d.D).bytes(kAheadBase + ahead_floats<32>());
      k_target_critic1<Rows32<1>, true><<<grid, block, a > c ? a : c, s>>>(d, t, nt);
    } else if (d.rows_c == 32) k_target_critic1<Rows32<1>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
    else k_target_critic1<Rows32<2>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
    return hipGetLastError();
  }
  const dim3 grid(nt + nc), block(kThreads);
  if (!(d.rows_t == 16 && (d.rows_c == 64 || d.rows_c == 32)) && !(d.rows_t == d.rows_c && (d.rows_t == 32 || d.rows_t == 64)))
    return hipErrorInvalidValue;                     // the kernel exists for these row classes only
  if (d.actor_ahead && !(d.rows_t == 16 && d.rows_c == 32)) return hipErrorInvalidValue;
  if (d.rows_t == 16 && d.rows_c == 32) {
    const size_t a = LdsMap<16, 16>(d.D).bytes(vec), b = Lds<1>(d.D).bytes(vec);
    if (d.actor_ahead) k_target_critic<Rows16, Rows32<1>, true><<<grid, block, Lds<1>(d.D).bytes(kAheadBase + ahead_floats<32>()), s>>>(d, t, nt);
    else k_target_critic<Rows16, Rows32<1>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
  } else if (d.rows_t == 16) {
    const size_t a = LdsMap<16, 16>(d.D).bytes(vec), b = Lds<2>(d.D).bytes(vec);
    k_target_critic<Rows16, Rows32<2>><<<grid, block, a > b ? a : b, s>>>(d, t, nt);
  } else if (d.rows_t == 32) {
    // more workgroups than CUs: two share a CU, and the products that issue their loads between the MFMAs pay
    if (nt + nc > kCUs) k_target_critic<Rows32<1, true>, Rows32<1, true>><<<grid, block, Lds<1>(d.D).bytes(vec), s>>>(d, t, nt);
    else k_target_critic<Rows32<1>, Rows32<1>><<<grid, block, Lds<1>(d.D).bytes(vec), s>>>(d, t, nt);
  } else {
    k_target_critic<Rows32<2>, Rows32<2>><<<grid, block, Lds<2>(d.D).bytes(vec), s>>>(d, t, nt);
  }
  return hipGetLastError();
}
hipError_t launch_actor(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(d.P, d.B / d.rows_a)), block(kThreads);
  if (d.A > kMaxAct) {
    if (d.actor_ahead) return hipErrorInvalidValue;
    if (d.rows_a == 16) k_actor<Rows16Deep, 1, false, kSacMaxAct><<<grid, block, LdsMap<16, 16>(d.D, kWideScratch).bytes(vec_actor(d)) + kStage16 * sizeof(float), s>>>(d, t);
    else if (d.rows_a == 32) k_actor<Rows32Deep<1>, 1, false, kSacMaxAct><<<grid, block, LdsMap<32, 8>(d.D, kWideScratch).bytes(vec_actor(d)), s>>>(d, t);
    else return hipErrorInvalidValue;
  } else if (d.D > kMaxIn) {
    if (d.actor_ahead) return hipErrorInvalidValue;
    if (d.rows_a == 16) k_actor<Rows16Deep><<<grid, block, LdsMap<16, 16>(d.D).bytes(vec_actor(d)) + kStage16 * sizeof(float), s>>>(d, t);
    else if (d.rows_a == 32) k_actor<Rows32Deep<1>><<<grid, block, Lds<1>(d.D).bytes(vec_actor(d)), s>>>(d, t);
    else return hipErrorInvalidValue;
  } else if (d.actor_ahead) {
    if (d.rows_a != 16) return hipErrorInvalidValue;
    k_actor<Rows16, 1, true><<<grid, block, LdsMap<16, 16>(d.D).bytes(vec_actor(d)) + kStage16 * sizeof(float), s>>>(d, t);
  } else if (d.rows_a == 16) k_actor<Rows16><<<grid, block, LdsMap<16, 16>(d.D).bytes(vec_actor(d)) + kStage16 * sizeof(float), s>>>(d, t);
  else if (d.rows_a == 32 && (int)grid.x > kCUs) k_actor<Rows32<1, true>, 2><<<grid, block, Lds<1>(d.D).bytes(vec_actor(d)), s>>>(d, t);
  else if (d.rows_a == 32) k_actor<Rows32<1>><<<grid, block, Lds<1>(d.D).bytes(vec_actor(d)), s>>>(d, t);
  else k_actor<Rows32<2>><<<grid, block, Lds<2>(d.D).bytes(vec_actor(d)), s>>>(d, t);
  return hipGetLastError();
}
hipError_t launch_act(const PopDev& d, const float* obs, int n, float* act, const float* sigma, uint32_t step,
                      uint32_t row_base, hipStream_t s) {
  k_act<<<dim3((n + 31) / 32, d.P), dim3(kThreads), Lds<1>(d.O, kActScratch).bytes(vec_act(d)), s>>>(d, obs, n, act, sigma, step,
                                                                                        row_base);
  return hipGetLastError();
}

}  // namespace pop
