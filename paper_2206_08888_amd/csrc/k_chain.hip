// Fused forward/backward chains of one TD3 update step (Sec. 4.1 of the paper:
// every population member takes the ordinary TD3 update on its own batch).
//
// The batch of an agent is cut into row chunks of R = 32 MT rows.  One
// workgroup owns one (agent or network, chunk) and walks the whole layer chain
// for its rows with the activations resident in LDS; only what the
// weight-gradient kernel needs later (layer inputs and pre-activation
// gradients) is written to global memory.  Rows of a batch interact only
// through the weight gradients, which are contracted over the full batch by a
// separate kernel, so chunks need no communication here.
//
//   k_target : s' -> target actor -> smoothing noise -> twin target critics -> y
//   k_critic : [s, a] -> critic k forward -> MSE seed gradient -> backward to
//              the pre-activation gradients of layers 2 and 1
//   k_actor  : s -> actor -> a_pi -> critic 1 forward -> gradient w.r.t. the
//              action -> actor backward
//   k_act    : obs -> actor (acting, no gradient)
//
// LDS economy: a hidden layer overwrites its own input tile (all wavefronts
// finish reading, barrier, then write), and ReLU patterns travel from the
// forward to the backward product as bit masks in registers, so one 256-wide
// tile per workgroup is enough (two in k_actor, which must keep the actor's
// second hidden layer while the critic runs).
#include "launch.h"
#include "mfma_tiles.h"
#include "rng.h"

namespace pop {

static_assert(kMaxAct == 8, "the action-gradient loops read dz3 rows as two 16-byte vectors");

namespace {

template <int MT, int NBUF>
struct Lds {
  static constexpr int R = 32 * MT;
  static constexpr int x_off = 0;                         // [R][kXld] first-layer input
  static constexpr int a_off = x_off + R * kXld;          // [R][kLda]
  static constexpr int b_off = a_off + R * kLda;          // [R][kLda] (NBUF == 2)
  static constexpr int s0_off = a_off + NBUF * R * kLda;  // [R][kMaxAct] scratch
  static constexpr int s1_off = s0_off + R * kMaxAct;
  static constexpr int s2_off = s1_off + R * kMaxAct;
  static constexpr int floats = s2_off + R * kMaxAct;
  static constexpr size_t bytes = (size_t)floats * sizeof(float);
};

// Copy columns [c0, c0 + n) of R batch rows into the LDS input tile at columns
// [0, n), zero the remaining columns; rows at or beyond `valid` become zero.
template <int R>
__device__ inline void load_input(float* Xl, const float* rows, int row_stride, int c0, int n, int valid, int tid) {
  for (int e = tid; e < R * kXld; e += kThreads) {
    const int r = e / kXld, c = e - r * kXld;
    Xl[e] = (c < n && r < valid) ? rows[(size_t)r * row_stride + c0 + c] : 0.0f;
  }
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// First layer (small fan-in) from the input tile into `Yl` (+ optional global copy).
template <int MT>
__device__ inline uint64_t first_layer(const float* Xs, int K, const float* W, const float* b, float* Yl, float* Yg,
                                       int wave, int lane) {
  Acc<MT> acc;
  acc.zero();
  gemm_xw_small<MT>(Xs, kXld, K, W, wave, lane, acc);
  return relu_store<MT>(acc, b, Yl, Yg, wave, lane);
}

// Second layer: reads the tile `Xl` and writes `Yl`; Yl == Xl is allowed (the
// barrier between product and store makes the overwrite safe).
template <int MT>
__device__ inline uint64_t hidden_layer(const float* Xl, const float* W, const float* b, float* Yl, float* Yg,
                                        int wave, int lane) {
  Acc<MT> acc;
  acc.zero();
  gemm256<MT, false>(Xl, kLda, W, wave, lane, acc);
  if (Yl == Xl) __syncthreads();
  return relu_store<MT>(acc, b, Yl, Yg, wave, lane);
}

// dX = (dZ W^T) * mask written to global [rows][256]; column sums of the result
// (over this workgroup's rows) go to colsum_out[256].
template <int MT>
__device__ inline void input_grad_to_global(const float* Zl, const float* W, uint64_t mask, float* __restrict__ dXg,
                                            float* __restrict__ colsum_out, int wave, int lane) {
  Acc<MT> acc;
  acc.zero();
  gemm256<MT, true>(Zl, kLda, W, wave, lane, acc);
  float cs[2] = {0.0f, 0.0f};
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float z = mask_bit(mask, mt, nt, v) ? acc.t[mt][nt][v] : 0.0f;
        dXg[(size_t)(32 * mt + acc_row(v, lane)) * kH + 64 * wave + 32 * nt + (lane & 31)] = z;
        cs[nt] += z;
      }
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float tot = cs[nt] + __shfl_xor(cs[nt], 32);
    if (lane < 32) colsum_out[64 * wave + 32 * nt + lane] = tot;
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Target chain.  One workgroup per (agent, chunk).
//   a~ = clip(pi'(s') + clip(sigma eps, -c, c), -1, 1), eps = normal e = b A + j of stream 1
//   y  = r + gamma (1 - d) min(Q1'(s', a~), Q2'(s', a~))
template <int MT>
__global__ __launch_bounds__(kThreads) void k_target(PopDev d, uint32_t t) {
  using L = Lds<MT, 1>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* buf = lds + L::a_off;
  float* head = lds + L::s0_off;
  float* qmin = lds + L::s1_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  int agent, chunk;
  if (!decode_block(blockIdx.x, d.P, d.chunks, agent, chunk)) return;
  const int r0 = chunk * R;
  const HpDev hp = d.hp[agent];
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;

  load_input<R>(Xs, rows, d.row, d.D + 2, d.O, R, tid);
  __syncthreads();
  const float* ta = net_ptr(d, d.target, agent, 0);
  first_layer<MT>(Xs, d.O, ta + d.actor.w1, ta + d.actor.b1, buf, nullptr, wave, lane);
  __syncthreads();
  hidden_layer<MT>(buf, ta + d.actor.w2, ta + d.actor.b2, buf, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, true>(buf, ta + d.actor.w3, d.A, head, tid);
  __syncthreads();
  for (int e = tid; e < R * d.A; e += kThreads) {
    const int r = e / d.A, j = e - r * d.A;
    const float mu = tanhf(head[r * kMaxAct + j] + ta[d.actor.b3 + j]);
    const uint32_t el = (uint32_t)((r0 + r) * d.A + j);
    const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, el >> 2, t, kStreamSmooth, 0u);
    float n4[4];
    normals4(blk, n4);
    const float noise = fminf(fmaxf(hp.policy_noise * ((el & 2u) ? ((el & 1u) ? n4[3] : n4[2]) : ((el & 1u) ? n4[1] : n4[0])), -hp.noise_clip), hp.noise_clip);
    const float at = fminf(fmaxf(mu + noise, -1.0f), 1.0f);
    Xs[r * kXld + d.O + j] = at;
    d.atilde[((size_t)agent * d.B + r0 + r) * d.A + j] = at;
  }
  __syncthreads();

  for (int k = 0; k < 2; ++k) {
    const float* tc = net_ptr(d, d.target, agent, 1 + k);
    first_layer<MT>(Xs, d.D, tc + d.critic.w1, tc + d.critic.b1, buf, nullptr, wave, lane);
    __syncthreads();
    hidden_layer<MT>(buf, tc + d.critic.w2, tc + d.critic.b2, buf, nullptr, wave, lane);
    __syncthreads();
    thin_dot<R, false>(buf, tc + d.critic.w3, 1, head, tid);
    __syncthreads();
    if (tid < R) {
      const float q = head[tid * kMaxAct] + tc[d.critic.b3];
      qmin[tid] = k == 0 ? q : fminf(qmin[tid], q);
    }
    __syncthreads();
  }
  if (tid < R) {
    const float rew = rows[(size_t)tid * d.row + d.D];
    const float done = rows[(size_t)tid * d.row + d.D + 1];
    d.y[(size_t)agent * d.B + r0 + tid] = rew + hp.gamma * (1.0f - done) * qmin[tid];
  }
}

// ---------------------------------------------------------------------------------------------
// Critic forward + backward.  One workgroup per (critic network, chunk); network = 2 agent + k.
//   L = (1/B) sum_b (Q_k(s_b, a_b) - y_b)^2 ;  dq = 2 (q - y) / B
//   dz2 = (dq W3^T) * [h2 > 0] ;  dz1 = (dz2 W2^T) * [h1 > 0]
// Outputs for the weight-gradient kernel: h1, dz2, dz1 (global), and the chunk's
// partial sums of dW3, db3, db2, db1 and of the loss.
template <int MT>
__global__ __launch_bounds__(kThreads) void k_critic(PopDev d, uint32_t t) {
  using L = Lds<MT, 1>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* buf = lds + L::a_off;
  float* head = lds + L::s0_off;
  float* dq = lds + L::s1_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  int net, chunk;
  if (!decode_block(blockIdx.x, 2 * d.P, d.chunks, net, chunk)) return;
  const int agent = net >> 1, k = net & 1, r0 = chunk * R;
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  const float* cn = net_ptr(d, d.theta, agent, 1 + k);
  const size_t act_off = ((size_t)net * d.B + r0) * kH;
  float* part = d.cpart + ((size_t)net * d.chunks + chunk) * kCPart;

  load_input<R>(Xs, rows, d.row, 0, d.D, R, tid);
  __syncthreads();
  const uint64_t mask1 = first_layer<MT>(Xs, d.D, cn + d.critic.w1, cn + d.critic.b1, buf, d.cH1 + act_off, wave, lane);
  __syncthreads();
  hidden_layer<MT>(buf, cn + d.critic.w2, cn + d.critic.b2, buf, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, false>(buf, cn + d.critic.w3, 1, head, tid);
  __syncthreads();
  if (tid < 64) {                                   // R <= 64: one wavefront covers the chunk
    float err = 0.0f, g = 0.0f;
    if (tid < R) {
      err = head[tid * kMaxAct] + cn[d.critic.b3] - d.y[(size_t)agent * d.B + r0 + tid];
      g = 2.0f * err / (float)d.B;
      dq[tid] = g;
    }
    const float sq = wave_sum(err * err);
    const float sdq = wave_sum(g);
    if (tid == 0) { part[kCP_loss] = sq / (float)d.B; part[kCP_db3] = sdq; }
  }
  __syncthreads();
  {                                                 // one thread per hidden unit, 8 rows at a time
    const int c = tid;
    const float w3 = cn[d.critic.w3 + c];
    float gw3 = 0.0f, gb2 = 0.0f;
    float* zg = d.cdZ2 + act_off + c;
#pragma unroll 1
    for (int rb = 0; rb < R; rb += 8) {
      float h[8], g[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { h[i] = buf[(rb + i) * kLda + c]; g[i] = dq[rb + i]; }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        gw3 += h[i] * g[i];
        const float z = h[i] > 0.0f ? g[i] * w3 : 0.0f;
        buf[(rb + i) * kLda + c] = z;
        zg[(size_t)(rb + i) * kH] = z;
        gb2 += z;
      }
    }
    part[kCP_dW3 + c] = gw3;
    part[kCP_db2 + c] = gb2;
  }
  __syncthreads();
  input_grad_to_global<MT>(buf, cn + d.critic.w2, mask1, d.cdZ1 + act_off, part + kCP_db1, wave, lane);
}

// ---------------------------------------------------------------------------------------------
// Actor chain (steps with t % policy_delay == 0).  One workgroup per (agent, chunk).
//   L = -(1/B) sum_b Q1(s_b, pi(s_b)) through the critic updated earlier in this step.
//   Critic 1: dz2c = -(1/B) W3c^T * [c2 > 0]; dz1c = (dz2c W2c^T) * [c1 > 0];
//             da = dz1c W1c[O:O+A, :]^T
//   Actor:    dz3 = da (1 - a_pi^2); dz2 = (dz3 W3^T) * [h2 > 0]; dz1 = (dz2 W2^T) * [h1 > 0]
template <int MT>
__global__ __launch_bounds__(kThreads) void k_actor(PopDev d, uint32_t t) {
  using L = Lds<MT, 2>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* bufA = lds + L::a_off;
  float* bufB = lds + L::b_off;
  float* head = lds + L::s0_off;
  float* api = lds + L::s1_off;
  float* dz3 = lds + L::s2_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  int agent, chunk;
  if (!decode_block(blockIdx.x, d.P, d.chunks, agent, chunk)) return;
  const int r0 = chunk * R;
  const HpDev hp = d.hp[agent];
  if (t % (uint32_t)hp.policy_delay != 0u) return;
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  const float* an = net_ptr(d, d.theta, agent, 0);
  const float* cn = net_ptr(d, d.theta, agent, 1);
  const size_t act_off = ((size_t)agent * d.B + r0) * kH;
  float* part = d.apart + ((size_t)agent * d.chunks + chunk) * kAPart;
  const int A = d.A;

  load_input<R>(Xs, rows, d.row, 0, d.O, R, tid);
  __syncthreads();
  const uint64_t mask_a1 = first_layer<MT>(Xs, d.O, an + d.actor.w1, an + d.actor.b1, bufA, d.aH1 + act_off, wave, lane);
  __syncthreads();
  hidden_layer<MT>(bufA, an + d.actor.w2, an + d.actor.b2, bufB, nullptr, wave, lane);   // bufB = h2 of the actor
  __syncthreads();
  thin_dot<R, true>(bufB, an + d.actor.w3, A, head, tid);
  __syncthreads();
  for (int e = tid; e < R * A; e += kThreads) {
    const int r = e / A, j = e - r * A;
    const float a = tanhf(head[r * kMaxAct + j] + an[d.actor.b3 + j]);
    api[r * kMaxAct + j] = a;
    Xs[r * kXld + d.O + j] = a;
  }
  __syncthreads();

  // critic 1 on [s, a_pi]
  const uint64_t mask_c1 = first_layer<MT>(Xs, d.D, cn + d.critic.w1, cn + d.critic.b1, bufA, nullptr, wave, lane);
  __syncthreads();
  hidden_layer<MT>(bufA, cn + d.critic.w2, cn + d.critic.b2, bufA, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, false>(bufA, cn + d.critic.w3, 1, head, tid);     // q, for the loss value only
  __syncthreads();
  if (tid < 64) {
    const float q = tid < R ? head[tid * kMaxAct] + cn[d.critic.b3] : 0.0f;
    const float s = wave_sum(q);
    if (tid == 0) part[kAP_loss] = -s / (float)d.B;
  }
  {
    const int c = tid;
    const float seed = -cn[d.critic.w3 + c] / (float)d.B;
#pragma unroll 1
    for (int rb = 0; rb < R; rb += 8) {
      float h[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) h[i] = bufA[(rb + i) * kLda + c];
#pragma unroll
      for (int i = 0; i < 8; ++i) bufA[(rb + i) * kLda + c] = h[i] > 0.0f ? seed : 0.0f;
    }
  }
  __syncthreads();
  {
    Acc<MT> acc;
    acc.zero();
    gemm256<MT, true>(bufA, kLda, cn + d.critic.w2, wave, lane, acc);
    __syncthreads();                                 // every wavefront is done reading dz2 of the critic
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          bufA[(32 * mt + acc_row(v, lane)) * kLda + 64 * wave + 32 * nt + (lane & 31)] =
              mask_bit(mask_c1, mt, nt, v) ? acc.t[mt][nt][v] : 0.0f;      // dz1 of the critic
  }
  __syncthreads();
  thin_dot<R, false>(bufA, cn + d.critic.w1 + (size_t)d.O * kH, A, head, tid);   // da
  __syncthreads();
  for (int e = tid; e < R * kMaxAct; e += kThreads) {
    const int j = e % kMaxAct;
    const float a = j < A ? api[e] : 0.0f;
    dz3[e] = j < A ? head[e] * (1.0f - a * a) : 0.0f;     // unused columns are kept at zero
  }
  __syncthreads();
  if (tid < A) {
    float s = 0.0f;
    for (int r = 0; r < R; ++r) s += dz3[r * kMaxAct + tid];
    part[kAP_db3 + tid] = s;
  }
  {                                                  // actor head backward, one thread per hidden unit
    const int c = tid;
    float w3[kMaxAct], gw3[kMaxAct];
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j) { w3[j] = j < A ? an[d.actor.w3 + c * A + j] : 0.0f; gw3[j] = 0.0f; }
    float gb2 = 0.0f;
    float* zg = d.adZ2 + act_off + c;
#pragma unroll 1
    for (int rb = 0; rb < R; rb += 4) {
      float h[4];
      f32x4 g[4][2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        h[i] = bufB[(rb + i) * kLda + c];
        g[i][0] = *reinterpret_cast<const f32x4*>(&dz3[(rb + i) * kMaxAct]);      // columns >= A hold zeros
        g[i][1] = *reinterpret_cast<const f32x4*>(&dz3[(rb + i) * kMaxAct + 4]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float dh = 0.0f;
#pragma unroll
        for (int j = 0; j < kMaxAct; ++j) {
          const float gj = g[i][j >> 2][j & 3];
          gw3[j] += h[i] * gj;
          dh += gj * w3[j];
        }
        const float z = h[i] > 0.0f ? dh : 0.0f;
        bufB[(rb + i) * kLda + c] = z;
        zg[(size_t)(rb + i) * kH] = z;
        gb2 += z;
      }
    }
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j)
      if (j < A) part[kAP_dW3 + c * A + j] = gw3[j];
    part[kAP_db2 + c] = gb2;
  }
  __syncthreads();
  input_grad_to_global<MT>(bufB, an + d.actor.w2, mask_a1, d.adZ1 + act_off, part + kAP_db1, wave, lane);
}

// ---------------------------------------------------------------------------------------------
// Acting: act[agent][r] = pi_agent(obs[agent][r]).  grid (ceil(n / 32), P).
__global__ __launch_bounds__(kThreads) void k_act(PopDev d, const float* __restrict__ obs, int n,
                                                  float* __restrict__ act) {
  using L = Lds<1, 1>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* buf = lds + L::a_off;
  float* head = lds + L::s0_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = blockIdx.y, r0 = blockIdx.x * R;
  const int valid = n - r0 < R ? n - r0 : R;
  const float* an = net_ptr(d, d.theta, agent, 0);
  load_input<R>(Xs, obs + ((size_t)agent * n + r0) * d.O, d.O, 0, d.O, valid, tid);
  __syncthreads();
  first_layer<1>(Xs, d.O, an + d.actor.w1, an + d.actor.b1, buf, nullptr, wave, lane);
  __syncthreads();
  hidden_layer<1>(buf, an + d.actor.w2, an + d.actor.b2, buf, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, true>(buf, an + d.actor.w3, d.A, head, tid);
  __syncthreads();
  for (int e = tid; e < valid * d.A; e += kThreads) {
    const int r = e / d.A, j = e - r * d.A;
    act[((size_t)agent * n + r0 + r) * d.A + j] = tanhf(head[r * kMaxAct + j] + an[d.actor.b3 + j]);
  }
}

// ---------------------------------------------------------------------------------------------
hipError_t setup_kernels() {
  hipError_t e;
#define POP_SET_LDS(fn, bytes)                                                                       \
  if ((e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes))) != hipSuccess) return e
  POP_SET_LDS(k_target<1>, (Lds<1, 1>::bytes));
  POP_SET_LDS(k_target<2>, (Lds<2, 1>::bytes));
  POP_SET_LDS(k_critic<1>, (Lds<1, 1>::bytes));
  POP_SET_LDS(k_critic<2>, (Lds<2, 1>::bytes));
  POP_SET_LDS(k_actor<1>, (Lds<1, 2>::bytes));
  POP_SET_LDS(k_actor<2>, (Lds<2, 2>::bytes));
  POP_SET_LDS(k_act, (Lds<1, 1>::bytes));
#undef POP_SET_LDS
  return hipSuccess;
}

hipError_t launch_target(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(d.P, d.chunks));
  if (d.mt == 2) k_target<2><<<grid, dim3(kThreads), Lds<2, 1>::bytes, s>>>(d, t);
  else k_target<1><<<grid, dim3(kThreads), Lds<1, 1>::bytes, s>>>(d, t);
  return hipGetLastError();
}
hipError_t launch_critic(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(2 * d.P, d.chunks));
  if (d.mt == 2) k_critic<2><<<grid, dim3(kThreads), Lds<2, 1>::bytes, s>>>(d, t);
  else k_critic<1><<<grid, dim3(kThreads), Lds<1, 1>::bytes, s>>>(d, t);
  return hipGetLastError();
}
hipError_t launch_actor(const PopDev& d, uint32_t t, hipStream_t s) {
  const dim3 grid(xcd_grid(d.P, d.chunks));
  if (d.mt == 2) k_actor<2><<<grid, dim3(kThreads), Lds<2, 2>::bytes, s>>>(d, t);
  else k_actor<1><<<grid, dim3(kThreads), Lds<1, 2>::bytes, s>>>(d, t);
  return hipGetLastError();
}
hipError_t launch_act(const PopDev& d, const float* obs, int n, float* act, hipStream_t s) {
  k_act<<<dim3((n + 31) / 32, d.P), dim3(kThreads), Lds<1, 1>::bytes, s>>>(d, obs, n, act);
  return hipGetLastError();
}

}  // namespace pop
