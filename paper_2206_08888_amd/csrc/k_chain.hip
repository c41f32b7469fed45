// Fused forward/backward chains of one TD3 update step (Sec. 4.1 of the paper:
// every population member takes the ordinary TD3 update on its own batch).
//
// The batch of an agent is cut into row chunks of R = 32 MT rows.  One
// workgroup owns one (agent, network, chunk) and walks the whole layer chain
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
#include "launch.h"
#include "mfma_tiles.h"
#include "rng.h"

namespace pop {

namespace {

template <int MT>
struct Lds {
  static constexpr int R = 32 * MT;
  static constexpr int x_off = 0;                      // [R][kXld] first-layer input
  static constexpr int a_off = x_off + R * kXld;       // [R][kLda]
  static constexpr int b_off = a_off + R * kLda;       // [R][kLda]
  static constexpr int s0_off = b_off + R * kLda;      // [R][kMaxAct] scratch
  static constexpr int s1_off = s0_off + R * kMaxAct;  // [R][kMaxAct]
  static constexpr int s2_off = s1_off + R * kMaxAct;  // [R][kMaxAct]
  static constexpr int floats = s2_off + R * kMaxAct;
  static constexpr size_t bytes = (size_t)floats * sizeof(float);
};

// Copy columns [c0, c0 + n) of R batch rows into the LDS input tile at
// columns [dst, dst + n); rows at or beyond `valid` become zero.
template <int R>
__device__ inline void load_cols(float* Xl, int dst, const float* rows, int row_stride, int c0, int n, int valid,
                                 int tid) {
  for (int e = tid; e < R * n; e += kThreads) {
    const int r = e / n, c = e - r * n;
    Xl[r * kXld + dst + c] = r < valid ? rows[(size_t)r * row_stride + c0 + c] : 0.0f;
  }
}

template <int R>
__device__ inline void zero_input(float* Xl, int tid) {
  for (int e = tid; e < R * kXld; e += kThreads) Xl[e] = 0.0f;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Column sums over the rows this wavefront holds in its accumulators (all R
// rows of its 64 columns); lanes < 32 end up with the sums of columns
// 64 wave + 32 nt + lane.
template <int MT, class F>
__device__ inline void store_masked_and_colsum(const Acc<MT>& acc, int wave, int lane, F elem, float* colsum_out) {
  float cs[2] = {0.0f, 0.0f};
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        cs[nt] += elem(32 * mt + acc_row(v, lane), 64 * wave + 32 * nt + (lane & 31), acc.t[mt][nt][v]);
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const float tot = cs[nt] + __shfl_xor(cs[nt], 32);
    if (lane < 32) colsum_out[64 * wave + 32 * nt + lane] = tot;
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Target chain.  grid (chunks, P).
//   a~ = clip(pi'(s') + clip(sigma eps, -c, c), -1, 1), eps = normal e = b A + j of stream 1
//   y  = r + gamma (1 - d) min(Q1'(s', a~), Q2'(s', a~))
template <int MT>
__global__ __launch_bounds__(kThreads) void k_target(PopDev d, uint32_t t) {
  using L = Lds<MT>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* bufA = lds + L::a_off;
  float* bufB = lds + L::b_off;
  float* head = lds + L::s0_off;
  float* qmin = lds + L::s1_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = blockIdx.y, r0 = blockIdx.x * R;
  const HpDev hp = d.hp[agent];
  const float* rows = d.batch + ((size_t)agent * d.B + r0) * d.row;

  zero_input<R>(Xs, tid);
  __syncthreads();
  load_cols<R>(Xs, 0, rows, d.row, d.D + 2, d.O, R, tid);
  __syncthreads();

  const float* ta = net_ptr(d, d.target, agent, 0);
  layer_relu<MT, false>(Xs, kXld, d.O, ta + d.actor.w1, ta + d.actor.b1, bufA, nullptr, wave, lane);
  __syncthreads();
  layer_relu<MT, true>(bufA, kLda, kH, ta + d.actor.w2, ta + d.actor.b2, bufB, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, true>(bufB, ta + d.actor.w3, d.A, head, tid);
  __syncthreads();
  for (int e = tid; e < R * d.A; e += kThreads) {
    const int r = e / d.A, j = e - r * d.A;
    const float mu = tanhf(head[r * kMaxAct + j] + ta[d.actor.b3 + j]);
    const uint32_t el = (uint32_t)((r0 + r) * d.A + j);
    const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, el >> 2, t, kStreamSmooth, 0u);
    float n4[4];
    normals4(blk, n4);
    const float noise = fminf(fmaxf(hp.policy_noise * n4[el & 3], -hp.noise_clip), hp.noise_clip);
    const float at = fminf(fmaxf(mu + noise, -1.0f), 1.0f);
    Xs[r * kXld + d.O + j] = at;
    d.atilde[((size_t)agent * d.B + r0 + r) * d.A + j] = at;
  }
  __syncthreads();

  for (int k = 0; k < 2; ++k) {
    const float* tc = net_ptr(d, d.target, agent, 1 + k);
    layer_relu<MT, false>(Xs, kXld, d.D, tc + d.critic.w1, tc + d.critic.b1, bufA, nullptr, wave, lane);
    __syncthreads();
    layer_relu<MT, true>(bufA, kLda, kH, tc + d.critic.w2, tc + d.critic.b2, bufB, nullptr, wave, lane);
    __syncthreads();
    thin_dot<R, false>(bufB, tc + d.critic.w3, 1, head, tid);
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
// Critic forward + backward.  grid (chunks, 2 P); blockIdx.y = 2 agent + k.
//   L = (1/B) sum_b (Q_k(s_b, a_b) - y_b)^2 ;  dq = 2 (q - y) / B
//   dz2 = (dq W3^T) * [h2 > 0] ;  dz1 = (dz2 W2^T) * [h1 > 0]
// Outputs for the weight-gradient kernel: h1, dz2, dz1 (global), and the chunk's
// partial sums of dW3, db3, db2, db1 and of the loss.
template <int MT>
__global__ __launch_bounds__(kThreads) void k_critic(PopDev d, uint32_t t) {
  using L = Lds<MT>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* bufA = lds + L::a_off;
  float* bufB = lds + L::b_off;
  float* head = lds + L::s0_off;
  float* dq = lds + L::s1_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = blockIdx.y >> 1, k = blockIdx.y & 1, chunk = blockIdx.x, r0 = chunk * R;
  const float* rows = d.batch + ((size_t)agent * d.B + r0) * d.row;
  const float* cn = net_ptr(d, d.theta, agent, 1 + k);
  const size_t act_off = (((size_t)agent * 2 + k) * d.B + r0) * kH;
  float* part = d.cpart + (((size_t)agent * 2 + k) * d.chunks + chunk) * kCPart;

  zero_input<R>(Xs, tid);
  __syncthreads();
  load_cols<R>(Xs, 0, rows, d.row, 0, d.D, R, tid);
  __syncthreads();
  layer_relu<MT, false>(Xs, kXld, d.D, cn + d.critic.w1, cn + d.critic.b1, bufA, d.cH1 + act_off, wave, lane);
  __syncthreads();
  layer_relu<MT, true>(bufA, kLda, kH, cn + d.critic.w2, cn + d.critic.b2, bufB, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, false>(bufB, cn + d.critic.w3, 1, head, tid);
  __syncthreads();
  if (tid < 64) {                                   // R <= 64: one wavefront covers the chunk
    float err = 0.0f;
    if (tid < R) {
      err = head[tid * kMaxAct] + cn[d.critic.b3] - d.y[(size_t)agent * d.B + r0 + tid];
      dq[tid] = 2.0f * err / (float)d.B;
    }
    const float sq = wave_sum(err * err);
    const float sdq = wave_sum(tid < R ? 2.0f * err / (float)d.B : 0.0f);
    if (tid == 0) { part[kCP_loss] = sq / (float)d.B; part[kCP_db3] = sdq; }
  }
  __syncthreads();
  {                                                 // one thread per hidden unit
    const int c = tid;
    const float w3 = cn[d.critic.w3 + c];
    float gw3 = 0.0f, gb2 = 0.0f;
    float* zg = d.cdZ2 + act_off + c;
    for (int r = 0; r < R; ++r) {
      const float h = bufB[r * kLda + c];
      gw3 += h * dq[r];
      const float z = h > 0.0f ? dq[r] * w3 : 0.0f;
      bufB[r * kLda + c] = z;
      zg[(size_t)r * kH] = z;
      gb2 += z;
    }
    part[kCP_dW3 + c] = gw3;
    part[kCP_db2 + c] = gb2;
  }
  __syncthreads();
  Acc<MT> acc;
  acc.zero();
  gemm_zwt<MT>(bufB, cn + d.critic.w2, wave, lane, acc);
  float* z1g = d.cdZ1 + act_off;
  store_masked_and_colsum<MT>(acc, wave, lane,
      [&](int row, int col, float v) {
        const float z = bufA[row * kLda + col] > 0.0f ? v : 0.0f;
        z1g[(size_t)row * kH + col] = z;
        return z;
      }, part + kCP_db1);
}

// ---------------------------------------------------------------------------------------------
// Actor chain (steps with t % policy_delay == 0).  grid (chunks, P).
//   L = -(1/B) sum_b Q1(s_b, pi(s_b)) through the critic updated earlier in this step.
//   Critic 1: dz2c = -(1/B) W3c^T * [c2 > 0]; dz1c = (dz2c W2c^T) * [c1 > 0];
//             da = dz1c W1c[O:O+A, :]^T
//   Actor:    dz3 = da (1 - a_pi^2); dz2 = (dz3 W3^T) * [h2 > 0]; dz1 = (dz2 W2^T) * [h1 > 0]
template <int MT>
__global__ __launch_bounds__(kThreads) void k_actor(PopDev d, uint32_t t) {
  using L = Lds<MT>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* bufA = lds + L::a_off;
  float* bufB = lds + L::b_off;
  float* head = lds + L::s0_off;
  float* api = lds + L::s1_off;
  float* dz3 = lds + L::s2_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = blockIdx.y, chunk = blockIdx.x, r0 = chunk * R;
  const HpDev hp = d.hp[agent];
  if (t % (uint32_t)hp.policy_delay != 0u) return;
  const float* rows = d.batch + ((size_t)agent * d.B + r0) * d.row;
  const float* an = net_ptr(d, d.theta, agent, 0);
  const float* cn = net_ptr(d, d.theta, agent, 1);
  const size_t act_off = ((size_t)agent * d.B + r0) * kH;
  float* part = d.apart + ((size_t)agent * d.chunks + chunk) * kAPart;
  const int A = d.A;

  zero_input<R>(Xs, tid);
  __syncthreads();
  load_cols<R>(Xs, 0, rows, d.row, 0, d.O, R, tid);
  __syncthreads();
  layer_relu<MT, false>(Xs, kXld, d.O, an + d.actor.w1, an + d.actor.b1, bufA, d.aH1 + act_off, wave, lane);
  __syncthreads();
  layer_relu<MT, true>(bufA, kLda, kH, an + d.actor.w2, an + d.actor.b2, bufB, d.aH2 + act_off, wave, lane);
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
  layer_relu<MT, false>(Xs, kXld, d.D, cn + d.critic.w1, cn + d.critic.b1, bufA, nullptr, wave, lane);
  __syncthreads();
  layer_relu<MT, true>(bufA, kLda, kH, cn + d.critic.w2, cn + d.critic.b2, bufB, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, false>(bufB, cn + d.critic.w3, 1, head, tid);     // q, for the loss value only
  __syncthreads();
  if (tid < 64) {
    const float q = tid < R ? head[tid * kMaxAct] + cn[d.critic.b3] : 0.0f;
    const float s = wave_sum(q);
    if (tid == 0) part[kAP_loss] = -s / (float)d.B;
  }
  {
    const int c = tid;
    const float seed = -cn[d.critic.w3 + c] / (float)d.B;
    for (int r = 0; r < R; ++r) bufB[r * kLda + c] = bufB[r * kLda + c] > 0.0f ? seed : 0.0f;
  }
  __syncthreads();
  {
    Acc<MT> acc;
    acc.zero();
    gemm_zwt<MT>(bufB, cn + d.critic.w2, wave, lane, acc);
    for_each_acc<MT>(acc, wave, lane, [&](int row, int col, float v) {
      float* p = &bufA[row * kLda + col];
      *p = *p > 0.0f ? v : 0.0f;                     // dz1 of the critic, in place over c1
    });
  }
  __syncthreads();
  thin_dot<R, false>(bufA, cn + d.critic.w1 + (size_t)d.O * kH, A, head, tid);   // da
  __syncthreads();
  for (int e = tid; e < R * A; e += kThreads) {
    const int r = e / A, j = e - r * A;
    const float a = api[r * kMaxAct + j];
    dz3[r * kMaxAct + j] = head[r * kMaxAct + j] * (1.0f - a * a);
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
    const float* h2g = d.aH2 + act_off + c;           // written by this workgroup above
    float* zg = d.adZ2 + act_off + c;
    for (int r = 0; r < R; ++r) {
      const float h = h2g[(size_t)r * kH];
      float dh = 0.0f;
#pragma unroll
      for (int j = 0; j < kMaxAct; ++j) {
        const float g = j < A ? dz3[r * kMaxAct + j] : 0.0f;
        gw3[j] += h * g;
        dh += g * w3[j];
      }
      const float z = h > 0.0f ? dh : 0.0f;
      bufB[r * kLda + c] = z;
      zg[(size_t)r * kH] = z;
      gb2 += z;
    }
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j)
      if (j < A) part[kAP_dW3 + c * A + j] = gw3[j];
    part[kAP_db2 + c] = gb2;
  }
  __syncthreads();
  Acc<MT> acc;
  acc.zero();
  gemm_zwt<MT>(bufB, an + d.actor.w2, wave, lane, acc);
  const float* h1g = d.aH1 + act_off;
  float* z1g = d.adZ1 + act_off;
  store_masked_and_colsum<MT>(acc, wave, lane,
      [&](int row, int col, float v) {
        const float z = h1g[(size_t)row * kH + col] > 0.0f ? v : 0.0f;
        z1g[(size_t)row * kH + col] = z;
        return z;
      }, part + kAP_db1);
}

// ---------------------------------------------------------------------------------------------
// Acting: act[agent][r] = pi_agent(obs[agent][r]).  grid (ceil(n / R), P).
template <int MT>
__global__ __launch_bounds__(kThreads) void k_act(PopDev d, const float* __restrict__ obs, int n,
                                                  float* __restrict__ act) {
  using L = Lds<MT>;
  constexpr int R = L::R;
  extern __shared__ float lds[];
  float* Xs = lds + L::x_off;
  float* bufA = lds + L::a_off;
  float* bufB = lds + L::b_off;
  float* head = lds + L::s0_off;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = blockIdx.y, r0 = blockIdx.x * R;
  const int valid = n - r0 < R ? n - r0 : R;
  const float* an = net_ptr(d, d.theta, agent, 0);
  zero_input<R>(Xs, tid);
  __syncthreads();
  load_cols<R>(Xs, 0, obs + ((size_t)agent * n + r0) * d.O, d.O, 0, d.O, valid, tid);
  __syncthreads();
  layer_relu<MT, false>(Xs, kXld, d.O, an + d.actor.w1, an + d.actor.b1, bufA, nullptr, wave, lane);
  __syncthreads();
  layer_relu<MT, true>(bufA, kLda, kH, an + d.actor.w2, an + d.actor.b2, bufB, nullptr, wave, lane);
  __syncthreads();
  thin_dot<R, true>(bufB, an + d.actor.w3, d.A, head, tid);
  __syncthreads();
  for (int e = tid; e < valid * d.A; e += kThreads) {
    const int r = e / d.A, j = e - r * d.A;
    act[((size_t)agent * n + r0 + r) * d.A + j] = tanhf(head[r * kMaxAct + j] + an[d.actor.b3 + j]);
  }
}

// ---------------------------------------------------------------------------------------------
namespace {
constexpr int kMT = 1;   // rows per workgroup = 32 kMT
}

int rows_per_workgroup() { return 32 * kMT; }

hipError_t setup_kernels() {
  const int bytes = (int)Lds<kMT>::bytes;
  hipError_t e;
  if ((e = hipFuncSetAttribute((const void*)k_target<kMT>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute((const void*)k_critic<kMT>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute((const void*)k_actor<kMT>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute((const void*)k_act<kMT>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_target(const PopDev& d, uint32_t t, hipStream_t s) {
  hipLaunchKernelGGL(k_target<kMT>, dim3(d.chunks, d.P), dim3(kThreads), Lds<kMT>::bytes, s, d, t);
  return hipGetLastError();
}
hipError_t launch_critic(const PopDev& d, uint32_t t, hipStream_t s) {
  hipLaunchKernelGGL(k_critic<kMT>, dim3(d.chunks, 2 * d.P), dim3(kThreads), Lds<kMT>::bytes, s, d, t);
  return hipGetLastError();
}
hipError_t launch_actor(const PopDev& d, uint32_t t, hipStream_t s) {
  hipLaunchKernelGGL(k_actor<kMT>, dim3(d.chunks, d.P), dim3(kThreads), Lds<kMT>::bytes, s, d, t);
  return hipGetLastError();
}
hipError_t launch_act(const PopDev& d, const float* obs, int n, float* act, hipStream_t s) {
  const int R = 32 * kMT;
  hipLaunchKernelGGL(k_act<kMT>, dim3((n + R - 1) / R, d.P), dim3(kThreads), Lds<kMT>::bytes, s, d, obs, n, act);
  return hipGetLastError();
}

}  // namespace pop
