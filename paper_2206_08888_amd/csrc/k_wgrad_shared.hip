// Weight gradients of the shared critics (Sec. 4.2 of the paper: one critic pair for the whole population, the
// critic loss averaged over the agents).  The gradient of a critic matrix is sum_i X_i^T dZ_i over the P agents'
// batches (the 1/P sits in the chain's error seed): a contraction over P * 256 rows, split over `groups` agent
// groups so that the chip stays full.
//   k_shared_partial: workgroup (network, group g, role) accumulates the role's 32 x 128 tile of dW (or, last
//     role, the small tensors b1, b2, W3, b3 and the loss) over the agents g, g + groups, ... and writes it to
//     spart[network][g], an array laid out like the network's parameter block;
//   k_shared_adam: one thread per parameter adds the group partials in a fixed order and applies Adam and, on
//     delayed steps, Polyak to the one critic pair (agent 0's blocks), with agent 0's hyperparameters.
// No atomics: the result does not depend on scheduling.
#include "gather.h"
#include "launch.h"
#include "wgrad.h"

namespace pop {

// Blocks at and beyond main_blocks gather the replay rows of step t + 1 into the other half of the batch buffer
// (prefetch != 0), as the tail of the per-agent weight-gradient launch does.
__global__ __launch_bounds__(kThreads, 3) void k_shared_partial(PopDev d, uint32_t t, int roles, int main_blocks, int prefetch) {
  __shared__ __attribute__((aligned(16))) float xt_lds[32 * kLda];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  if ((int)blockIdx.x >= main_blocks) {
    if (prefetch) {
      const int g = blockIdx.x - main_blocks, per = gather_blocks_per_agent(d);
      gather_block(d, t + 1u, g / per, g % per, tid);
    }
    return;
  }
  // block -> (network, group, role): the roles of one (network, group) share an XCD -- the eight row slabs of a
  // weight matrix read the same dZ tiles of the group's agents, and find them in that XCD's L2 (numbered plainly,
  // round-robin over the XCDs, every XCD fetched its own copy: 351 MB per launch at P = 80 against 126 MB of activations)
  int ng, role;
  if (!decode_block(blockIdx.x, 2 * d.groups, roles, ng, role)) return;
  const int net = ng % 2, g = ng / 2;
  const NetLayout& L = d.critic;
  float* out = d.spart + ((size_t)net * d.groups + g) * L.padded;
  const int n1 = (L.in + 31) / 32;
  const int chunks = d.B / d.rows_c;
  if (role < 16 + 2 * n1) {
    const bool w2 = role < 16;
    const int n0 = 128 * (role & 1), m0 = 32 * ((w2 ? role : role - 16) >> 1);
    const int M = w2 ? kH : L.in, ldx = w2 ? kH : d.row;
    Acc<1, 1> acc;
    acc.zero();
    for (int agent = g; agent < d.P; agent += d.groups) {
      const size_t o = (size_t)(2 * agent + net) * d.B * kH;
      const float* x = w2 ? d.cH1 + o : batch_rows(d, t, agent);
      const float* z = (w2 ? d.cdZ2 : d.cdZ1) + o + n0;
      XSlice xsl;
      xsl.load(x, ldx, M, m0, wave, lane);
      WeightBlock<1, false, 1> z0;
      z0.load(z, 0, wave, lane);
      __syncthreads();                               // the previous agent's product has read the slice
      xsl.store(xt_lds, ldx, M, m0, wave, lane);
      __syncthreads();
      gemm256_unrolled<1, false, 1, 4, true>(xt_lds, kLda, z, z0, wave, lane, acc, NoTail());
    }
    const int half = lane >> 5, l32 = lane & 31;
    const uint32_t elem0 = (uint32_t)((w2 ? L.w2 : L.w1) + (m0 + 4 * half) * kH + n0 + 32 * wave + l32);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if ((m0 + acc_row(v, lane)) < M) out[elem0 + (uint32_t)((8 * (v >> 2) + (v & 3)) * kH)] = acc.t[0][0][v];
  } else {
    const int c = tid;
    float gb1 = 0.0f, gb2 = 0.0f, gw3 = 0.0f, gb3 = 0.0f, loss = 0.0f;
    for (int agent = g; agent < d.P; agent += d.groups) {
#pragma unroll 4
      for (int ch = 0; ch < chunks; ++ch) {
        const float* p = d.cpart + ((size_t)(2 * agent + net) * d.cstride + ch) * kCPart;
        const float t1 = p[kCP_db1 + c], t2 = p[kCP_db2 + c], tw = p[kCP_dW3 + c], t3 = p[kCP_db3], tl = p[kCP_loss];
        gb1 += t1; gb2 += t2; gw3 += tw; gb3 += t3; loss += tl;
      }
    }
    out[L.b1 + c] = gb1;
    out[L.b2 + c] = gb2;
    out[L.w3 + c] = gw3;
    if (c == 0) { out[L.b3] = gb3; d.sloss[net * d.groups + g] = loss; }
  }
}

__global__ __launch_bounds__(256) void k_shared_adam(PopDev d, uint32_t t) {
  // grid: (ceil(critic.size / 256), 2 networks)
  const int net = 1 + blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const NetLayout& L = d.critic;
  const HpDev hp = d.hp[0];
  if (e == 0) {                                      // the loss of the population, reported for every agent
    float loss = 0.0f;
    for (int g = 0; g < d.groups; ++g) loss += d.sloss[(net - 1) * d.groups + g];
    for (int a = 0; a < d.P; ++a) d.losses[(size_t)a * 4 + (net - 1)] = loss;
  }
  __shared__ Adam sh;
  if (threadIdx.x == 0) {                            // the step's constants, once per workgroup (double arithmetic)
    Adam a;
    const uint32_t count = t + 1u;
    a.lr = hp.lr_critic; a.b1 = hp.b1; a.b2 = hp.b2; a.eps = hp.eps;
    a.inv_c1 = (float)(1.0 / (1.0 - ipow((double)hp.b1, count)));
    a.inv_c2 = (float)(1.0 / (1.0 - ipow((double)hp.b2, count)));
    a.tau = hp.tau;
    a.polyak = (t % (uint32_t)hp.policy_delay) == 0u ? 1 : 0;
    a.record = d.record_grads;
    sh = a;
  }
  __syncthreads();
  if (e >= L.size) return;
  const Adam a = sh;
  float g = 0.0f;
  const float* sp = d.spart + (size_t)(net - 1) * d.groups * L.padded + e;
  for (int k = 0; k < d.groups; ++k) g += sp[(size_t)k * L.padded];
  float* th = net_ptr(d, d.theta, 0, net);
  float* mo = net_ptr(d, d.m, 0, net);
  float* ve = net_ptr(d, d.v, 0, net);
  float* tg = net_ptr(d, d.target, 0, net);
  float* gr = net_ptr(d, d.grad, 0, net);
  AdamRegs r;
  r.th = th[e]; r.m = mo[e]; r.v = ve[e];
  r.tg = a.polyak ? tg[e] : 0.0f;
  adam_store<false>(a, r, g, (uint32_t)e, th, mo, ve, tg, gr);
}

hipError_t launch_wgrad_shared(const PopDev& d, uint32_t t, int prefetch_next, hipStream_t s) {
  const int roles = 16 + 2 * ((d.critic.in + 31) / 32) + 1;
  const int main_blocks = 2 * d.groups * roles, extra = prefetch_next ? d.P * gather_blocks_per_agent(d) : 0;
  hipLaunchKernelGGL(k_shared_partial, dim3(main_blocks + extra), dim3(kThreads), 0, s, d, t, roles, main_blocks, prefetch_next);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_shared_adam, dim3((d.critic.size + 255) / 256, 2), dim3(256), 0, s, d, t);
  return hipGetLastError();
}

}  // namespace pop
