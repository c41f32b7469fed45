// Initial parameters (Sec. 4.1 of the paper: every replica starts from its own
// random weights).  Weight e (row-major flat index in [in][out]) of layer l of
// online network n is (2u - 1) * limit with u = top 24 bits of word e of the
// agent's stream 4, sub-stream 16 n + l; limit = sqrt(6 / (fan_in + fan_out))
// comes from the host.  2u - 1 is exact in fp32 and the product rounds once,
// so the values are reproducible bit for bit on any IEEE machine.  Biases,
// Adam moments and padding are zeroed by the host before this kernel runs;
// targets receive the same values as the online networks.
#include <algorithm>
#include "launch.h"
#include "rng.h"

namespace pop {

__global__ __launch_bounds__(256) void k_init(PopDev d, InitLimits lim) {
  // grid: (ceil(max tensor / 256), 9 tensors, P)
  const int agent = blockIdx.z;
  const int net = blockIdx.y / 3, layer = blockIdx.y % 3;
  if (d.share > 1 && net >= 1 && agent != 0) return;  // shared critics: the one pair is agent 0's
  const NetLayout& L = net == 0 ? d.actor : d.critic;
  const int fan_in = layer == 0 ? L.in : kH;
  const int fan_out = layer == 2 ? L.out : kH;
  const int off = layer == 0 ? L.w1 : (layer == 1 ? L.w2 : L.w3);
  const float limit = net == 0 ? lim.actor[layer] : lim.critic[layer];
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= fan_in * fan_out) return;
  const HpDev hp = d.hp[agent];
  const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, (uint32_t)(e >> 2), 0u, kStreamInit, (uint32_t)(16 * net + layer));
  const float u = (float)(pick(blk, (uint32_t)e & 3u) >> 8) * 5.9604644775390625e-8f;
  const float centred = 2.0f * u - 1.0f;          // exact
  const float w = __fmul_rn(centred, limit);      // a single rounding, never fused
  net_ptr(d, d.theta, agent, net)[off + e] = w;
  net_ptr(d, d.target, agent, net)[off + e] = w;
}

hipError_t launch_init(const PopDev& d, const InitLimits& lim, hipStream_t s) {
  const int biggest = kH * std::max(kH, std::max(d.D, d.actor.out));   // largest weight matrix of the three networks
  dim3 grid((biggest + 255) / 256, 9, d.P);
  hipLaunchKernelGGL(k_init, grid, dim3(256), 0, s, d, lim);
  return hipGetLastError();
}

}  // namespace pop
