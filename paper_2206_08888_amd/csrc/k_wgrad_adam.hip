// Weight gradients contracted over the full batch, with the Adam update and the
// Polyak target update applied in the epilogue (Sec. 1 of the paper: compute a
// loss, differentiate it, apply a variant of SGD; Sec. 4.1: standard TD3
// hyperparametrization, i.e. Adam and soft target updates).
//
// The gradient of a weight matrix is dW = X^T dZ with the batch as the
// contraction index.  Each wavefront computes one 32x32 tile of dW on the MFMA
// unit reading X and dZ (written by the chain kernels) straight from global
// memory, and then updates exactly the parameters of its tile:
//     m <- b1 m + (1 - b1) g ;  v <- b2 v + (1 - b2) g^2
//     theta <- theta - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
//     theta' <- (1 - tau) theta' + tau theta        (only on delayed steps)
// so a gradient never makes a round trip through HBM.  The parameters, moments
// and targets of the tile are requested before the product starts, so their
// HBM latency is hidden behind the MFMA work.  The small tensors (biases, head
// weights) arrive as per-chunk partial sums and are reduced and updated by one
// extra workgroup per network.
//
// 1-D grid, decoded so that the roles of one network share an XCD (its L2 then
// serves the re-reads of X and dZ).  Roles of one network:
//   [0, 16)            64x64 blocks of W2 (4 wavefronts, one 32x32 tile each)
//   [16, 16 + n1)      layer-1 weights: 32 rows x 128 columns per workgroup
//   16 + n1            b1, b2, W3, b3 and the loss value
// Blocks past the last network gather the replay rows of step t + 1 into the
// other half of the double-buffered batch (App. A of the paper: the next
// batches are fetched while the current update runs).
#include "gather.h"
#include "launch.h"
#include "mfma_tiles.h"

namespace pop {

namespace {

struct Adam {
  float lr, b1, b2, eps, c1, c2, tau;
  int polyak, record;
};

struct AdamRegs { float th, m, v, tg; };

__device__ inline AdamRegs adam_load(const Adam& a, size_t i, const float* __restrict__ th, const float* __restrict__ m,
                                     const float* __restrict__ v, const float* __restrict__ tg) {
  AdamRegs r;
  r.th = th[i]; r.m = m[i]; r.v = v[i];
  r.tg = a.polyak ? tg[i] : 0.0f;
  return r;
}

__device__ inline void adam_store(const Adam& a, const AdamRegs& r, float g, size_t i, float* __restrict__ th,
                                  float* __restrict__ m, float* __restrict__ v, float* __restrict__ tg,
                                  float* __restrict__ gr) {
  const float mm = a.b1 * r.m + (1.0f - a.b1) * g;
  const float vv = a.b2 * r.v + (1.0f - a.b2) * (g * g);
  m[i] = mm;
  v[i] = vv;
  const float tn = r.th - a.lr * (mm / a.c1) / (sqrtf(vv / a.c2) + a.eps);
  th[i] = tn;
  if (a.polyak) tg[i] = (1.0f - a.tau) * r.tg + a.tau * tn;
  if (a.record) gr[i] = g;
}

}  // namespace

__global__ __launch_bounds__(kThreads) void k_wgrad_adam(PopDev d, uint32_t t, int actor_phase, int main_blocks,
                                                          int roles, int prefetch) {
  __shared__ Adam sh_adam;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  if ((int)blockIdx.x >= main_blocks) {              // gather role: rows of the next step
    if (prefetch) {
      const int g = blockIdx.x - main_blocks, per = gather_blocks_per_agent(d);
      gather_element(d, t + 1u, g / per, (g % per) * 256 + tid);
    }
    return;
  }
  int unit, role;
  if (!decode_block(blockIdx.x, actor_phase ? d.P : 2 * d.P, roles, unit, role)) return;
  const int agent = actor_phase ? unit : unit >> 1;
  const int net = actor_phase ? 0 : 1 + (unit & 1);
  const HpDev hp = d.hp[agent];
  const uint32_t delay = (uint32_t)hp.policy_delay;
  const bool delayed_step = (t % delay) == 0u;
  if (actor_phase && !delayed_step) return;

  if (tid == 0) {
    Adam a;
    const uint32_t count = actor_phase ? t / delay + 1u : t + 1u;   // 1-based Adam step
    a.lr = actor_phase ? hp.lr_actor : hp.lr_critic;
    a.b1 = hp.b1; a.b2 = hp.b2; a.eps = hp.eps;
    a.c1 = (float)(1.0 - pow((double)hp.b1, (double)count));
    a.c2 = (float)(1.0 - pow((double)hp.b2, (double)count));
    a.tau = hp.tau;
    a.polyak = delayed_step ? 1 : 0;
    a.record = d.record_grads;
    sh_adam = a;
  }
  __syncthreads();
  const Adam adam = sh_adam;

  const NetLayout& L = actor_phase ? d.actor : d.critic;
  float* th = net_ptr(d, d.theta, agent, net);
  float* mo = net_ptr(d, d.m, agent, net);
  float* ve = net_ptr(d, d.v, agent, net);
  float* tg = net_ptr(d, d.target, agent, net);
  float* gr = net_ptr(d, d.grad, agent, net);

  const int n1 = 2 * ((L.in + 31) / 32);
  if (role < 16 + n1) {
    // operands of the product and the tile this wavefront owns
    const float *x, *z;
    int ldx, M, m0, n0;
    size_t base;
    const size_t o = (size_t)unit * d.B * kH;        // unit = agent (actor) or network (critics)
    if (role < 16) {
      x = (actor_phase ? d.aH1 : d.cH1) + o; ldx = kH; M = kH;
      z = (actor_phase ? d.adZ2 : d.cdZ2) + o;
      m0 = 64 * (role >> 2) + 32 * (wave >> 1);
      n0 = 64 * (role & 3) + 32 * (wave & 1);
      base = (size_t)L.w2;
    } else {
      const int q = role - 16;
      x = batch_rows(d, t, agent); ldx = d.row; M = L.in;   // layer-1 input = leading columns of the batch rows
      z = (actor_phase ? d.adZ1 : d.cdZ1) + o;
      m0 = 32 * (q >> 1);
      n0 = 128 * (q & 1) + 32 * wave;
      base = (size_t)L.w1;
    }
    AdamRegs regs[16];
    const f32x16 acc = wgrad_tile(x, ldx, M, m0, z, kH, n0, d.B, lane, [&]() {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int mrow = m0 + acc_row(v, lane);
        const size_t i = base + (size_t)(mrow < M ? mrow : 0) * kH + n0 + (lane & 31);
        regs[v] = adam_load(adam, i, th, mo, ve, tg);
      }
    });
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int mrow = m0 + acc_row(v, lane);
      if (mrow < M) {
        const size_t i = base + (size_t)mrow * kH + n0 + (lane & 31);
        adam_store(adam, regs[v], acc[v], i, th, mo, ve, tg, gr);
      }
    }
  } else {
    // small tensors from per-chunk partial sums; thread c owns hidden unit c
    const int c = tid;
    const int out = L.out;
    float gb1 = 0.0f, gb2 = 0.0f, gw3[kMaxAct], gb3 = 0.0f, loss = 0.0f;
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j) gw3[j] = 0.0f;
    for (int ch = 0; ch < d.chunks; ++ch) {
      if (actor_phase) {
        const float* p = d.apart + ((size_t)agent * d.chunks + ch) * kAPart;
        gb1 += p[kAP_db1 + c];
        gb2 += p[kAP_db2 + c];
#pragma unroll
        for (int j = 0; j < kMaxAct; ++j)
          if (j < out) gw3[j] += p[kAP_dW3 + c * out + j];
        if (c < out) gb3 += p[kAP_db3 + c];
        if (c == 0) loss += p[kAP_loss];
      } else {
        const float* p = d.cpart + ((size_t)unit * d.chunks + ch) * kCPart;
        gb1 += p[kCP_db1 + c];
        gb2 += p[kCP_db2 + c];
        gw3[0] += p[kCP_dW3 + c];
        if (c == 0) { gb3 += p[kCP_db3]; loss += p[kCP_loss]; }
      }
    }
    auto upd = [&](float g, size_t i) { adam_store(adam, adam_load(adam, i, th, mo, ve, tg), g, i, th, mo, ve, tg, gr); };
    upd(gb1, (size_t)L.b1 + c);
    upd(gb2, (size_t)L.b2 + c);
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j)
      if (j < out) upd(gw3[j], (size_t)L.w3 + (size_t)c * out + j);
    if (c < out) upd(gb3, (size_t)L.b3 + c);
    if (c == 0) {
      // critic loss = sum over the twins; the two critic workgroups of an agent write
      // their halves to separate slots and the reader adds them
      if (actor_phase) d.losses[(size_t)agent * 4 + 2] = loss;
      else d.losses[(size_t)agent * 4 + (net - 1)] = loss;
    }
  }
}

hipError_t launch_wgrad_adam(const PopDev& d, uint32_t t, int actor_phase, int prefetch_next, hipStream_t s) {
  const NetLayout& L = actor_phase ? d.actor : d.critic;
  const int roles = 16 + 2 * ((L.in + 31) / 32) + 1;
  const int main_blocks = xcd_grid(actor_phase ? d.P : 2 * d.P, roles);
  const int extra = prefetch_next ? d.P * gather_blocks_per_agent(d) : 0;
  hipLaunchKernelGGL(k_wgrad_adam, dim3(main_blocks + extra), dim3(kThreads), 0, s, d, t, actor_phase, main_blocks,
                     roles, prefetch_next);
  return hipGetLastError();
}

}  // namespace pop
