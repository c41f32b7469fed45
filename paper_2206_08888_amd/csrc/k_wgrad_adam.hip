// Weight gradients contracted over the full batch, with the Adam update and the
// Polyak target update applied in the epilogue (Sec. 1 of the paper: compute a
// loss, differentiate it, apply a variant of SGD; Sec. 4.1: standard TD3
// hyperparametrization, i.e. Adam and soft target updates).
//
// The gradient of a weight matrix is dW = X^T dZ with the batch as the
// contraction index.  A workgroup walks the batch in stages of 32 rows: the
// slices of X and dZ it needs (written by the chain kernels) are fetched with
// coalesced 16-byte loads into registers one stage ahead, parked in a
// double-buffered LDS tile, and each wavefront feeds its 32x32 MFMA tile of dW
// from there.  The wavefront then updates exactly the parameters of its tile:
//     m <- b1 m + (1 - b1) g ;  v <- b2 v + (1 - b2) g^2
//     theta <- theta - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
// (the two bias corrections enter as reciprocals computed once per workgroup in
// double; the final quotient uses the hardware reciprocal, 1 ulp)
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
  float lr, b1, b2, eps, inv_c1, inv_c2, tau;
  int polyak, record;
};

struct AdamRegs { float th, m, v, tg; };

// one LDS stage: a slice of X (32 rows x up to 64 columns) and of dZ (32 rows x up to 128 columns)
constexpr int kStageA = 32 * 64, kStageZ = 32 * 128, kStageFloats = kStageA + kStageZ;

// b^n in double by repeated squaring (at most 64 roundings: far below fp32 resolution)
__device__ inline double ipow(double b, uint32_t n) {
  double r = 1.0;
  for (; n; n >>= 1) {
    if (n & 1u) r *= b;
    b *= b;
  }
  return r;
}

__device__ inline AdamRegs adam_load(const Adam& a, uint32_t i, const float* __restrict__ th, const float* __restrict__ m,
                                     const float* __restrict__ v, const float* __restrict__ tg) {
  AdamRegs r;
  r.th = th[i]; r.m = m[i]; r.v = v[i];
  r.tg = a.polyak ? tg[i] : 0.0f;
  return r;
}

__device__ inline void adam_store(const Adam& a, const AdamRegs& r, float g, uint32_t i, float* __restrict__ th,
                                  float* __restrict__ m, float* __restrict__ v, float* __restrict__ tg,
                                  float* __restrict__ gr) {
  const float mm = a.b1 * r.m + (1.0f - a.b1) * g;
  const float vv = a.b2 * r.v + (1.0f - a.b2) * (g * g);
  m[i] = mm;
  v[i] = vv;
  const float denom = __builtin_amdgcn_sqrtf(vv * a.inv_c2) + a.eps;
  const float tn = r.th - a.lr * (mm * a.inv_c1) * __builtin_amdgcn_rcpf(denom);
  th[i] = tn;
  if (a.polyak) tg[i] = (1.0f - a.tau) * r.tg + a.tau * tn;
  if (a.record) gr[i] = g;
}

// One block of a weight matrix: WIDE = a 64x64 block of W2 (wavefront tiles 2x2), else a
// 32x128 block of layer-1 weights (wavefront tiles 1x4, rows >= M masked).
//   x: [B][ldx] layer input, z: [B][256] pre-activation gradient, both global;
//   (m0w, n0w): block origin inside the weight matrix; base: offset of that matrix in the net.
template <bool WIDE>
__device__ inline void weight_block(const Adam& adam, const float* __restrict__ x, int ldx, int M, int m0w,
                                    const float* __restrict__ z, int n0w, uint32_t base, int B, float* stage_lds,
                                    float* __restrict__ th, float* __restrict__ mo, float* __restrict__ ve,
                                    float* __restrict__ tg, float* __restrict__ gr, int tid) {
  constexpr int as = WIDE ? 64 : 32, zs = WIDE ? 64 : 128;
  const int wave = tid >> 6, lane = tid & 63;
  const int ma = WIDE ? 32 * (wave >> 1) : 0;
  const int na = WIDE ? 32 * (wave & 1) : 32 * wave;
  const int m0 = m0w + ma, n0 = n0w + na;
  const int half = lane >> 5, l32 = lane & 31;

  // global -> register staging of one stage (32 batch rows)
  f32x4 ra[2], rz[4];
  float rs[4];
  auto fetch = [&](int b0) {
    if (WIDE) {
      const int r = tid >> 4, c4 = tid & 15;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        ra[i] = *reinterpret_cast<const f32x4*>(x + (uint32_t)((b0 + r + 16 * i) * kH + m0w + 4 * c4));
        rz[i] = *reinterpret_cast<const f32x4*>(z + (uint32_t)((b0 + r + 16 * i) * kH + n0w + 4 * c4));
      }
    } else {
      const int r = tid >> 5, c = tid & 31;
      const bool ok = (m0w + c) < M;
      const int cc = ok ? m0w + c : M - 1;           // always a valid column: the load needs no branch
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float xv = x[(uint32_t)((b0 + r + 8 * i) * ldx + cc)];
        rs[i] = ok ? xv : 0.0f;
        rz[i] = *reinterpret_cast<const f32x4*>(z + (uint32_t)((b0 + r + 8 * i) * kH + n0w + 4 * c));
      }
    }
  };
  auto park = [&](float* Al, float* Zl) {
    if (WIDE) {
      const int r = tid >> 4, c4 = tid & 15;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        *reinterpret_cast<f32x4*>(&Al[(r + 16 * i) * as + 4 * c4]) = ra[i];
        *reinterpret_cast<f32x4*>(&Zl[(r + 16 * i) * zs + 4 * c4]) = rz[i];
      }
    } else {
      const int r = tid >> 5, c = tid & 31;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        Al[(r + 8 * i) * as + c] = rs[i];
        *reinterpret_cast<f32x4*>(&Zl[(r + 8 * i) * zs + 4 * c]) = rz[i];
      }
    }
  };
  // flat offset of accumulator element 0 of this lane (row m0 + 4 half; for a layer-1 block that
  // row may be beyond M: then no element of this lane with a valid row exists below it either)
  const uint32_t elem0 = base + (uint32_t)((m0 + 4 * half) * kH + n0 + l32);
  AdamRegs regs[16];
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  const int stages = B / 32;
  fetch(0);
  park(stage_lds, stage_lds + kStageA);
  __syncthreads();
#pragma unroll 1
  for (int st = 0; st < stages; ++st) {
    const float* Al = stage_lds + (st & 1) * kStageFloats + half * as + ma + l32;
    const float* Zl = stage_lds + (st & 1) * kStageFloats + kStageA + half * zs + na + l32;
    if (st + 1 < stages) {
      fetch(32 * (st + 1));
    } else {                                       // last stage: start the epilogue's loads instead
      uint32_t e0 = elem0;
      asm volatile("" : "+v"(e0));                 // keeps the 64 addresses from being hoisted out of the loop
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const bool ok = WIDE || (m0 + acc_row(v, lane)) < M;
        regs[v] = adam_load(adam, ok ? e0 + (uint32_t)((8 * (v >> 2) + (v & 3)) * kH) : e0, th, mo, ve, tg);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    float fa[16], fz[16];
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
      fa[ks] = Al[2 * ks * as];
      fz[ks] = Zl[2 * ks * zs];
    }
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) acc = mfma32(fa[ks], fz[ks], acc);
    __builtin_amdgcn_sched_barrier(0);
    if (st + 1 < stages) {
      float* An = stage_lds + ((st + 1) & 1) * kStageFloats;
      park(An, An + kStageA);
    }
    __syncthreads();
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    if (WIDE || (m0 + acc_row(v, lane)) < M)
      adam_store(adam, regs[v], acc[v], elem0 + (uint32_t)((8 * (v >> 2) + (v & 3)) * kH), th, mo, ve, tg, gr);
    if ((v & 3) == 3) __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace

__global__ __launch_bounds__(kThreads) void k_wgrad_adam(PopDev d, uint32_t t, int actor_phase, int main_blocks,
                                                          int roles, int prefetch) {
  __shared__ Adam sh_adam;
  __shared__ __attribute__((aligned(16))) float stage_lds[2 * kStageFloats];
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
    a.inv_c1 = (float)(1.0 / (1.0 - ipow((double)hp.b1, count)));
    a.inv_c2 = (float)(1.0 / (1.0 - ipow((double)hp.b2, count)));
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
    const size_t o = (size_t)unit * d.B * kH;        // unit = agent (actor) or network (critics)
    if (role < 16) {
      weight_block<true>(adam, (actor_phase ? d.aH1 : d.cH1) + o, kH, kH, 64 * (role >> 2),
                         (actor_phase ? d.adZ2 : d.cdZ2) + o, 64 * (role & 3), (uint32_t)L.w2, d.B, stage_lds,
                         th, mo, ve, tg, gr, tid);
    } else {
      const int q = role - 16;                       // layer-1 input = leading columns of the batch rows
      weight_block<false>(adam, batch_rows(d, t, agent), d.row, L.in, 32 * (q >> 1),
                          (actor_phase ? d.adZ1 : d.cdZ1) + o, 128 * (q & 1), (uint32_t)L.w1, d.B, stage_lds,
                          th, mo, ve, tg, gr, tid);
    }
  } else {
    // small tensors from per-chunk partial sums; thread c owns hidden unit c
    const int c = tid;
    const int out = L.out;
    float gb1 = 0.0f, gb2 = 0.0f, gw3[kMaxAct], gb3 = 0.0f, loss = 0.0f;
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j) gw3[j] = 0.0f;
#pragma unroll 1
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
    auto upd = [&](float g, uint32_t i) { adam_store(adam, adam_load(adam, i, th, mo, ve, tg), g, i, th, mo, ve, tg, gr); };
    upd(gb1, (uint32_t)(L.b1 + c));
    upd(gb2, (uint32_t)(L.b2 + c));
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j)
      if (j < out) upd(gw3[j], (uint32_t)(L.w3 + c * out + j));
    if (c < out) upd(gb3, (uint32_t)(L.b3 + c));
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
