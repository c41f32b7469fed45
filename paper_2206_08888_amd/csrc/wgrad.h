// Weight gradients contracted over the full batch, with the Adam update and the
// Polyak target update applied in the epilogue (Sec. 1 of the paper: compute a
// loss, differentiate it, apply a variant of SGD; Sec. 4.1: standard TD3
// hyperparametrization, i.e. Adam and soft target updates).
//
// The gradient of a weight matrix is dW = X^T dZ with the batch as the
// contraction index.  A workgroup owns a tile of 32 rows x 128 columns of dW
// (one 32-column accumulator tile per wavefront): it transposes its 32 columns
// of X (written by the chains) into an LDS tile [32][batch] and runs a
// pipelined 256-deep MFMA product with dZ streamed from global memory in the
// role of the weights.  Each wavefront then updates exactly the parameters it
// holds in its accumulators:
//     m <- b1 m + (1 - b1) g ;  v <- b2 v + (1 - b2) g^2
//     theta <- theta - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
//     theta' <- (1 - tau) theta' + tau theta        (only on delayed steps)
// (the two bias corrections enter as reciprocals computed once per workgroup in
// double; the final quotient uses the hardware reciprocal, 1 ulp)
// so a gradient never makes a round trip through HBM.  Parameters, moments and
// targets of the tile do not depend on the product: they are requested right
// after the product's own first operands and arrive under it.  The small
// tensors (biases, head weights) arrive as per-chunk partial sums and are
// reduced and updated by one extra workgroup per network, which for SAC also
// takes the Adam step of the temperature.
//
// Roles of one network (n1 = ceil(fan-in of layer 1 / 32)):
//   [0, 16)              tiles of W2: 32-row slab role / 2, column half role % 2
//   [16, 16 + 2 n1)      tiles of the layer-1 weights (rows >= fan-in masked)
//   16 + 2 n1            b1, b2, W3, b3, the loss value (and log alpha)
// The kernels decode block indices so that the roles of one network share an
// XCD (its L2 then serves the re-reads of dZ).  The batch size must be 256 for
// the tile product (its contraction depth is fixed).
#pragma once
#include "chains.h"

namespace pop {

struct Adam {
  float lr, b1, b2, eps, inv_c1, inv_c2, tau;
  int polyak, record;
  int through;   // another workgroup of this launch reads the updated parameters (critic 1 ahead of an actor chain)
};

struct AdamRegs { float th, m, v, tg; };

// b^n in double by repeated squaring (at most 64 roundings: far below fp32 resolution)
__device__ inline double ipow(double b, uint32_t n) {
  double r = 1.0;
  for (; n; n >>= 1) {
    if (n & 1u) r *= b;
    b *= b;
  }
  return r;
}

// THROUGH: the launch hands results from workgroup to workgroup; the updated parameter goes through to memory if
// this network is one whose parameters the actor chain of the same launch reads (a.through)
template <bool THROUGH = false>
__device__ inline void adam_store(const Adam& a, const AdamRegs& r, float g, uint32_t i, float* __restrict__ th,
                                  float* __restrict__ m, float* __restrict__ v, float* __restrict__ tg,
                                  float* __restrict__ gr) {
  const float mm = a.b1 * r.m + (1.0f - a.b1) * g;
  const float vv = a.b2 * r.v + (1.0f - a.b2) * (g * g);
  m[i] = mm;
  v[i] = vv;
  const float denom = __builtin_amdgcn_sqrtf(vv * a.inv_c2) + a.eps;
  const float tn = r.th - a.lr * (mm * a.inv_c1) * __builtin_amdgcn_rcpf(denom);
  if (THROUGH && a.through) put<true>(th + i, tn);
  else th[i] = tn;
  if (a.polyak) tg[i] = (1.0f - a.tau) * r.tg + a.tau * tn;
  if (a.record) gr[i] = g;
}

// Four neighbouring parameters at once (16-byte operands; the updated parameters, when another workgroup of the
// launch reads them, as two 8-byte write-through stores).
struct AdamRegs4 { f32x4 th, m, v, tg; };
template <bool THROUGH = false>
__device__ inline void adam_store4(const Adam& a, const AdamRegs4& r, const f32x4& g, uint32_t i, float* __restrict__ th,
                                   float* __restrict__ m, float* __restrict__ v, float* __restrict__ tg,
                                   float* __restrict__ gr) {
  f32x4 mm, vv, tn, tt;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    mm[e] = a.b1 * r.m[e] + (1.0f - a.b1) * g[e];
    vv[e] = a.b2 * r.v[e] + (1.0f - a.b2) * (g[e] * g[e]);
    const float denom = __builtin_amdgcn_sqrtf(vv[e] * a.inv_c2) + a.eps;
    tn[e] = r.th[e] - a.lr * (mm[e] * a.inv_c1) * __builtin_amdgcn_rcpf(denom);
    tt[e] = (1.0f - a.tau) * r.tg[e] + a.tau * tn[e];
  }
  *reinterpret_cast<f32x4*>(m + i) = mm;
  *reinterpret_cast<f32x4*>(v + i) = vv;
  if (THROUGH && a.through) {
    put2<true>(th + i, tn[0], tn[1]);
    put2<true>(th + i + 2, tn[2], tn[3]);
  } else {
    *reinterpret_cast<f32x4*>(th + i) = tn;
  }
  if (a.polyak) *reinterpret_cast<f32x4*>(tg + i) = tt;
  if (a.record) *reinterpret_cast<f32x4*>(gr + i) = g;
}

// The X slice [256 batch rows][32 columns] of a weight-gradient tile, read so that one load instruction
// covers whole 128-byte row pieces (a lane-per-row pattern touches 64 cache lines per instruction and lives
// off the L1), then written transposed into LDS as Xl[column][batch row]:
//   16-byte path (row stride a multiple of 4: a hidden layer's output): instruction i, lane l takes
//     4 columns 4 (l & 7) .. of row 64 wave + 8 i + (l >> 3);
//   else (batch rows of any stride): instruction i, lane l takes column l & 31 of row 64 wave + 2 i + (l >> 5),
//     columns at or beyond M read column 0 and are zeroed on the way into LDS.
struct XSlice {
  float xs[32];
  __device__ __forceinline__ void load(const float* __restrict__ x, int ldx, int M, int m0, int wave, int lane) {
    if ((ldx & 3) == 0) {
      const uint32_t o0 = (uint32_t)((64 * wave + (lane >> 3)) * ldx + m0 + 4 * (lane & 7)), step = (uint32_t)(8 * ldx);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(x + (o0 + (uint32_t)i * step));
        xs[4 * i] = v[0]; xs[4 * i + 1] = v[1]; xs[4 * i + 2] = v[2]; xs[4 * i + 3] = v[3];
      }
    } else {
      const int col = lane & 31;
      const uint32_t o0 = (uint32_t)((64 * wave + (lane >> 5)) * ldx + m0 + ((m0 + col) < M ? col : 0)), step = (uint32_t)(2 * ldx);
#pragma unroll
      for (int i = 0; i < 32; ++i) xs[i] = x[o0 + (uint32_t)i * step];
    }
  }
  __device__ __forceinline__ void store(float* Xl, int ldx, int M, int m0, int wave, int lane) const {
    if ((ldx & 3) == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) Xl[(4 * (lane & 7) + e) * kLda + 64 * wave + 8 * i + (lane >> 3)] = xs[4 * i + e];
    } else {
      const int col = lane & 31;
      const bool live = (m0 + col) < M;
#pragma unroll
      for (int i = 0; i < 32; ++i) Xl[col * kLda + 64 * wave + 2 * i + (lane >> 5)] = live ? xs[i] : 0.0f;
    }
  }
};

// One 32 x 128 tile of a weight matrix [M][256]: rows m0 .. m0+31 (rows >= M masked),
// columns n0 .. n0+127, 32 per wavefront.
//   x: [256][ldx] layer input, z: [256][256] pre-activation gradient, both global;
//   base: offset of the matrix inside the network's parameter block.
// The tile's parameters, moments and targets do not depend on the product, so they are
// requested first and arrive while the operands are staged and multiplied.  `setup()` fills
// `sh` (thread 0 only; a few hundred cycles of double arithmetic): it runs once the loads are
// on their way, and `sh` is read after the barrier that follows.
template <bool WAIT, bool SLIM, bool HALF, class Setup>
__device__ __forceinline__ void weight_tile(const PopDev& d, const uint32_t* wait_on, uint32_t want, const Adam* sh,
                                            Setup setup, bool polyak, const float* __restrict__ x, int ldx, int M, int m0,
                                   int n0, const float* __restrict__ z, uint32_t base, float* Xl,
                                   float* __restrict__ th, float* __restrict__ mo, float* __restrict__ ve,
                                   float* __restrict__ tg, float* __restrict__ gr, int tid) {
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31;
  POP_MARK(50);
  // The Adam step works on whole row pieces: thread `tid` owns, for q = 0 .. 3, the four parameters of row
  // (tid >> 5) + 8 q at columns 4 (tid & 31) .. of the tile -- 16-byte operands, a quarter of the load and store
  // instructions of a one-float-per-lane layout (the CU's one load path is what the tile launches queue for).
  // The product leaves the gradients in the MFMA layout; they change over through LDS (the X slice is done with).
  // HALF: the tile is 64 columns wide; wavefront pairs take the two column groups for one half of the batch each
  // (kh), the halves are summed where the gradients change layout, and a thread owns two row pieces, 16 rows apart.
  constexpr int Q = HALF ? 2 : 4, QR = HALF ? 16 : 8;
  const int cw = HALF ? (wave & 1) : wave, kh = HALF ? (wave >> 1) : 0;
  const int arow = HALF ? tid >> 4 : tid >> 5, acol = 4 * (tid & (HALF ? 15 : 31));
  const uint32_t elem0 = base + (uint32_t)((m0 + arow) * kH + n0 + acol);      // q = 0; q adds QR rows
  AdamRegs4 regs[Q];
  auto load_adam = [&]() {
#pragma unroll
    for (int q = 0; q < Q; ++q) {
      const bool ok = (m0 + arow + QR * q) < M;
      const uint32_t i = ok ? elem0 + (uint32_t)(QR * q * kH) : elem0 - (uint32_t)(arow * kH);   // else: row m0, always valid
      regs[q].th = *reinterpret_cast<const f32x4*>(th + i);
      regs[q].m = *reinterpret_cast<const f32x4*>(mo + i);
      regs[q].v = *reinterpret_cast<const f32x4*>(ve + i);
      regs[q].tg = polyak ? *reinterpret_cast<const f32x4*>(tg + i) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
  };
  XSlice xsl;
  auto load_x = [&]() { xsl.load(x, ldx, M, m0, wave, lane); };
  auto store_x = [&]() { xsl.store(Xl, ldx, M, m0, wave, lane); };
  WeightBlock<1, false, 1> z0;
  const float* zk = z + n0 + (size_t)kh * 128 * kH;   // this wavefront's rows of dZ
  if (WAIT && wait_on) {                             // x and z come from a chain of this launch
    // The counter is read before anything else is requested: a wavefront's loads come back in the order they went
    // out, so a poll issued behind the Adam operands would only return once those 64 KB have arrived from memory,
    // and x and z, which cannot be requested before it, one more trip later.  setup() runs under the poll's trip.
    uint32_t seen = 0u;
    if (tid == 0) seen = __hip_atomic_load(wait_on, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    setup();
    if (tid == 0) {
      if (seen < want) wait_count(d, wait_on, want);
      else __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
  }
  load_x();                                          // what the product needs first goes out first
  z0.load(zk, 0, cw, lane);
  __builtin_amdgcn_sched_barrier(0);
  load_adam();
  __builtin_amdgcn_sched_barrier(0);
  if (!(WAIT && wait_on)) setup();
  __builtin_amdgcn_sched_barrier(0);
  POP_MARK(51);
  store_x();
  __syncthreads();
  POP_MARK(52);
  const Adam adam = *sh;
  Acc<1, 1> acc;
  acc.zero();
  gemm256_unrolled<1, false, 1, SLIM ? 4 : 8, true, HALF ? 8 : 16>(Xl + 128 * kh, kLda, zk, z0, cw, lane, acc, NoTail());   // loads between the MFMAs: a
                                                     // block is 8 MFMAs and 8 load instructions, and these kernels run two workgroups per CU
  POP_MARK(53);
  __syncthreads();                                   // every wavefront is done with the X slice
#pragma unroll
  for (int v = 0; v < 16; ++v) Xl[acc_row(v, lane) * kLda + 32 * wave + l32] = acc.t[0][0][v];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    if ((m0 + arow + QR * q) < M) {
      f32x4 g = *reinterpret_cast<const f32x4*>(&Xl[(arow + QR * q) * kLda + acol]);
      if (HALF) g += *reinterpret_cast<const f32x4*>(&Xl[(arow + QR * q) * kLda + 64 + acol]);
      adam_store4<WAIT>(adam, regs[q], g, elem0 + (uint32_t)(QR * q * kH), th, mo, ve, tg, gr);
    }
  }
  POP_MARK(54);
}

constexpr int kSmallHeadBlock = 8;   // head columns of an actor that one small-tensor role sums and updates

// One role of the weight-gradient step of one network (unit = agent in the actor phase, else network).
// WAIT: consumers (the actor chain, for critic 1) and, if producer_in_launch, producers (the
// chain of this network) run in the same launch -- hold before the first read of chain
// output, count in at the end.
// SLIM: the register budget of three workgroups per CU (four dZ buffers, head columns eight at a time).
template <bool WAIT, bool SLIM = false, bool HALF = false>
__device__ __forceinline__ void wgrad_roles(const PopDev& d, uint32_t t, int actor_phase, int unit, int role,
                                            float* xt_lds, Adam* sh_adam, bool producer_in_launch = true) {
  const int tid = threadIdx.x;
  const int agent = actor_phase ? unit : unit >> 1;
  const int net = actor_phase ? 0 : 1 + (unit & 1);
  const HpDev hp = d.hp[agent];
  const uint32_t delay = (uint32_t)hp.policy_delay;
  const bool delayed_step = (t % delay) == 0u;
  if (actor_phase && !delayed_step) return;

  // Only critic 1, and only on a step on which its agent's actor chain follows in this launch, has a reader of its
  // updated parameters inside the launch: the others store plainly and leave without waiting for their stores to be
  // acknowledged and counting in (that wait keeps a tile's slot for a trip to memory: 5 us of the 310 us a step's critic half takes at P = 80).
  const bool feeds_actor = WAIT && !actor_phase && (unit & 1) == 0 && delayed_step;
  auto setup = [&]() {
    if (tid != 0) return;                            // read by everyone after the next barrier
    Adam a;
    // 1-based Adam step: critics count every step; the actor its own updates, i.e. the multiples of
    // its delay in [t_base, t] on top of those taken before t_base (t is one of them here)
    const uint32_t count = actor_phase ? hp.actor_base + (t / delay - (hp.t_base + delay - 1u) / delay + 1u) : t + 1u;
    a.lr = actor_phase ? hp.lr_actor : hp.lr_critic;
    a.b1 = hp.b1; a.b2 = hp.b2; a.eps = hp.eps;
    a.inv_c1 = (float)(1.0 / (1.0 - ipow((double)hp.b1, count)));
    a.inv_c2 = (float)(1.0 / (1.0 - ipow((double)hp.b2, count)));
    a.tau = hp.tau;
    a.polyak = (delayed_step && !(actor_phase && d.algo == 1)) ? 1 : 0;   // SAC has no target actor
    a.record = d.record_grads;
    a.through = feeds_actor ? 1 : 0;
    *sh_adam = a;
  };

  const NetLayout& L = actor_phase ? d.actor : d.critic;
  float* th = net_ptr(d, d.theta, agent, net);
  float* mo = net_ptr(d, d.m, agent, net);
  float* ve = net_ptr(d, d.v, agent, net);
  float* tg = net_ptr(d, d.target, agent, net);
  float* gr = net_ptr(d, d.grad, agent, net);

  // WAIT: the chain that produces this network's activations runs in the same launch
  const uint32_t* wait_on = !producer_in_launch ? nullptr
                            : actor_phase       ? d.done_a + parity_base(d, t, d.P) + agent
                                                : d.done_c + parity_base(d, t, 2 * d.P) + unit;
  const int chunks = d.B / (actor_phase ? d.rows_a : (unit & 1) ? d.rows_c : d.rows_c1);   // row chunks of the chain that feeds this network
  const int n1 = (L.in + 31) / 32;
  const int tiles = 16 + 2 * n1;                      // 32 x 128 tiles; HALF: each as two roles, 64 columns wide
  if (role < (HALF ? 2 * tiles : tiles)) {
    const size_t o = (size_t)unit * d.B * kH;        // unit = agent (actor) or network (critics)
    const int half = HALF ? (role & 1) : 0;
    if (HALF) role >>= 1;
    const int n0 = 128 * (role & 1) + 64 * half;
    const bool w2 = role < 16;                       // else layer 1, whose input is the leading columns of the batch rows
    const float* x = w2 ? (actor_phase ? d.aH1 : d.cH1) + o : batch_rows(d, t, agent);
    const float* z = (w2 ? (actor_phase ? d.adZ2 : d.cdZ2) : (actor_phase ? d.adZ1 : d.cdZ1)) + o;
    weight_tile<WAIT, SLIM, HALF>(d, wait_on, (uint32_t)chunks, sh_adam, setup, delayed_step && !(actor_phase && d.algo == 1), x, w2 ? kH : d.row, w2 ? kH : L.in, 32 * ((w2 ? role : role - 16) >> 1), n0, z,
                (uint32_t)(w2 ? L.w2 : L.w1), xt_lds, th, mo, ve, tg, gr, tid);
  } else {
    // Small tensors from per-chunk partial sums; thread c owns hidden unit c.  Role `small` = 0: the hidden biases,
    // and for a critic its one head column, head bias and loss, for an actor its head bias and loss (SAC: the
    // temperature).  An actor's head columns are roles of their own, kSmallHeadBlock columns each (small - 1 =
    // block): as one role they made the longest workgroup of the launch by far (16 chunk records walked once per
    // block of columns, a trip to memory every few records: 17 us at P = 10 where a tile takes 8).
    // The Adam operands are requested first: they depend on nothing and arrive while the partial sums are read.
    constexpr int HB = kSmallHeadBlock;
    const int small = role - (HALF ? 2 * tiles : tiles);
    const int c = tid;
    const int out = L.out;
    POP_MARK(55);
    const bool polyak = delayed_step && !(actor_phase && d.algo == 1);
    auto ld = [&](uint32_t i) {
      AdamRegs r;
      r.th = th[i]; r.m = mo[i]; r.v = ve[i];
      r.tg = polyak ? tg[i] : 0.0f;
      return r;
    };
    if (small > 0) {                                  // actor: head columns [j0, j0 + HB)
      const int j0 = (small - 1) * HB;
      const uint32_t i_w3 = (uint32_t)(L.w3 + c * out);
      AdamRegs r_w3[HB];
#pragma unroll
      for (int j = 0; j < HB; ++j) r_w3[j] = ld(i_w3 + (uint32_t)(j0 + j < out ? j0 + j : 0));
      setup();
      if (WAIT && wait_on && tid == 0) wait_count(d, wait_on, (uint32_t)chunks);
      __syncthreads();
      const Adam adam = *sh_adam;
      float gw3[HB];
#pragma unroll
      for (int j = 0; j < HB; ++j) gw3[j] = 0.0f;
      // every load goes out unconditionally (columns beyond `out` re-read column 0 and are dropped at the store),
      // so that the loads of several chunks are in flight together
#pragma unroll 4
      for (int ch = 0; ch < chunks; ++ch) {
        const float* p = d.apart + ((size_t)agent * chunks + ch) * kAPart + kAP_dW3 + c;
        float tw[HB];
#pragma unroll
        for (int j = 0; j < HB; ++j) tw[j] = p[(j0 + j < out ? j0 + j : 0) * kH];
#pragma unroll
        for (int j = 0; j < HB; ++j) gw3[j] += tw[j];
      }
#pragma unroll
      for (int j = 0; j < HB; ++j)
        if (j0 + j < out) adam_store<WAIT>(adam, r_w3[j], gw3[j], i_w3 + (uint32_t)(j0 + j), th, mo, ve, tg, gr);
      POP_MARK(58);
      return;                                         // (actor roles do not count themselves in for anybody)
    }
    const uint32_t i_b1 = (uint32_t)(L.b1 + c), i_b2 = (uint32_t)(L.b2 + c), i_w3 = (uint32_t)(L.w3 + c * out),
                   i_b3 = (uint32_t)(L.b3 + (c < out ? c : 0));
    const AdamRegs r_b1 = ld(i_b1), r_b2 = ld(i_b2), r_b3 = ld(i_b3);
    AdamRegs r_w3 = ld(i_w3);                         // critic: its one head column
    setup();
    if (WAIT && wait_on && tid == 0) wait_count(d, wait_on, (uint32_t)chunks);
    __syncthreads();
    const Adam adam = *sh_adam;
    POP_MARK(56);
    float gb1 = 0.0f, gb2 = 0.0f, gw3 = 0.0f, gb3 = 0.0f, loss = 0.0f, logp = 0.0f;
    if (actor_phase) {
#pragma unroll 4
      for (int ch = 0; ch < chunks; ++ch) {
        const float* p = d.apart + ((size_t)agent * chunks + ch) * kAPart;
        const float t1 = p[kAP_db1 + c], t2 = p[kAP_db2 + c], t3 = p[kAP_db3 + (c < out ? c : 0)];
        const float tl = p[kAP_loss], tp = p[kAP_logp];
        gb1 += t1; gb2 += t2; gb3 += t3; loss += tl; logp += tp;
      }
    } else {
#pragma unroll 4
      for (int ch = 0; ch < chunks; ++ch) {
        const float* p = d.cpart + ((size_t)unit * d.cstride + ch) * kCPart;
        const float t1 = p[kCP_db1 + c], t2 = p[kCP_db2 + c], tw = p[kCP_dW3 + c], t3 = p[kCP_db3], tl = p[kCP_loss];
        gb1 += t1; gb2 += t2; gw3 += tw; gb3 += t3; loss += tl;
      }
    }
    POP_MARK(57);
    adam_store<WAIT>(adam, r_b1, gb1, i_b1, th, mo, ve, tg, gr);
    adam_store<WAIT>(adam, r_b2, gb2, i_b2, th, mo, ve, tg, gr);
    if (!actor_phase) adam_store<WAIT>(adam, r_w3, gw3, i_w3, th, mo, ve, tg, gr);
    if (c < out) adam_store<WAIT>(adam, r_b3, gb3, i_b3, th, mo, ve, tg, gr);
    if (actor_phase && d.algo == 1 && c == 0) {
      // SAC temperature: gradient of -alpha mean(log pi + target entropy) with respect to log_alpha, log pi
      // from this step's actor pass held constant; one Adam step with lr_alpha, no target
      float* la = d.log_alpha + agent;
      const float cur = la[0], m0 = la[d.P], v0 = la[2 * d.P];
      const float g = -expf(cur) * (logp / (float)d.B + hp.target_entropy);
      const float mm = adam.b1 * m0 + (1.0f - adam.b1) * g;
      const float vv = adam.b2 * v0 + (1.0f - adam.b2) * (g * g);
      la[d.P] = mm;
      la[2 * d.P] = vv;
      la[0] = cur - hp.lr_alpha * (mm * adam.inv_c1) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(vv * adam.inv_c2) + adam.eps);
    }
    POP_MARK(58);
    if (c == 0) {
      // critic loss = sum over the twins; the two critic workgroups of an agent write
      // their halves to separate slots and the reader adds them
      if (actor_phase) d.losses[(size_t)agent * 4 + 2] = loss;
      else d.losses[(size_t)agent * 4 + (net - 1)] = loss;
    }
  }
  if (feeds_actor) signal_count(d.done_wc + parity_base(d, t, 2 * d.P) + unit, tid);
}

}  // namespace pop
