// Layer chains of the SAC update step (Sec. 4.1 of the paper names Soft Actor-Critic with the
// learned temperature, Haarnoja et al. 2018, next to TD3; same networks, same batch).
//
// The policy is a tanh-squashed diagonal Gaussian.  The actor MLP has 2A outputs,
//   (mu, ls) = actor(s), ls clamped to [-20, 2] (no gradient outside);
//   u = mu + exp(ls) eps, eps unit normal from the counter RNG;  a = tanh(u);
//   log pi(a|s) = sum_j [ -eps_j^2/2 - ls_j - ln(2 pi)/2 ] - sum_j 2 (ln 2 - u_j - softplus(-2 u_j)).
// One step, with alpha = exp(log_alpha) as it stands when the step starts:
//   sac_target_chain : a' ~ pi(.|s') from the ONLINE actor (stream 3), twin target critics,
//                      y = r + gamma (1 - d) (min_k Q'_k(s', a') - alpha log pi(a'|s'))
//   critic_chain     : the TD3 one, unchanged (chains.h)
//   sac_actor_chain  : a ~ pi(.|s) (stream 2), both updated critics on [s, a], per sample the
//                      gradient of -min_k Q_k flows through the smaller critic (the first on
//                      ties), plus alpha log pi; backward through the sampling into the actor
//   the temperature  : d/dlog_alpha of -alpha mean(log pi + target entropy), one Adam step on
//                      log_alpha in the actor's weight-gradient launch (wgrad.h)
// The critic targets move every step; there is no target actor and no delay.
#pragma once
#include "chains.h"

namespace pop {

namespace {

__device__ inline float softplusf(float x) { return fmaxf(x, 0.0f) + log1pf(expf(-fabsf(x))); }

constexpr float kLogStdMin = -20.0f, kLogStdMax = 2.0f;
constexpr float kHalfLog2Pi = 0.91893853320467274178f;
constexpr float kLn2 = 0.69314718055994530942f;

// Unit normal number `el` of stream `stream` at counter t (the update step's noise streams).
__device__ inline float normal_at(const HpDev& hp, uint32_t el, uint32_t t, uint32_t stream) {
  const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, el >> 2, t, stream, 0u);
  float n4[4];
  normals4(blk, n4);
  return (el & 2u) ? ((el & 1u) ? n4[3] : n4[2]) : ((el & 1u) ? n4[1] : n4[0]);
}

}  // namespace

// LDS scratch of the SAC chains: nine blocks of [R][kSs] floats (a block = kSacRegion of the
// map's [R][8] regions); the action dimension goes up to kSacMaxAct here.
constexpr int kSs = kSacMaxAct;
constexpr int kSacRegion = kSs / kMaxAct;
constexpr int kSacScratch = 9 * kSacRegion;
static_assert(kSs % kMaxAct == 0 && 2 * kSs >= kMaxHead, "dz3 rows of kMaxHead floats fit two scratch blocks");

// vectors the chains keep in LDS: the actor's head bias, the two critic heads and their biases (the wide
// operands -- the actor's head, the critics' first-layer rows of the action -- go through the matrix pipe
// straight from global memory)
inline int vec_sac_target(const PopDev&) { return kMaxHead + 2 * kH + 8 + kHeadRed; }
constexpr int vec_sac_actor_floats = kMaxHead + 2 * kH + 8 + kHeadRed;   // behind them: the weight stage of the 16-row chains
inline int vec_sac_actor(const PopDev&) { return vec_sac_actor_floats; }

// ---------------------------------------------------------------------------------------------
// Target chain.  One workgroup per (agent, chunk).
template <class G>
__device__ __forceinline__ void sac_target_chain(const PopDev& d, uint32_t t, int agent, int chunk, float* lds) {
  constexpr int R = G::R;
  const LdsMap<G::R, G::kPad> L(d.D, kSacScratch);
  const int A = d.A;
  float* Xs = lds;
  float* buf = lds + L.buf;
  float* hd = lds + L.s(0);                          // [R][kMaxHead]: means | log-stds (later the terms of log pi)
  float* qmin = lds + L.s(2 * kSacRegion);           // [R] min of the target critics, [R..2R) log pi
  float* v_ab3 = lds + L.vec;                        // [kMaxHead]
  float* v_cw3 = v_ab3 + kMaxHead;                   // [2][256]
  float* v_cb3 = v_cw3 + 2 * kH;                     // [2]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = chunk * R;
  const float* an = net_ptr(d, d.theta, agent, 0);   // the online actor: SAC has no target actor
  const float* tc0 = net_ptr(d, d.target, agent, 1);
  const float* tc1 = net_ptr(d, d.target, agent, 2);
  typename G::Pre pre;
  pre.load(an, d.actor, wave, lane);
  const HpDev hp = d.hp[agent];
  const float alpha = expf(d.log_alpha[agent]);
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  POP_MARK(0);
  stage_vector(v_ab3, an + d.actor.b3, 2 * A, tid);
  stage_vector(v_cw3, tc0 + d.critic.w3, kH, tid);
  stage_vector(v_cw3 + kH, tc1 + d.critic.w3, kH, tid);
  if (tid < 2) v_cb3[tid] = (tid == 0 ? tc0 : tc1)[d.critic.b3];
  G::load_input(Xs, L.xld, rows, d.row, d.D + 2, d.O, R, tid);
  __syncthreads();
  POP_MARK(1);

  G::template first_layer<false>(Xs, L.xld, an, d.actor, pre, buf, nullptr, wave, lane);
  __syncthreads();
  POP_MARK(2);
  G::template hidden_layer<false>(buf, an, d.actor, pre, nullptr, wave, lane, [&]() { pre.load(tc0, d.critic, wave, lane); });
  __syncthreads();
  POP_MARK(3);
  if (R <= 32 && 2 * A <= 16) head_mfma_split<R <= 32 ? R : 16, false>(buf, an + d.actor.w3, 2 * A, hd, kMaxHead, wave, lane, v_cb3 + 8);
  else head_mfma<R>(buf, an + d.actor.w3, 2 * A, hd, kMaxHead, wave, lane);
  __syncthreads();
  POP_MARK(4);
  for (int e = tid; e < R * A; e += kThreads) {
    const int r = e / A, j = e - r * A;
    const float mu = hd[r * kMaxHead + j] + v_ab3[j];
    const float ls = fminf(fmaxf(hd[r * kMaxHead + A + j] + v_ab3[A + j], kLogStdMin), kLogStdMax);
    const float eps = normal_at(hp, (uint32_t)((r0 + r) * A + j), t, kStreamSacS2);
    const float u = mu + expf(ls) * eps;
    Xs[r * L.xld + d.O + j] = tanhf(u);
    hd[r * kMaxHead + A + j] = -0.5f * eps * eps - ls - kHalfLog2Pi - 2.0f * (kLn2 - u - softplusf(-2.0f * u));
  }
  __syncthreads();
  if (tid < R) {
    float lp = 0.0f;
    for (int j = 0; j < A; ++j) lp += hd[tid * kMaxHead + A + j];
    qmin[R + tid] = lp;
  }
  POP_MARK(5);

#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const float* tc = k == 0 ? tc0 : tc1;
    G::template first_layer<false>(Xs, L.xld, tc, d.critic, pre, buf, nullptr, wave, lane);
    __syncthreads();
    POP_MARK(6 + 3 * k);
    G::template hidden_layer<false>(buf, tc, d.critic, pre, nullptr, wave, lane,
                                    [&]() { if (k == 0) pre.load(tc1, d.critic, wave, lane); });
    __syncthreads();
    POP_MARK(7 + 3 * k);
    G::thin(buf, v_cw3 + k * kH, 1, hd, tid, kMaxHead);
    __syncthreads();
    if (tid < R) {
      const float q = hd[tid * kMaxHead] + v_cb3[k];
      qmin[tid] = k == 0 ? q : fminf(qmin[tid], q);
    }
    __syncthreads();
    POP_MARK(8 + 3 * k);
  }
  if (tid < R) {
    const float rew = rows[(size_t)tid * d.row + d.D];
    const float done = rows[(size_t)tid * d.row + d.D + 1];
    const float yv = rew + hp.gamma * (1.0f - done) * (qmin[tid] - alpha * qmin[R + tid]);
    d.y[(size_t)agent * d.B + r0 + tid] = yv;
    publish_y(d, (size_t)agent * d.B + r0 + tid, t, yv);
  }
  POP_MARK(12);
}

// Backward through the actor's head for one chunk, thread c = hidden unit c:
//   gW3[c][j] = sum_r h2[r][c] dz3[r][j];  dz2[r][c] = [h2[r][c] > 0] sum_j dz3[r][j] W3[c][j]
// buf: h2 in, dz2 out (LDS tile, row stride kLda); dz3: [R][kMaxHead], columns >= H2 hold zeros; W3: the
// head's weights [256][H2] in global memory;
// NC: head columns handled (a multiple of 4, >= H2).
template <int R, int NC>
__device__ __forceinline__ void sac_head_backward(float* buf, const float* dz3, const float* __restrict__ W3, int H2,
                                                  float* zg, float* part, int c) {
  float w3[NC], gw3[NC];
#pragma unroll
  for (int j = 0; j < NC; ++j) { w3[j] = W3[c * H2 + (j < H2 ? j : 0)]; gw3[j] = 0.0f; }
#pragma unroll
  for (int j = 0; j < NC; ++j) w3[j] = j < H2 ? w3[j] : 0.0f;
  float gb2 = 0.0f;
  zg += c;
#pragma unroll 1
  for (int r = 0; r < R; ++r) {
    const float h = buf[r * kLda + c];
    float dh = 0.0f;
#pragma unroll
    for (int q = 0; q < NC / 4; ++q) {
      const f32x4 g = *reinterpret_cast<const f32x4*>(&dz3[r * kMaxHead + 4 * q]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        gw3[4 * q + i] += h * g[i];
        dh += g[i] * w3[4 * q + i];
      }
    }
    const float z = h > 0.0f ? dh : 0.0f;
    buf[r * kLda + c] = z;
    zg[r * kH] = z;
    gb2 += z;
  }
#pragma unroll
  for (int j = 0; j < NC; ++j)
    if (j < H2) part[kAP_dW3 + j * kH + c] = gw3[j];
  part[kAP_db2 + c] = gb2;
}

// ---------------------------------------------------------------------------------------------
// Actor chain.  One workgroup per (agent, chunk).
//   L = (1/B) sum_b [ alpha log pi(a_b|s_b) - min_k Q_k(s_b, a_b) ]
//   critic k (k = the smaller one for that sample): dz2 = -(1/B) W3^T * [h2 > 0]; dz1 = (dz2 W2^T) * [h1 > 0];
//             da += dz1 W1[O:O+A, :]^T
//   sampling:  du = da (1 - a^2) + (alpha/B) 2a;  dmu = du;  dls = (du std eps - alpha/B) * [ls inside its range]
//   actor:     dz3 = [dmu, dls]; dz2 = (dz3 W3^T) * [h2 > 0]; dz1 = (dz2 W2^T) * [h1 > 0]
template <class G>
__device__ __forceinline__ void sac_actor_chain(const PopDev& d, uint32_t t, int agent, int chunk, float* lds) {
  constexpr int R = G::R;
  const LdsMap<G::R, G::kPad> L(d.D, kSacScratch);
  const int A = d.A, H2 = 2 * d.A;
  float* Xs = lds;
  float* buf = lds + L.buf;
  float* hd = lds + L.s(0);                          // [R][kMaxHead]: means -> terms of log pi -> thin-product scratch
                                                     //                | log-stds -> std * eps
  float* ap = lds + L.s(2 * kSacRegion);             // a = tanh(u)
  float* ins = lds + L.s(3 * kSacRegion);            // 1 where the log-std was inside its range
  float* qv = lds + L.s(4 * kSacRegion);             // [R] q1 | q2 | seed1 | seed2 | log pi
  float* da1 = lds + L.s(5 * kSacRegion);
  float* da2 = lds + L.s(6 * kSacRegion);
  float* dz3 = lds + L.s(7 * kSacRegion);            // [R][kMaxHead] (two blocks)
  float* v_ab3 = lds + L.vec;                        // [kMaxHead]
  float* v_cw3 = v_ab3 + kMaxHead;                   // [2][256] critic heads
  float* v_cb3 = v_cw3 + 2 * kH;                     // [2]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = chunk * R;
  const HpDev hp = d.hp[agent];
  const float alpha = expf(d.log_alpha[agent]);
  const float invB = 1.0f / (float)d.B;
  const float* an = net_ptr(d, d.theta, agent, 0);
  const float* cn[2] = {net_ptr(d, d.theta, agent, 1), net_ptr(d, d.theta, agent, 2)};
  typename G::Pre pre;
  pre.load(an, d.actor, wave, lane);
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  const size_t act_off = ((size_t)agent * d.B + r0) * kH;
  float* part = d.apart + ((size_t)agent * (d.B / R) + chunk) * kAPart;
  POP_MARK(20);
  stage_vector(v_ab3, an + d.actor.b3, H2, tid);
  for (int k = 0; k < 2; ++k) stage_vector(v_cw3 + k * kH, cn[k] + d.critic.w3, kH, tid);
  if (tid < 2) v_cb3[tid] = cn[tid][d.critic.b3];
  G::load_input(Xs, L.xld, rows, d.row, 0, d.O, R, tid);
  __syncthreads();
  POP_MARK(21);

  const uint64_t mask_a1 = G::template first_layer<false>(Xs, L.xld, an, d.actor, pre, buf, d.aH1 + act_off, wave, lane);
  __syncthreads();
  G::template hidden_layer<false>(buf, an, d.actor, pre, d.aH2 + act_off, wave, lane,
                                  [&]() { pre.load(cn[0], d.critic, wave, lane); });
  __syncthreads();
  POP_MARK(22);
  if (R <= 32 && H2 <= 16) head_mfma_split<R <= 32 ? R : 16, false>(buf, an + d.actor.w3, H2, hd, kMaxHead, wave, lane, v_cb3 + 8);
  else head_mfma<R>(buf, an + d.actor.w3, H2, hd, kMaxHead, wave, lane);
  __syncthreads();
  for (int e = tid; e < R * A; e += kThreads) {
    const int r = e / A, j = e - r * A, o = r * kSs + j, om = r * kMaxHead + j, ol = om + A;
    const float mu = hd[om] + v_ab3[j];
    const float ls_raw = hd[ol] + v_ab3[A + j];
    const float ls = fminf(fmaxf(ls_raw, kLogStdMin), kLogStdMax);
    const float eps = normal_at(hp, (uint32_t)((r0 + r) * A + j), t, kStreamSacS);
    const float se = expf(ls) * eps;
    const float u = mu + se;
    const float a = tanhf(u);
    ap[o] = a;
    Xs[r * L.xld + d.O + j] = a;
    hd[ol] = se;
    ins[o] = (ls_raw >= kLogStdMin && ls_raw <= kLogStdMax) ? 1.0f : 0.0f;
    hd[om] = -0.5f * eps * eps - ls - kHalfLog2Pi - 2.0f * (kLn2 - u - softplusf(-2.0f * u));
  }
  __syncthreads();
  if (tid < R) {
    float lp = 0.0f;
    for (int j = 0; j < A; ++j) lp += hd[tid * kMaxHead + j];
    qv[4 * R + tid] = lp;
  }
  POP_MARK(23);

  // both critics forward on [s, a]; the ReLU patterns of both layers stay in registers
  uint64_t mask1[2], mask2[2];
  typename G::WtBlock wt;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    mask1[k] = G::template first_layer<false>(Xs, L.xld, cn[k], d.critic, pre, buf, nullptr, wave, lane);
    __syncthreads();
    mask2[k] = G::template hidden_layer<false>(buf, cn[k], d.critic, pre, nullptr, wave, lane, [&]() {
      if (k == 0) pre.load(cn[1], d.critic, wave, lane);
      else G::load_wt(wt, cn[0] + d.critic.w2, wave, lane);
    });
    __syncthreads();
    G::thin(buf, v_cw3 + k * kH, 1, hd, tid, kMaxHead);
    __syncthreads();
    if (tid < R) qv[k * R + tid] = hd[tid * kMaxHead] + v_cb3[k];
    __syncthreads();
    POP_MARK(24 + k);
  }
  if (tid < 64) {                                    // R <= 64: one wavefront covers the chunk
    float term = 0.0f, lp = 0.0f;
    if (tid < R) {
      const float q1 = qv[tid], q2 = qv[R + tid];
      const bool first = q1 <= q2;                   // ties go to the first critic
      qv[2 * R + tid] = first ? -invB : 0.0f;
      qv[3 * R + tid] = first ? 0.0f : -invB;
      lp = qv[4 * R + tid];
      term = alpha * lp - (first ? q1 : q2);
    }
    const float s_loss = wave_sum(term), s_lp = wave_sum(lp);
    if (tid == 0) { part[kAP_loss] = s_loss * invB; part[kAP_logp] = s_lp; }
  }
  __syncthreads();

  // both critics backward to the action
  f32x4 h2r[R / 4];                                  // this thread's share of the actor's parked h2 tile
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    G::store_outer_masked(buf, mask2[k], qv + (2 + k) * R, v_cw3 + k * kH, wave, lane);     // dz2 of critic k
    __syncthreads();
    const float* h2g = d.aH2 + act_off;
    G::input_grad_to_lds(buf, cn[k] + d.critic.w2, wt, mask1[k], wave, lane, [&]() {
      if (k == 0) return;
#pragma unroll
      for (int i = 0; i < R / 4; ++i)
        h2r[i] = *reinterpret_cast<const f32x4*>(h2g + (4 * i + (tid >> 6)) * kH + 4 * (tid & 63));
    }, lds + L.vec + vec_sac_actor_floats);          // buf = dz1 of critic k
    __syncthreads();
    if (R <= 32 && A <= 16) head_mfma_split<R <= 32 ? R : 16, true>(buf, cn[k] + d.critic.w1 + d.O * kH, A, k == 0 ? da1 : da2, kSs, wave, lane, v_cb3 + 8);
    else head_mfma_t<R>(buf, cn[k] + d.critic.w1 + d.O * kH, A, k == 0 ? da1 : da2, kSs, wave, lane);
    if (k == 0) G::load_wt(wt, cn[1] + d.critic.w2, wave, lane);
    else G::load_wt(wt, an + d.actor.w2, wave, lane);
    __syncthreads();
    POP_MARK(26 + k);
  }

  // through the sampling into the actor's head
  const float ab = alpha * invB;
  for (int e = tid; e < R * kMaxHead; e += kThreads) {
    const int r = e / kMaxHead, c = e - r * kMaxHead;
    float g = 0.0f;
    if (c < H2) {
      const int j = c < A ? c : c - A, o = r * kSs + j;
      const float a = ap[o];
      const float du = (da1[o] + da2[o]) * (1.0f - a * a) + ab * 2.0f * a;
      g = c < A ? du : (du * hd[r * kMaxHead + A + j] - ab) * ins[o];
    }
    dz3[e] = g;                                      // unused columns are kept at zero
  }
#pragma unroll
  for (int i = 0; i < R / 4; ++i)                    // h2 of the actor back into the tile
    *reinterpret_cast<f32x4*>(&buf[(4 * i + (tid >> 6)) * kLda + 4 * (tid & 63)]) = h2r[i];
  __syncthreads();
  if (tid < H2) {
    float s = 0.0f;
    for (int r = 0; r < R; ++r) s += dz3[r * kMaxHead + tid];
    part[kAP_db3 + tid] = s;
  }
  POP_MARK(28);
  // actor head backward, one thread per hidden unit; the common small heads stay in 16 registers
  if (H2 <= 16) sac_head_backward<R, 16>(buf, dz3, an + d.actor.w3, H2, d.adZ2 + act_off, part, tid);
  else sac_head_backward<R, kMaxHead>(buf, dz3, an + d.actor.w3, H2, d.adZ2 + act_off, part, tid);
  __syncthreads();
  POP_MARK(29);
  G::template input_grad_to_global<false>(buf, an + d.actor.w2, wt, mask_a1, d.adZ1 + act_off, part + kAP_db1, wave, lane,
                                          lds + L.vec + vec_sac_actor_floats);
  POP_MARK(30);
}

}  // namespace pop
