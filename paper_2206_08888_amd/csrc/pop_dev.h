// Device-side view of a population and shared constants.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Timeline instrumentation, compiled out of the library proper.  The traced build (trace_unity.hip: every source of
// the library in one translation unit with POP_TRACE defined, built as libpop_trace.so) keeps, per kernel kind and
// block, the constant-rate clock at the block's start and end, and the phase marks of one chosen block; the
// trace_* calls of that build read them back (paper_2206_08888_amd/timeline.py prints the timelines).
#ifdef POP_TRACE
constexpr int kTraceKinds = 8, kTraceBlocks = 32768;
enum { kTraceStep = 0, kTraceTargetCritic = 1, kTraceWgradCritic = 2, kTraceActor = 3, kTraceWgradActor = 4, kTraceTarget = 5, kTraceCritic = 6 };
extern __device__ unsigned long long g_pop_trace[64];
extern __device__ int g_pop_trace_block;            // the block whose marks are recorded
extern __device__ unsigned long long g_pop_block_time[kTraceKinds][2][kTraceBlocks];
#define POP_MARK(i)                                                                 \
  do {                                                                              \
    if ((int)blockIdx.x == g_pop_trace_block && threadIdx.x == 0) g_pop_trace[i] = wall_clock64(); \
    if (blockIdx.x == 0 && threadIdx.x == 0 && (i) == 63) g_pop_trace[63] = wall_clock64();       \
  } while (0)
#define POP_BLOCK_TIME(kind, w) do { if (threadIdx.x == 0 && blockIdx.x < kTraceBlocks) g_pop_block_time[kind][w][blockIdx.x] = wall_clock64(); } while (0)
#else
#define POP_MARK(i)
#define POP_BLOCK_TIME(kind, w)
#endif

namespace pop {

constexpr int kH = 256;        // hidden width the kernels are specialised for
constexpr int kLda = kH + 4;   // LDS row stride of a 256-wide activation tile: 4*odd words, so
                               // 8 lanes reading 16 B each from 8 consecutive rows hit all 32 banks
constexpr int kThreads = 256;  // 4 wavefronts of 64 per workgroup in every compute kernel
constexpr int kMaxIn = 64;     // narrow shapes: largest first-layer fan-in (obs_dim + act_dim) of the chains without a pipelined
                               // first layer -- all fused launch structures are built for these
constexpr int kMaxAct = 8;     // narrow shapes: largest action dimension; also the row stride of the small LDS scratch blocks
constexpr int kSacMaxIn = 448; // wide shapes (SAC and plain TD3): largest first-layer fan-in (the Humanoid shapes need 393)
constexpr int kSacMaxAct = 24; // wide shapes: largest action dimension (Humanoid: 17) and row stride of their scratch blocks
constexpr int kCUs = 256;       // compute units of the chip
constexpr int kLdsPerCU = 160 * 1024;   // bytes of LDS one workgroup can ask for
constexpr int kMaxHead = 48;   // largest actor head: 2 * kSacMaxAct outputs (mean and log-std of the SAC policy)

struct HpDev {                 // per-agent hyperparameters as the kernels read them
  uint32_t seed_lo, seed_hi;
  float lr_actor, lr_critic, gamma, tau, policy_noise, noise_clip;
  int32_t policy_delay;
  float b1, b2, eps;
  // Adam step count of the actor: actor_base updates were taken before step t_base; since then one at every
  // step that is a multiple of policy_delay (both change only when the host resets hyperparameters or copies an agent)
  uint32_t actor_base, t_base;
  float lr_alpha, target_entropy;   // SAC
};
static_assert(sizeof(HpDev) == 64, "HpDev layout");

// Offsets (floats) of the tensors of one network in canonical order.
struct NetLayout {
  int in, out;                 // fan-in of layer 1, fan-out of the head
  int w1, b1, w2, b2, w3, b3;  // offsets
  int size, padded;            // true length, length rounded up to 64 floats
};

__host__ __device__ inline NetLayout make_layout(int in, int out) {
  NetLayout L;
  L.in = in; L.out = out;
  L.w1 = 0;            L.b1 = in * kH;
  L.w2 = L.b1 + kH;    L.b2 = L.w2 + kH * kH;
  L.w3 = L.b2 + kH;    L.b3 = L.w3 + kH * out;
  L.size = L.b3 + out; L.padded = (L.size + 63) / 64 * 64;
  return L;
}

struct PopDev {
  int algo;                    // POP_ALGO_TD3 (0), POP_ALGO_SAC (1; its actor has 2 A outputs) or POP_ALGO_TD3_SHARED (2)
  int share;                   // 1; shared critics (Sec. 4.2 of the paper): P -- every agent's critic blocks are agent
                               // 0's and the critic loss is the mean over the population
  int groups;                  // shared critics: agent groups whose gradients are summed separately (spart)
  float* spart;                // shared critics: [2][groups][critic.padded] partial gradients, laid out like the network
  float* sloss;                // shared critics: [2][groups] partial losses
  int P, O, A, D, B, row;      // D = O + A; row = 2 O + A + 2 floats
  int rows_t, rows_c, rows_a;  // batch rows per workgroup of the target / critic / actor chain: (16, 32 or 64, 16) for
                               // small populations, else (32, 32, 32); (64, 64, 64) on request
  int rows_c1;                 // rows per workgroup of critic 1's chain: rows_c, or 16 where the target workgroups run it (k_chain.hip)
  int cstride;                 // chunk slots per network in cpart: B / min(rows_c1, rows_c)
  int half_tiles;              // the stand-alone weight-gradient launch runs tiles of half the width (k_wgrad_adam.hip)
  NetLayout actor, critic;
  int agent_sz;                // actor.padded + 2 * critic.padded
  // parameter state, each [P][agent_sz] = [actor | critic1 | critic2]
  float *theta, *target, *m, *v, *grad;
  int record_grads;
  const HpDev* hp;
  // replay
  float* replay;               // [P][capacity][row]
  uint64_t capacity;
  uint32_t *count, *cursor;    // [P]
  // state of the current step; idx and batch are double-buffered by step parity so
  // that the rows of step t + 1 can be gathered while step t is still computing
  uint32_t* idx;               // [2][P][B]
  float* batch;                // [2][P][B][row]
  float* atilde;               // [P][B][A]
  float* api;                  // [P][B][A] actions of the current policy on the batch, where the critic-2 workgroups of the
                               // fused target / critic launch run the actor's forward pass ahead of the actor launch
  int actor_ahead;             // 1: they do (small populations: those workgroups would otherwise idle until the targets arrive)
  float* y;                    // [P][B]
  // activations handed from the chain kernels to the weight-gradient kernel
  float *cH1, *cdZ2, *cdZ1;    // [P][2][B][256]
  float *aH1, *aH2, *adZ2, *adZ1;  // [P][B][256]
  // per-row-chunk partial sums of the small gradients and of the losses
  float* cpart;                // [P][2][cstride][kCPart]
  float* apart;                // [P][chunks][kAPart]
  float* losses;               // [P][4]: critic 1, critic 2, actor, unused
  float* log_alpha;            // SAC: [3][P] log temperature, its Adam m, its Adam v
  // cross-workgroup signalling inside a launch
  uint64_t* y_tagged;          // [P][B]: (t + 1) << 32 | bits of y, for readers inside the launch that writes y
  int sync_half;               // which half of the counters below this launch counts in (set per launch)
  uint32_t* done_c;            // [2][2P] critic chunks finished per network
  uint32_t* done_wc;           // [2][2P] critic weight-gradient roles finished per network
  uint32_t* done_a;            // [2][P]  actor chunks finished per agent
  uint32_t* fault;             // [2] in pinned host memory: [0] != 0: a wait for y ran out, [1] != 0: a wait for a count
  unsigned long long wait_limit;   // longest wait of one workgroup for another of the same launch, in 10 ns ticks of the
                               // constant-rate clock (default 50 ms; a healthy wait is a fraction of a millisecond)
};

// critic partial record: dW3[256] db3[1] pad[3] db2[256] db1[256] loss[1] pad[3]
constexpr int kCP_dW3 = 0, kCP_db3 = 256, kCP_db2 = 260, kCP_db1 = 516, kCP_loss = 772, kCPart = 776;
// actor partial record: dW3[kMaxHead][256] (head column j of hidden unit c at j*256 + c) db3[kMaxHead] db2[256] db1[256] loss[1] logp[1] pad
constexpr int kAP_dW3 = 0, kAP_db3 = 256 * kMaxHead, kAP_db2 = kAP_db3 + kMaxHead, kAP_db1 = kAP_db2 + 256,
              kAP_loss = kAP_db1 + 256, kAP_logp = kAP_loss + 1 /* SAC: sum of log pi over the chunk */, kAPart = kAP_loss + 8;

__device__ inline const float* batch_rows(const PopDev& d, uint32_t t, int agent) {
  return d.batch + ((size_t)(t & 1u) * d.P + agent) * d.B * d.row;
}

// Workgroup ids are handed to the 8 XCDs round-robin; decode a 1-D block id so that
// all `per_unit` workgroups of one unit (an agent or a network) land on the same
// XCD and share its L2 (weights and activations of that unit).  That works for whole
// groups of 8 units.  The r = units % 8 left over cannot each have an XCD of their own while
// the grid keeps exactly units * per_unit blocks (blocks that only exit would still take a
// turn in the dispatcher's walk over the CUs, and push later workgroups onto CUs that are
// already busy while others stand empty), so their workgroups are numbered XCD by XCD: a
// left-over unit then sits on about 8 / r neighbouring XCDs instead of on all 8 (P = 10: the
// two left-over agents on four XCDs each, the four left-over critics on two), and its weights
// are fetched from memory that many times instead of eight.
// The grouping only needs ids that are congruent mod 8 to share an XCD, so `id` may be
// offset by any constant (a kernel that runs two kinds of workgroups).
// ORDERED: the caller needs `sub` to grow with `id` within a unit (a later sub-block waits for an
// earlier one of the same unit); the left-over units are then laid out plainly, over all XCDs.
template <bool ORDERED = false>
__host__ __device__ inline bool decode_block(int id, int units, int per_unit, int& unit, int& sub) {
  const int full = units & ~7, nfull = full * per_unit;
  if (id < nfull) {
    const int x = id & 7, slot = id >> 3;
    unit = (slot / per_unit) * 8 + x;
    sub = slot % per_unit;
  } else {
    int j = id - nfull;
    if (!ORDERED) {                                    // position of block j when the left-over blocks are listed XCD by XCD
      const int n = (units - full) * per_unit, q = n >> 3, rem = n & 7, x = j & 7;
      j = x * q + (x < rem ? x : rem) + (j >> 3);
    }
    unit = full + j / per_unit;
    sub = j % per_unit;
  }
  return unit < units;
}
__host__ inline int xcd_grid(int units, int per_unit) { return units * per_unit; }

__device__ inline const float* net_ptr(const PopDev& d, const float* base, int agent, int net) {
  if (d.share > 1 && net >= 1) agent = 0;            // the one critic pair lives in agent 0's blocks
  const float* p = base + (size_t)agent * d.agent_sz;
  if (net >= 1) p += d.actor.padded;
  if (net >= 2) p += d.critic.padded;
  return p;
}
__device__ inline float* net_ptr(const PopDev& d, float* base, int agent, int net) {
  return const_cast<float*>(net_ptr(d, (const float*)base, agent, net));
}

}  // namespace pop
