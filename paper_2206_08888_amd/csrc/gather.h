// Replay sample + gather of the stacked batch of step t.
// Slot b of agent i takes word b & 3 of block b >> 2 of the agent's stream 0 at
// step t and maps it to a row of the agent's buffer; element e = b * row + c of
// the batch copies column c of that row.  Shared by the stand-alone gather
// kernel and by the prefetch role of the weight-gradient kernel.
#pragma once
#include "pop_dev.h"
#include "rng.h"

#ifndef POP_GATHER_MIN_E
#define POP_GATHER_MIN_E 4
#endif

namespace pop {

// Floats of the stacked batch one thread copies: 1 for narrow rows; for wide rows (SAC at the Humanoid shapes:
// 771 floats) one per 64 floats of a row, so that the gather of a step stays a few dozen workgroups per agent
// (as the tail of the weight-gradient launch, tens of thousands of one-float workgroups cost more in dispatch
// than the rows cost to fetch).
__host__ __device__ inline int gather_floats_per_thread(const PopDev& d) {
  const int e = (d.row + 63) / 64;
  return e < POP_GATHER_MIN_E ? POP_GATHER_MIN_E : (e > 16 ? 16 : e);
}
__host__ __device__ inline int gather_blocks_per_agent(const PopDev& d) {
  const int per = 256 * gather_floats_per_thread(d);
  return (d.B * d.row + per - 1) / per;
}

// Workgroup `block` (of gather_blocks_per_agent) of one agent: thread `tid` copies the floats
// (block * E + k) * 256 + tid, k < E, of the agent's stacked batch.
__device__ inline void gather_block(const PopDev& d, uint32_t t, int agent, int block, int tid) {
  constexpr int kMaxE = 16;
  const int E = gather_floats_per_thread(d);
  const HpDev hp = d.hp[agent];
  const uint32_t count = d.count[agent];
  const int total = d.B * d.row;
  const float* src = d.replay + (size_t)agent * d.capacity * d.row;
  float* dst = d.batch + ((size_t)(t & 1u) * d.P + agent) * d.B * d.row;
  uint32_t* idx_out = d.idx + ((size_t)(t & 1u) * d.P + agent) * d.B;
  int drawn = -1;                                    // batch slot whose index is held in idx
  uint32_t idx = 0;
  float v[kMaxE];
  // all loads of a thread go out before the first store: the rows are random, every load a trip to HBM
#pragma unroll
  for (int k = 0; k < kMaxE; ++k) {
    const int e = (block * E + k) * 256 + tid;
    v[k] = 0.0f;
    if (k < E && e < total) {
      const int b = e / d.row, c = e - b * d.row;
      if (b != drawn) {
        const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, (uint32_t)(b >> 2), t, kStreamIndex, 0u);
        idx = index_from_word(pick(blk, (uint32_t)b & 3u), count);
        drawn = b;
        if (c == 0) idx_out[b] = idx;
      }
      v[k] = src[(size_t)idx * d.row + c];
    }
  }
#pragma unroll
  for (int k = 0; k < kMaxE; ++k) {
    const int e = (block * E + k) * 256 + tid;
    if (k < E && e < total) dst[e] = v[k];
  }
}

}  // namespace pop
