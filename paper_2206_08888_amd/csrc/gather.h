// Replay sample + gather of one float of the stacked batch of step t.
// Slot b of agent i takes word b & 3 of block b >> 2 of the agent's stream 0 at
// step t and maps it to a row of the agent's buffer; element e = b * row + c of
// the batch copies column c of that row.  Shared by the stand-alone gather
// kernel and by the prefetch role of the weight-gradient kernel.
#pragma once
#include "pop_dev.h"
#include "rng.h"

namespace pop {

__host__ __device__ inline int gather_blocks_per_agent(const PopDev& d) { return (d.B * d.row + 255) / 256; }

__device__ inline void gather_element(const PopDev& d, uint32_t t, int agent, int e) {
  if (e >= d.B * d.row) return;
  const int b = e / d.row, c = e - b * d.row;
  const HpDev hp = d.hp[agent];
  const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, (uint32_t)(b >> 2), t, kStreamIndex, 0u);
  const uint32_t idx = index_from_word(pick(blk, (uint32_t)b & 3u), d.count[agent]);
  const size_t slot = ((size_t)(t & 1u) * d.P + agent) * d.B + b;
  d.batch[slot * d.row + c] = d.replay[((size_t)agent * d.capacity + idx) * d.row + c];
  if (c == 0) d.idx[slot] = idx;
}

}  // namespace pop
