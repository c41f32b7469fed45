// Replay buffer kernels: ring insertion and the per-step sample + gather.
//
// App. A of the paper: each agent owns a bounded first-in-first-out buffer and
// the sampled batches of all agents are stacked on a new leading axis.  Here
// the buffers live in HBM as dense rows [P][capacity][obs, act, reward, done,
// next_obs]; a step draws B row indices per agent from the counter RNG
// (stream 0, slot b = word b & 3 of block b >> 2) and copies the rows into the
// stacked batch [P][B][row].  Consecutive lanes read consecutive floats of one
// row, so each random row costs two or three contiguous 64-byte segments.
#include "launch.h"
#include "gather.h"

namespace pop {

__global__ __launch_bounds__(256) void k_insert(PopDev d, int agent_arg, uint32_t n, uint32_t first, uint32_t rows,
                                                const float* __restrict__ obs, const float* __restrict__ act,
                                                const float* __restrict__ rew, const float* __restrict__ done,
                                                const float* __restrict__ next_obs) {
  // grid: (ceil(rows * row / 256), agents).  Writes source rows [first, first + rows) of a
  // call that appends n rows; source row j lands in slot (cursor + j) mod capacity.
  const int which = blockIdx.y;
  const int agent = agent_arg < 0 ? which : agent_arg;
  const uint64_t e = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (uint64_t)rows * d.row) return;
  const uint32_t j = first + (uint32_t)(e / d.row);
  const int c = (int)(e % d.row);
  const size_t src_row = (size_t)which * n + j;        // which == 0 for a single agent
  float val;
  if (c < d.O) val = obs[src_row * d.O + c];
  else if (c < d.D) val = act[src_row * d.A + (c - d.O)];
  else if (c == d.D) val = rew[src_row];
  else if (c == d.D + 1) val = done[src_row];
  else val = next_obs[src_row * d.O + (c - d.D - 2)];
  const uint64_t slot = ((uint64_t)d.cursor[agent] + j) % d.capacity;
  d.replay[((size_t)agent * d.capacity + slot) * d.row + c] = val;
}

__global__ void k_advance(PopDev d, int agent_arg, uint32_t n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d.P) return;
  if (agent_arg >= 0 && i != agent_arg) return;
  d.cursor[i] = (uint32_t)(((uint64_t)d.cursor[i] + n) % d.capacity);
  const uint64_t c = (uint64_t)d.count[i] + n;
  d.count[i] = (uint32_t)(c < d.capacity ? c : d.capacity);
}

hipError_t launch_insert(const PopDev& d, int agent, int64_t n, const float* obs, const float* act,
                         const float* rew, const float* done, const float* next_obs, hipStream_t s) {
  // Rows that later rows of the same call would overwrite (n > capacity) are skipped, so
  // no two threads ever write the same slot.
  const uint32_t n32 = (uint32_t)n;
  const uint32_t skip = (uint64_t)n > d.capacity ? (uint32_t)((uint64_t)n - d.capacity) : 0u;
  const uint32_t piece = 1u << 22;
  for (uint64_t f = skip; f < n32; f += piece) {
    const uint32_t first = (uint32_t)f;
    const uint32_t rows = n32 - first < piece ? n32 - first : piece;
    dim3 grid((unsigned)(((uint64_t)rows * d.row + 255) / 256), agent < 0 ? d.P : 1);
    hipLaunchKernelGGL(k_insert, grid, dim3(256), 0, s, d, agent, n32, first, rows, obs, act, rew, done, next_obs);
  }
  hipLaunchKernelGGL(k_advance, dim3((d.P + 255) / 256), dim3(256), 0, s, d, agent, n32);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_sample_gather(PopDev d, uint32_t t) {
  // grid: (gather_blocks_per_agent, P); a thread copies one float of the stacked batch (several for wide rows)
  gather_block(d, t, blockIdx.y, blockIdx.x, threadIdx.x);
}

hipError_t launch_sample_gather(const PopDev& d, uint32_t t, hipStream_t s) {
  dim3 grid(gather_blocks_per_agent(d), d.P);
  hipLaunchKernelGGL(k_sample_gather, grid, dim3(256), 0, s, d, t);
  return hipGetLastError();
}

}  // namespace pop
