// Counter-based random numbers on the device: Philox4x32 with 10 rounds
// (Salmon, Moraes, Dror, Shaw, SC'11).  Key = the agent's 64-bit seed; counter =
// (block, step, stream, sub), so a draw depends only on (agent seed, stream,
// step, element) and never on the agent's position in the population.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pop {

enum : uint32_t { kStreamIndex = 0, kStreamSmooth = 1, kStreamSacS = 2, kStreamSacS2 = 3, kStreamInit = 4, kStreamExplore = 5 };

struct U4 { uint32_t w[4]; };

__host__ __device__ inline U4 philox4x32_10(uint32_t k0, uint32_t k1, uint32_t block, uint32_t step,
                                             uint32_t stream, uint32_t sub) {
  uint32_t c0 = block, c1 = step, c2 = stream, c3 = sub;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint64_t pa = (uint64_t)0xD2511F53u * c0;
    const uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)pb; c3 = (uint32_t)pa; c0 = n0; c2 = n2;
  }
  U4 o; o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
  return o;
}

// Word i (0..3) of a block without indexing the register array dynamically.
__host__ __device__ inline uint32_t pick(const U4& r, uint32_t i) {
  const uint32_t lo = (i & 1u) ? r.w[1] : r.w[0];
  const uint32_t hi = (i & 1u) ? r.w[3] : r.w[2];
  return (i & 2u) ? hi : lo;
}

// Replay slot from one word: high half of word * count (integer only).
__host__ __device__ inline uint32_t index_from_word(uint32_t w, uint32_t count) {
  return (uint32_t)(((uint64_t)w * (uint64_t)count) >> 32);
}

// Four standard normals from one block: Box-Muller on word pairs (0,1) and
// (2,3); u1 = (top 24 bits + 1) 2^-24 in (0,1], u2 = top 24 bits 2^-24.
__device__ inline void normals4(const U4& r, float out[4]) {
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const float u1 = ((float)(r.w[2 * p] >> 8) + 1.0f) * 5.9604644775390625e-8f;
    const float u2 = (float)(r.w[2 * p + 1] >> 8) * 5.9604644775390625e-8f;
    const float rad = sqrtf(-2.0f * logf(u1));
    float s, c;
    sincospif(2.0f * u2, &s, &c);
    out[2 * p] = rad * c;
    out[2 * p + 1] = rad * s;
  }
}

}  // namespace pop
