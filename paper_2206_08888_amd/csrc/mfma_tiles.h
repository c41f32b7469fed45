// Wavefront-level fp32 MFMA building blocks for the per-agent MLP layers.
//
// All dense contractions of the update step (App. C of the paper: y = x W + b
// per population member, and the matching backward products) run on
// v_mfma_f32_32x32x2_f32: one instruction multiplies a 32x2 slice of A by a
// 2x32 slice of B into a 32x32 fp32 tile held as 16 registers per lane.
//
// Operand layout of that instruction on a 64-lane wavefront:
//   A: lane l supplies A[row = l & 31][k = l >> 5]
//   B: lane l supplies B[k = l >> 5][col = l & 31]
//   D: register v of lane l is D[row = 8 (v >> 2) + 4 (l >> 5) + (v & 3)][col = l & 31]
//
// A workgroup is 4 wavefronts; for a [R x 256] output each wavefront owns the
// 64 columns [64 wave, 64 wave + 64) for all R = 32 MT rows, i.e. MT x 2 tiles.
// Tile nt holds the columns of parity nt: lane l has columns 64 wave + 2 (l & 31) + nt
// (tile_col), two neighbours, which it loads and stores as one 8-byte access.
// The left operand (activations) lives in LDS and is shared by the 4
// wavefronts; the right operand (weights) is read by each wavefront straight
// from global memory/L2 into registers, because every weight element is used
// by exactly one wavefront of the workgroup -- staging it in LDS would add
// traffic and barriers without any reuse.
//
// The contraction index may be visited in any order as long as both operands
// agree, so one lane fetches 4 consecutive k of the LDS operand with a single
// 16-byte read and uses them in 4 successive MFMAs (lanes 0-31 take k0..k0+3,
// lanes 32-63 take k0+4..k0+7).
#pragma once
#include <hip/hip_runtime.h>
#include "pop_dev.h"

namespace pop {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ inline f32x16 mfma32(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Global store of a result that another workgroup of the SAME launch reads (THROUGH): a
// device-scope atomic store, which is written through the XCD's L2 to memory instead of
// waiting there as a dirty line, so that the producer only has to see its own stores
// acknowledged before it signals, not have the whole L2 written back.
template <bool THROUGH>
__device__ inline void put(float* p, float v) {
  if (THROUGH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else *p = v;
}
// the same for two neighbouring floats at an 8-byte aligned address (a lane's two columns, tile_col)
template <bool THROUGH>
__device__ inline void put2(float* p, float a, float b) {
  if (THROUGH) {
    const unsigned long long word = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    *reinterpret_cast<f32x2*>(p) = f32x2{a, b};
  }
}

__device__ inline int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }
// Column (of 256) that a lane holds of tile nt of its wavefront's two accumulator tiles: the lane's two columns
// are neighbours, so that a forward product fetches both weights of a row with one 8-byte load (half the load
// instructions, which is what the forward products were short of).
__device__ inline int tile_col(int wave, int nt, int lane) { return 64 * wave + 2 * (lane & 31) + nt; }

// NT = 32-column tiles per wavefront: 2 in the layer chains (a workgroup spans 256
// columns), 1 in the weight-gradient tiles (128 columns per workgroup).
template <int MT, int NT = 2>
struct Acc {
  f32x16 t[MT][NT];
  __device__ inline void zero() {
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
      for (int b = 0; b < NT; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) t[a][b][v] = 0.0f;
  }
};

// f(row, col, value) for every accumulator element this lane holds;
// row in [0, 32 MT), col in [0, 256).
template <int MT, class F>
__device__ inline void for_each_acc(const Acc<MT>& acc, int wave, int lane, F f) {
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        f(32 * mt + acc_row(v, lane), tile_col(wave, nt, lane), acc.t[mt][nt][v]);
}

// First-layer weights of one lane for the leading 32 rows of W (k = 8 i + 4 half + j),
// fetched ahead of time so that the product does not wait for memory.
struct SmallW {
  float w[4][2][4];
  __device__ inline void load(const float* __restrict__ W, int K, int wave, int lane) {
    const int half = lane >> 5, l32 = lane & 31;
    const float* wcol = W + tile_col(wave, 0, l32);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = 8 * i + 4 * half + j;
        const int kk = k < K ? k : 0;                 // always a valid row: the load needs no branch
        const f32x2 v = *reinterpret_cast<const f32x2*>(wcol + kk * kH);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) w[i][nt][j] = k < K ? v[nt] : 0.0f;
      }
  }
};

// acc[r][c] += sum_{k<K} X[r][k] W[k][c]   (forward product x W) for a small fan-in K.
//   X: LDS, row stride ldx, rows [0, 32 MT); columns >= K up to the next
//      multiple of 8 must hold finite values (they meet zero weights);
//   W: global, row-major [K][256]; `pre` holds its first 32 rows already.
template <int MT>
__device__ inline void gemm_xw_small(const float* __restrict__ Xl, int ldx, int K, const float* __restrict__ W,
                                     const SmallW& pre, int wave, int lane, Acc<MT>& acc) {
  const int half = lane >> 5, l32 = lane & 31;
  const int K8 = (K + 7) & ~7;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (8 * i < K8) {
      f32x4 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        a[mt] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + 8 * i + 4 * half]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) acc.t[mt][nt] = mfma32(a[mt][j], pre.w[i][nt][j], acc.t[mt][nt]);
    }
  }
  const float* wcol = W + tile_col(wave, 0, l32);
  for (int k0 = 32; k0 < K8; k0 += 8) {              // fan-in beyond 32: plain loop
    float b[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + 4 * half + j;
      const f32x2 v = *reinterpret_cast<const f32x2*>(wcol + (size_t)(k < K ? k : 0) * kH);
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) b[nt][j] = k < K ? v[nt] : 0.0f;
    }
    f32x4 a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      a[mt] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + k0 + 4 * half]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc.t[mt][nt] = mfma32(a[mt][j], b[nt][j], acc.t[mt][nt]);
  }
}

// The same product for a fan-in of several hundred: the 8-deep blocks beyond the prefetched 32
// rows are software-pipelined, PF weight blocks (8 PF rows of W) in flight ahead of the matrix pipe.
template <int MT, int PF>
__device__ inline void gemm_xw_deep(const float* __restrict__ Xl, int ldx, int K, const float* __restrict__ W,
                                    const SmallW& pre, int wave, int lane, Acc<MT>& acc) {
  const int half = lane >> 5, l32 = lane & 31;
  const int nb = (K + 7) >> 3;                       // 8-deep blocks in all; 0 .. 3 come from `pre`
  const float* wcol = W + tile_col(wave, 0, l32);
  float b[PF][2][4];
  auto request = [&](float (&dst)[2][4], int blk) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = 8 * blk + 4 * half + j;
      const f32x2 v = *reinterpret_cast<const f32x2*>(wcol + (size_t)(k < K ? k : 0) * kH);
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) dst[nt][j] = k < K ? v[nt] : 0.0f;
    }
  };
#pragma unroll
  for (int s = 0; s < PF; ++s)
    if (4 + s < nb) request(b[s], 4 + s);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < nb) {
      f32x4 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        a[mt] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + 8 * i + 4 * half]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt) acc.t[mt][nt] = mfma32(a[mt][j], pre.w[i][nt][j], acc.t[mt][nt]);
    }
  }
  auto lds_block = [&](f32x4 (&a)[MT], int i) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      a[mt] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + 8 * i + 4 * half]);
  };
  f32x4 an[MT];                                      // the LDS operand runs one block ahead of the matrix pipe
  if (4 < nb) lds_block(an, 4);
  // FAST: block i + PF lies wholly inside the K rows: its eight loads are one running pointer plus constants
  // (no per-load address arithmetic or row guard, which would sit in front of every group of MFMAs)
  const float* wrun = wcol + (size_t)(8 * (4 + PF) + 4 * half) * kH;     // rows of block 4 + PF for this lane
  auto step = [&](int s, int i, bool next_x, bool next_w, bool fast) {
    f32x4 a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) a[mt] = an[mt];
    if (next_x) lds_block(an, i + 1);
    float w[2][4];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int j = 0; j < 4; ++j) w[nt][j] = b[s][nt][j];
    if (fast) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x2 v = *reinterpret_cast<const f32x2*>(wrun + j * kH);
        b[s][0][j] = v[0];
        b[s][1][j] = v[1];
      }
    } else if (next_w) {
      request(b[s], i + PF);
    }
    wrun += 8 * kH;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc.t[mt][nt] = mfma32(a[mt][j], w[nt][j], acc.t[mt][nt]);
    __builtin_amdgcn_sched_barrier(0);
  };
  int blk = 4;
  // steady state, free of branches (a branch inside the loop makes the compiler drain every outstanding load at
  // the join): every block of the group exists and every block requested from it is a full one
  const int nfull = K >> 3;
  for (; blk + 2 * PF <= nfull; blk += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) step(s, blk + s, true, true, true);
  }
  for (; blk < nb; blk += PF) {                      // the last groups: guarded requests
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      const int i = blk + s;
      if (i < nb) step(s, i, i + 1 < nb, i + PF < nb, false);
    }
  }
}

// Software-pipelined 256-deep contraction of an LDS operand with a global weight
// operand; the contraction index is walked in 16 blocks of 16.
//   forward  (TRANSPOSED = false): acc[r][c] += sum_k X[r][k] W[k][c], c in this wave's 64 columns
//   backward (TRANSPOSED = true):  acc[r][k] += sum_n Z[r][n] W[k][n], k in this wave's 64 columns
// W is row-major [256][256] in both cases.  Weight registers rotate through four
// buffers: block j+3 is requested from memory before the MFMAs of block j start,
// so about 3000 MT cycles of matrix work cover the L2 / memory latency; the LDS
// operand is fetched one block ahead.  Block 0 is passed in by the caller, who
// requests it as early as it can (typically under the previous product);
// `tail()` runs once no further weight block of this product is needed, so the
// caller can start the loads of the next layer under the last three blocks.
// __builtin_amdgcn_sched_barrier keeps the compiler from sinking loads back next
// to their uses.
template <int MT, bool TRANSPOSED, int NT = 2>
struct WeightBlock {                       // the weights one lane needs for a 16-deep block
  float w[NT][8];                          // [column tile][4 s + j]  <->  index 16 i + 8 s + 4 half + j
  // column of W (forward) or row of W (transposed) that lane l32 holds of tile nt: with two tiles per wavefront
  // the lane's two columns are neighbours, so that the forward product fetches both with one load
  __device__ static constexpr int col_of(int wave, int nt, int l32) {
    return NT == 2 ? tile_col(wave, nt, l32) : 32 * wave + l32;
  }
  __device__ inline void load(const float* __restrict__ W, int i, int wave, int lane) {
    const int half = lane >> 5, l32 = lane & 31;
    if (TRANSPOSED) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const float* row = W + col_of(wave, nt, l32) * kH + 16 * i + 4 * half;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(row + 8 * s);
          w[nt][4 * s + 0] = v[0]; w[nt][4 * s + 1] = v[1]; w[nt][4 * s + 2] = v[2]; w[nt][4 * s + 3] = v[3];
        }
      }
    } else if (NT == 2) {                            // the lane's two columns are neighbours: one 8-byte load per row
      const float* col = W + (16 * i + 4 * half) * kH + 64 * wave + 2 * l32;
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const f32x2 v = *reinterpret_cast<const f32x2*>(col + (8 * s + j) * kH);
          w[0][4 * s + j] = v[0];
          w[NT - 1][4 * s + j] = v[1];
        }
    } else {
      const float* col = W + (16 * i + 4 * half) * kH + 32 * NT * wave + l32;
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) w[nt][4 * s + j] = col[(8 * s + j) * kH + 32 * nt];
    }
  }
  // The same block as kPieces separate load instructions, in the order of use, from this lane's pointer into W
  // (lane_base) moved on to block i by the caller: blk = lane_base(W) + 16 i kH (forward) or + 16 i (transposed).
  static constexpr int kPieces = TRANSPOSED ? 2 * NT : 8;
  __device__ static inline const float* lane_base(const float* __restrict__ W, int wave, int lane) {
    const int half = lane >> 5, l32 = lane & 31;
    return TRANSPOSED ? W + col_of(wave, 0, l32) * kH + 4 * half : W + 4 * half * kH + col_of(wave, 0, l32);
  }
  __device__ inline void load_piece(const float* __restrict__ blk, int p) {
    if (TRANSPOSED) {
      const int s = p / NT, nt = p % NT;
      const f32x4 v = *reinterpret_cast<const f32x4*>(blk + (col_of(0, nt, 0) - col_of(0, 0, 0)) * kH + 8 * s);
      w[nt][4 * s + 0] = v[0]; w[nt][4 * s + 1] = v[1]; w[nt][4 * s + 2] = v[2]; w[nt][4 * s + 3] = v[3];
    } else if (NT == 2) {
      const int s = p >> 2, j = p & 3;
      const f32x2 v = *reinterpret_cast<const f32x2*>(blk + (8 * s + j) * kH);
      w[0][4 * s + j] = v[0];
      w[NT - 1][4 * s + j] = v[1];
    } else {
      const int s = p >> 2, j = p & 3;
      w[0][4 * s + j] = blk[(8 * s + j) * kH];
    }
  }
};

template <int MT>
struct LdsBlock {                          // the LDS operand of one block (16 deep)
  f32x4 a[MT][2];
  __device__ inline void load(const float* __restrict__ Xl, int ldx, int k0, int lane) {
    const int half = lane >> 5, l32 = lane & 31;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int s = 0; s < 2; ++s)
        a[mt][s] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + k0 + 8 * s + 4 * half]);
  }
  __device__ inline void load_piece(const float* __restrict__ Xl, int ldx, int k0, int lane, int p) {   // p < 2 MT
    const int half = lane >> 5, l32 = lane & 31, mt = p >> 1, s = p & 1;
    a[mt][s] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + k0 + 8 * s + 4 * half]);
  }
};

template <int MT, bool TRANSPOSED, int NT = 2>
__device__ inline void mfma_block(const LdsBlock<MT>& x, const WeightBlock<MT, TRANSPOSED, NT>& b, Acc<MT, NT>& acc) {
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc.t[mt][nt] = mfma32(x.a[mt][s][j], b.w[nt][4 * s + j], acc.t[mt][nt]);
}

// The MFMAs of one block with the loads of a later block (weights `nb` <- the block at `blk` when FEED, LDS operand
// `nx` <- columns nk0.. when FEEDX) dealt out between them, one piece behind an MFMA until they are used up
// (scheduling groups tell the compiler that order).  A matrix instruction keeps its pipe busy for 64 cycles after
// it issues; load instructions issued in that shadow cost nothing, while a whole block's worth of them between
// two blocks -- some 16 cycles each -- leaves the pipe idle for as long as they take to issue.  That shows where
// two workgroups share a CU and the other wavefront of the SIMD is no further along: 25.6 us per 32-row product
// for such a pair, 19.9 us in this form.  With one workgroup per CU the plain order is the faster one (8.7
// against 9.4 us).
template <int MT, bool TRANSPOSED, int NT, bool FEED, bool FEEDX>
__device__ inline void mfma_block_fed(const LdsBlock<MT>& x, const WeightBlock<MT, TRANSPOSED, NT>& b, Acc<MT, NT>& acc,
                                      WeightBlock<MT, TRANSPOSED, NT>& nb, const float* __restrict__ blk, LdsBlock<MT>& nx,
                                      const float* __restrict__ Xl, int ldx, int nk0, int lane) {
  constexpr int M = 8 * MT * NT, L = WeightBlock<MT, TRANSPOSED, NT>::kPieces, LX = 2 * MT;
  constexpr int every = M / L > 0 ? M / L : 1;      // one MFMA in `every` is followed by a weight piece
  if (FEEDX) {
#pragma unroll
    for (int p = 0; p < LX; ++p) nx.load_piece(Xl, ldx, nk0, lane, p);
  }
  if (FEED) {
#pragma unroll
    for (int p = 0; p < L; ++p) nb.load_piece(blk, p);
  }
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc.t[mt][nt] = mfma32(x.a[mt][s][j], b.w[nt][4 * s + j], acc.t[mt][nt]);
#pragma unroll
  for (int m = 0; m < M; ++m) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (FEEDX && m < LX) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    if (FEED && m % every == 0 && m / every < L) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
}

struct NoTail { __device__ inline void operator()() const {} };

// four blocks i .. i+3 of the product; LAST: no further weight blocks exist, run tail() instead
template <int MT, bool TRANSPOSED, bool LAST, int NT, class Tail>
__device__ inline void gemm256_group(const float* __restrict__ Xl, int ldx, const float* __restrict__ W, int i,
                                     WeightBlock<MT, TRANSPOSED, NT>& b0, WeightBlock<MT, TRANSPOSED, NT>& b1,
                                     WeightBlock<MT, TRANSPOSED, NT>& b2, WeightBlock<MT, TRANSPOSED, NT>& b3,
                                     LdsBlock<MT>& x0, LdsBlock<MT>& x1, int wave, int lane, Acc<MT, NT>& acc,
                                     Tail& tail) {
  b3.load(W, i + 3, wave, lane);
  x1.load(Xl, ldx, 16 * (i + 1), lane);
  __builtin_amdgcn_sched_barrier(0);
  mfma_block<MT, TRANSPOSED, NT>(x0, b0, acc);
  __builtin_amdgcn_sched_barrier(0);
  if (!LAST) b0.load(W, i + 4, wave, lane); else tail();
  x0.load(Xl, ldx, 16 * (i + 2), lane);
  __builtin_amdgcn_sched_barrier(0);
  mfma_block<MT, TRANSPOSED, NT>(x1, b1, acc);
  __builtin_amdgcn_sched_barrier(0);
  if (!LAST) b1.load(W, i + 5, wave, lane);
  x1.load(Xl, ldx, 16 * (i + 3), lane);
  __builtin_amdgcn_sched_barrier(0);
  mfma_block<MT, TRANSPOSED, NT>(x0, b2, acc);
  __builtin_amdgcn_sched_barrier(0);
  if (!LAST) { b2.load(W, i + 6, wave, lane); x0.load(Xl, ldx, 16 * (i + 4), lane); }
  __builtin_amdgcn_sched_barrier(0);
  mfma_block<MT, TRANSPOSED, NT>(x1, b3, acc);
  __builtin_amdgcn_sched_barrier(0);
}

// the same four blocks with the loads dealt out between the MFMAs; wg: this lane's pointer at block i
template <int MT, bool TRANSPOSED, bool LAST, int NT, class Tail>
__device__ inline void gemm256_group_fed(const float* __restrict__ Xl, int ldx, const float* __restrict__ wg, int i,
                                         WeightBlock<MT, TRANSPOSED, NT>& b0, WeightBlock<MT, TRANSPOSED, NT>& b1,
                                         WeightBlock<MT, TRANSPOSED, NT>& b2, WeightBlock<MT, TRANSPOSED, NT>& b3,
                                         LdsBlock<MT>& x0, LdsBlock<MT>& x1, int lane, Acc<MT, NT>& acc, Tail& tail) {
  constexpr int step = TRANSPOSED ? 16 : 16 * kH;    // floats from one block to the next
  mfma_block_fed<MT, TRANSPOSED, NT, true, true>(x0, b0, acc, b3, wg + 3 * step, x1, Xl, ldx, 16 * (i + 1), lane);
  if (LAST) tail();
  mfma_block_fed<MT, TRANSPOSED, NT, !LAST, true>(x1, b1, acc, b0, wg + 4 * step, x0, Xl, ldx, 16 * (i + 2), lane);
  mfma_block_fed<MT, TRANSPOSED, NT, !LAST, true>(x0, b2, acc, b1, wg + 5 * step, x1, Xl, ldx, 16 * (i + 3), lane);
  mfma_block_fed<MT, TRANSPOSED, NT, !LAST, !LAST>(x1, b3, acc, b2, wg + 6 * step, x0, Xl, ldx, 16 * (i + 4), lane);
}

// FED: the loads of a block are issued between the MFMAs of an earlier one (mfma_block_fed) instead of ahead of them.
template <int MT, bool TRANSPOSED, int NT = 2, bool FED = false, class Tail>
__device__ inline void gemm256(const float* __restrict__ Xl, int ldx, const float* __restrict__ W,
                               WeightBlock<MT, TRANSPOSED, NT>& b0, int wave, int lane, Acc<MT, NT>& acc, Tail tail) {
  WeightBlock<MT, TRANSPOSED, NT> b1, b2, b3;
  LdsBlock<MT> x0, x1;
  b1.load(W, 1, wave, lane);
  b2.load(W, 2, wave, lane);
  x0.load(Xl, ldx, 0, lane);
  POP_MARK(20);
  if (FED) {
    const float* wg = WeightBlock<MT, TRANSPOSED, NT>::lane_base(W, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll 1
    for (int i = 0; i < 12; i += 4) {
      gemm256_group_fed<MT, TRANSPOSED, false, NT>(Xl, ldx, wg, i, b0, b1, b2, b3, x0, x1, lane, acc, tail);
      wg += 4 * (TRANSPOSED ? 16 : 16 * kH);
    }
    gemm256_group_fed<MT, TRANSPOSED, true, NT>(Xl, ldx, wg, 12, b0, b1, b2, b3, x0, x1, lane, acc, tail);
    return;
  }
#pragma unroll 1
  for (int i = 0; i < 12; i += 4) {
    gemm256_group<MT, TRANSPOSED, false, NT>(Xl, ldx, W, i, b0, b1, b2, b3, x0, x1, wave, lane, acc, tail);
    POP_MARK(21 + (i >> 2));
  }
  gemm256_group<MT, TRANSPOSED, true, NT>(Xl, ldx, W, 12, b0, b1, b2, b3, x0, x1, wave, lane, acc, tail);
  POP_MARK(24);
}

// The same product fully unrolled with NB rotating weight buffers (block i + NB - 1 is requested
// before the MFMAs of block i): for operands that come from memory rather than L2 and for
// narrow tiles (NT = 1), where a block is only 512 cycles of matrix work and four buffers
// cover too little latency.  KB: blocks of 16 to contract over (16: all 256; 8: the half that Xl and W point at).
template <int MT, bool TRANSPOSED, int NT, int NB, bool FED = false, int KB = 16, class Tail>
__device__ inline void gemm256_unrolled(const float* __restrict__ Xl, int ldx, const float* __restrict__ W,
                                        WeightBlock<MT, TRANSPOSED, NT>& b0, int wave, int lane, Acc<MT, NT>& acc,
                                        Tail tail) {
  WeightBlock<MT, TRANSPOSED, NT> wb[NB];
  LdsBlock<MT> xb[2];
  wb[0] = b0;
#pragma unroll
  for (int i = 1; i < NB - 1; ++i) wb[i].load(W, i, wave, lane);
  xb[0].load(Xl, ldx, 0, lane);
  if (FED) {                                         // loads between the MFMAs (mfma_block_fed)
    const float* wl = WeightBlock<MT, TRANSPOSED, NT>::lane_base(W, wave, lane);
    constexpr int step = TRANSPOSED ? 16 : 16 * kH;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < KB; ++i) {
      const int n = i + NB - 1;
      if (i == KB - NB + 1) tail();
      if (n < KB) mfma_block_fed<MT, TRANSPOSED, NT, true, true>(xb[i & 1], wb[i % NB], acc, wb[n % NB], wl + n * step, xb[(i + 1) & 1], Xl, ldx, 16 * (i + 1), lane);
      else if (i + 1 < KB) mfma_block_fed<MT, TRANSPOSED, NT, false, true>(xb[i & 1], wb[i % NB], acc, wb[n % NB], wl, xb[(i + 1) & 1], Xl, ldx, 16 * (i + 1), lane);
      else mfma_block_fed<MT, TRANSPOSED, NT, false, false>(xb[i & 1], wb[i % NB], acc, wb[n % NB], wl, xb[(i + 1) & 1], Xl, ldx, 0, lane);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < KB; ++i) {
    if (i + NB - 1 < KB) wb[(i + NB - 1) % NB].load(W, i + NB - 1, wave, lane);
    if (i == KB - NB + 1) tail();
    if (i + 1 < KB) xb[(i + 1) & 1].load(Xl, ldx, 16 * (i + 1), lane);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block<MT, TRANSPOSED, NT>(xb[i & 1], wb[i % NB], acc);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ReLU epilogue of a hidden layer: Y = max(acc + b, 0) goes to LDS (row stride
// kLda) and, when Yg != nullptr, to global memory as [rows][256].  Returns the
// activation pattern of this lane's elements (bb = the two bias values of
// this lane's columns 64 wave + 32 nt + (lane & 31), loaded by the caller ahead of the product), bit (2 mt + nt) 16 + v, so that
// the backward pass can apply ReLU' without re-reading the activations: the
// input-gradient product leaves element (row, col) in the same lane and
// register as the forward product did.
template <int MT, bool THROUGH = false>
__device__ inline uint64_t relu_store(const Acc<MT>& acc, const float (&bb)[2], float* __restrict__ Yl,
                                      float* __restrict__ Yg, int wave, int lane) {
  uint64_t mask = 0;
  const int col = tile_col(wave, 0, lane);           // the lane's two columns go out as one 8-byte store
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 32 * mt + acc_row(v, lane);
      const float h0 = fmaxf(acc.t[mt][0][v] + bb[0], 0.0f), h1 = fmaxf(acc.t[mt][1][v] + bb[1], 0.0f);
      if (h0 > 0.0f) mask |= 1ull << ((2 * mt + 0) * 16 + v);
      if (h1 > 0.0f) mask |= 1ull << ((2 * mt + 1) * 16 + v);
      *reinterpret_cast<f32x2*>(&Yl[row * kLda + col]) = f32x2{h0, h1};
      if (Yg) put2<THROUGH>(Yg + (size_t)row * kH + col, h0, h1);
    }
  return mask;
}

__device__ inline bool mask_bit(uint64_t mask, int mt, int nt, int v) {
  return (mask >> ((2 * mt + nt) * 16 + v)) & 1ull;
}

// Thin products on the vector ALU (heads with 1..8 outputs, action gradient):
// out[r*stride + j] = sum_{c<256} X[r][c] V[j*256 + c],  r < R, j < J <= 8, X and V in LDS.
// Thread t works on rows (t >> 3) + 32 i with column groups 32 q + 4 (t & 7);
// 8 neighbouring lanes share a row and are summed with lane shuffles.
// `stride`: row stride of `outl` (kMaxAct unless the caller keeps wider rows).
template <int R>
__device__ inline void thin_dot(const float* __restrict__ Xl, const float* __restrict__ V, int J,
                                float* __restrict__ outl, int tid, int stride = kMaxAct) {
  const int p = tid & 7;
  for (int i = 0; i < R / 32; ++i) {
    const int r = (tid >> 3) + 32 * i;
    float s[kMaxAct];
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j) s[j] = 0.0f;
#pragma unroll 2
    for (int q = 0; q < 8; ++q) {
      const int c = 32 * q + 4 * p;
      const f32x4 x = *reinterpret_cast<const f32x4*>(&Xl[r * kLda + c]);
#pragma unroll
      for (int j = 0; j < kMaxAct; ++j) {
        if (j < J) {
          const f32x4 w = *reinterpret_cast<const f32x4*>(&V[j * kH + c]);
          s[j] += x[0] * w[0] + x[1] * w[1] + x[2] * w[2] + x[3] * w[3];
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kMaxAct; ++j) {
      if (j < J) {
        float v = s[j];
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 4);
        if (p == 0) outl[r * stride + j] = v;
      }
    }
  }
}

}  // namespace pop
