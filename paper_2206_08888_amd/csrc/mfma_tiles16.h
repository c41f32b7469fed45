// 16-row flavour of the MFMA building blocks, for small populations.
//
// With few agents a launch has fewer workgroups than the chip has CUs, and a layer chain
// is as slow as the matrix pipe of ONE CU lets it be.  Halving the rows per workgroup
// halves the MFMA time of every product and uses twice as many CUs (weights are re-read
// from L2 twice as often, which is free at these sizes).  32x32 tiles would waste half of
// every instruction on 16 rows, so these products run on v_mfma_f32_16x16x4_f32: one
// instruction multiplies a 16x4 slice of A by a 4x16 slice of B into a 16x16 fp32 tile
// held as 4 registers per lane (32 cycles).
//
// Operand layout of that instruction on a 64-lane wavefront (checked against a CPU product):
//   A: lane l supplies A[row = l & 15][k = l >> 4]
//   B: lane l supplies B[k = l >> 4][col = l & 15]
//   D: register v of lane l is D[row = 4 (l >> 4) + v][col = l & 15]
//
// A workgroup is 4 wavefronts; for a [16 x 256] output each wavefront owns the 64 columns
// [64 wave, 64 wave + 64) as 4 tiles, INTERLEAVED: tile nt holds the columns
// 64 wave + 4 c + nt (c = l & 15).  A lane's 4 tiles then sit on 4 consecutive columns, so
//   * the right operand is fetched with 16-byte loads (forward: 4 consecutive columns of
//     one weight row = the 4 tiles' values for one k; backward: 4 consecutive k of one
//     weight row per tile),
//   * results go to LDS / global as 16-byte vectors.
// As in the 32-row flavour the contraction index is visited in the order the loads like:
// within a 16-deep block, MFMA j of a lane group kq = l >> 4 uses k = 16 i + 4 kq + j.
#pragma once
#include "mfma_tiles.h"

namespace pop {

struct Acc16 {
  f32x4 t[4];                                        // [tile nt][v]
  __device__ inline void zero() {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) t[nt] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  }
};

__device__ inline f32x4 mfma16(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

// the weights one lane needs for a 16-deep block
//   forward  (TRANSPOSED = false): w[j][nt] = W[16 i + 4 kq + j][64 wave + 4 c + nt]
//   backward (TRANSPOSED = true):  w[nt][j] = W[64 wave + 4 c + nt][16 i + 4 kq + j]
template <bool TRANSPOSED>
struct WeightBlock16 {
  f32x4 w[4];
  __device__ inline void load(const float* __restrict__ W, int i, int wave, int lane) {
    const int c = lane & 15, kq = lane >> 4;
    if (TRANSPOSED) {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
        w[nt] = *reinterpret_cast<const f32x4*>(W + (64 * wave + 4 * c + nt) * kH + 16 * i + 4 * kq);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        w[j] = *reinterpret_cast<const f32x4*>(W + (16 * i + 4 * kq + j) * kH + 64 * wave + 4 * c);
    }
  }
};

struct LdsBlock16 {                                  // the LDS operand of one block: 4 consecutive k of this lane's row
  f32x4 a;
  __device__ inline void load(const float* __restrict__ Xl, int ldx, int k0, int lane) {
    a = *reinterpret_cast<const f32x4*>(&Xl[(lane & 15) * ldx + k0 + 4 * (lane >> 4)]);
  }
};

template <bool TRANSPOSED>
__device__ inline void mfma_block16(const LdsBlock16& x, const WeightBlock16<TRANSPOSED>& b, Acc16& acc) {
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
      acc.t[nt] = mfma16(x.a[j], TRANSPOSED ? b.w[nt][j] : b.w[j][nt], acc.t[nt]);
}

// 256-deep product of a 16-row LDS operand with a global weight operand, 16 blocks of 16,
// fully unrolled; weight registers rotate through four buffers (block i+3 is requested
// before the MFMAs of block i, about 1500 cycles of matrix work ahead), the LDS operand one
// block ahead.  Block 0 comes from the caller; `tail()` runs once the last weight block has
// been requested, so the caller can start the next layer's loads under the last blocks.
template <bool TRANSPOSED, class Tail>
__device__ inline void gemm256_16(const float* __restrict__ Xl, int ldx, const float* __restrict__ W,
                                  WeightBlock16<TRANSPOSED>& b0, int wave, int lane, Acc16& acc, Tail tail) {
  WeightBlock16<TRANSPOSED> wb[4];
  LdsBlock16 xb[2];
  wb[0] = b0;
  wb[1].load(W, 1, wave, lane);
  wb[2].load(W, 2, wave, lane);
  xb[0].load(Xl, ldx, 0, lane);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (i + 3 < 16) wb[(i + 3) & 3].load(W, i + 3, wave, lane);
    if (i == 13) tail();
    if (i + 1 < 16) xb[(i + 1) & 1].load(Xl, ldx, 16 * (i + 1), lane);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block16<TRANSPOSED>(xb[i & 1], wb[i & 3], acc);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// The transposed product (backward: acc[r][k] += sum_n Z[r][n] W[k][n]) with its weight operand staged through LDS.
// Read straight from memory, that operand is 16 rows of W per quarter of a load instruction, 16 bytes of each: every
// 128-byte line comes through the CU's L1 twice, half used, and a 16-row product, which already asks the L1 for half
// of its bandwidth in the forward direction, takes 7.7 us instead of 4.9.  Here a wavefront fetches its 64 rows of W
// in double blocks of 32 n as whole lines (8 lanes x 16 bytes per row, 8 rows per instruction), parks them in an LDS
// area of its own and reads them back in the MFMA layout.  No barrier: a wavefront reads only what it wrote itself,
// and the LDS serves a wavefront's accesses in order.
//   LDS layout of a double block (two of them per wavefront, kStage16 floats per workgroup): row p = c + 16 nt
//   (holding W[64 wave + 4 c + nt][32 D ..]) at p * 32 floats, its eight 16-byte pieces rotated by p >> 1 -- the 16
//   lanes of a quarter wavefront then hit 64 different banks in the writes (two rows of opposite parity) and in the
//   reads (sixteen rows, one piece each).
constexpr int kStage16Wave = 2 * 64 * 32;            // floats per wavefront: two double blocks
constexpr int kStage16 = 4 * kStage16Wave;           // floats per workgroup (64 KB)
struct WeightStage16 {                               // one double block on its way from memory to LDS
  f32x4 g[8];
  __device__ inline void load(const float* __restrict__ W, int D, int wave, int lane) {
    const int s = lane >> 3, h = lane & 7;
#pragma unroll
    for (int q = 0; q < 8; ++q)                      // rows p = 8 q + s: c = 8 (q & 1) + s, nt = q >> 1
      g[q] = *reinterpret_cast<const f32x4*>(W + (64 * wave + 4 * (8 * (q & 1) + s) + (q >> 1)) * kH + 32 * D + 4 * h);
  }
  __device__ inline void put(float* __restrict__ stage_wave, int D, int lane) const {
    const int s = lane >> 3, h = lane & 7;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int p = 8 * q + s;
      *reinterpret_cast<f32x4*>(stage_wave + (D & 1) * 2048 + p * 32 + 4 * ((h + (p >> 1)) & 7)) = g[q];
    }
  }
};
// block i (16 n) of the staged operand in the MFMA layout: w[nt][j] = W[64 wave + 4 c + nt][16 i + 4 kq + j]
__device__ inline void staged_block16(WeightBlock16<true>& b, const float* __restrict__ stage_wave, int i, int lane) {
  const int c = lane & 15, kq = lane >> 4;
  const float* base = stage_wave + ((i >> 1) & 1) * 2048 + c * 32 + 4 * ((4 * (i & 1) + kq + (c >> 1)) & 7);
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) b.w[nt] = *reinterpret_cast<const f32x4*>(base + 16 * 32 * nt);
}
// g0: double block 0, requested by the caller as early as it can (with double block 1 as well the chains measured
// slower: 64 more registers held across the product before); `stage`: the workgroup's kStage16 floats; tail() runs
// once the last double block has been requested.
template <class Tail>
__device__ inline void gemm256_16_staged(const float* __restrict__ Xl, int ldx, const float* __restrict__ W,
                                         const WeightStage16& g0, float* __restrict__ stage, int wave, int lane, Acc16& acc,
                                         Tail tail) {
  float* sw = stage + wave * kStage16Wave;
  WeightStage16 g[3];                                // double blocks D + 1 .. D + 3 in flight
  WeightBlock16<true> wb[2];
  LdsBlock16 xb[2];
  g[0] = g0;
  g[1].load(W, 1, wave, lane);
  g[2].load(W, 2, wave, lane);
  g[0].put(sw, 0, lane);
  staged_block16(wb[0], sw, 0, lane);
  xb[0].load(Xl, ldx, 0, lane);
#pragma unroll
  for (int D = 0; D < 8; ++D) {
    if (D + 3 < 8) g[D % 3].load(W, D + 3, wave, lane);        // its registers were parked in LDS one round ago
    if (D == 5) tail();
    staged_block16(wb[1], sw, 2 * D + 1, lane);
    xb[1].load(Xl, ldx, 16 * (2 * D + 1), lane);
    __builtin_amdgcn_sched_barrier(0);
    mfma_block16<true>(xb[0], wb[0], acc);
    __builtin_amdgcn_sched_barrier(0);
    if (D + 1 < 8) {
      g[(D + 1) % 3].put(sw, D + 1, lane);           // requested two rounds ago (the first two: at the start)
      staged_block16(wb[0], sw, 2 * D + 2, lane);
      xb[0].load(Xl, ldx, 16 * (2 * D + 2), lane);
    }
    __builtin_amdgcn_sched_barrier(0);
    mfma_block16<true>(xb[1], wb[1], acc);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// First-layer weights for the leading 32 rows of W (two blocks), fetched ahead of time;
// rows at or beyond the fan-in K read as zero.
struct SmallW16 {
  f32x4 w[2][4];
  __device__ inline void load(const float* __restrict__ W, int K, int wave, int lane) {
    const int c = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = 16 * i + 4 * kq + j;
        const f32x4 v = *reinterpret_cast<const f32x4*>(W + (k < K ? k : 0) * kH + 64 * wave + 4 * c);
        w[i][j] = k < K ? v : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      }
  }
};

// acc[r][c] += sum_{k<K} X[r][k] W[k][c] for a small fan-in K <= 64.
//   X: LDS, row stride ldx, 16 rows; columns K .. roundup16(K)-1 must hold finite values
//      (they meet zero weights);  W: global, row-major [K][256]; `pre` holds rows 0..31.
__device__ inline void gemm_xw_small16(const float* __restrict__ Xl, int ldx, int K, const float* __restrict__ W,
                                       const SmallW16& pre, int wave, int lane, Acc16& acc) {
  const int c = lane & 15, kq = lane >> 4;
  const int K16 = (K + 15) & ~15;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (16 * i < K16) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(&Xl[c * ldx + 16 * i + 4 * kq]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc.t[nt] = mfma16(a[j], pre.w[i][j][nt], acc.t[nt]);
    }
  }
  for (int k0 = 32; k0 < K16; k0 += 16) {            // fan-in beyond 32: plain loop
    f32x4 b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + 4 * kq + j;
      const f32x4 v = *reinterpret_cast<const f32x4*>(W + (size_t)(k < K ? k : 0) * kH + 64 * wave + 4 * c);
      b[j] = k < K ? v : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    const f32x4 a = *reinterpret_cast<const f32x4*>(&Xl[c * ldx + k0 + 4 * kq]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) acc.t[nt] = mfma16(a[j], b[j][nt], acc.t[nt]);
  }
}

// The same product for a fan-in of several hundred: the blocks beyond the prefetched 32 rows are
// software-pipelined, four weight blocks (64 rows of W) in flight ahead of the matrix pipe.
__device__ inline void gemm_xw_deep16(const float* __restrict__ Xl, int ldx, int K, const float* __restrict__ W,
                                      const SmallW16& pre, int wave, int lane, Acc16& acc) {
  constexpr int PF = 4;
  const int c = lane & 15, kq = lane >> 4;
  const int nb = (K + 15) >> 4;                      // 16-deep blocks in all; 0 and 1 come from `pre`
  const float* wcol = W + 64 * wave + 4 * c;
  f32x4 b[PF][4];
  auto request = [&](f32x4 (&dst)[4], int blk) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = 16 * blk + 4 * kq + j;
      const f32x4 v = *reinterpret_cast<const f32x4*>(wcol + (size_t)(k < K ? k : 0) * kH);
      dst[j] = k < K ? v : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
  };
#pragma unroll
  for (int s = 0; s < PF; ++s)
    if (2 + s < nb) request(b[s], 2 + s);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (i < nb) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(&Xl[c * ldx + 16 * i + 4 * kq]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc.t[nt] = mfma16(a[j], pre.w[i][j][nt], acc.t[nt]);
    }
  }
  f32x4 an = {0.0f, 0.0f, 0.0f, 0.0f};               // the LDS operand runs one block ahead of the matrix pipe
  if (2 < nb) an = *reinterpret_cast<const f32x4*>(&Xl[c * ldx + 16 * 2 + 4 * kq]);
  // FAST: block i + PF lies wholly inside the K rows: its four loads are one running pointer plus constants
  const float* wrun = wcol + (size_t)(16 * (2 + PF) + 4 * kq) * kH;      // rows of block 2 + PF for this lane
  auto step = [&](int s, int i, bool next_x, bool next_w, bool fast) {
    const f32x4 a = an;
    if (next_x) an = *reinterpret_cast<const f32x4*>(&Xl[c * ldx + 16 * (i + 1) + 4 * kq]);
    f32x4 w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = b[s][j];
    if (fast) {
#pragma unroll
      for (int j = 0; j < 4; ++j) b[s][j] = *reinterpret_cast<const f32x4*>(wrun + j * kH);
    } else if (next_w) {
      request(b[s], i + PF);
    }
    wrun += 16 * kH;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) acc.t[nt] = mfma16(a[j], w[j][nt], acc.t[nt]);
    __builtin_amdgcn_sched_barrier(0);
  };
  int blk = 2;
  // steady state, free of branches (a branch inside the loop makes the compiler drain every outstanding load at
  // the join): every block of the group exists and every block requested from it is a full one
  const int nfull = K >> 4;
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

// ReLU epilogue: Y = max(acc + b, 0) to LDS (row stride kLda) and, when Yg != nullptr, to
// global memory as [rows][256]; bb = biases of this lane's 4 columns.  Returns the
// activation pattern, bit 4 nt + v; the backward product leaves element (row, col) in the
// same lane and register.
template <bool THROUGH = false>
__device__ inline uint64_t relu_store16(const Acc16& acc, const f32x4& bb, float* __restrict__ Yl, float* __restrict__ Yg,
                                        int wave, int lane) {
  const int c = lane & 15, kq = lane >> 4;
  uint64_t mask = 0;
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    f32x4 o;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      o[nt] = fmaxf(acc.t[nt][v] + bb[nt], 0.0f);
      if (o[nt] > 0.0f) mask |= 1ull << (4 * nt + v);
    }
    const int row = 4 * kq + v, col = 64 * wave + 4 * c;
    *reinterpret_cast<f32x4*>(&Yl[row * kLda + col]) = o;
    if (Yg) {
      if (THROUGH) {
        put2<true>(Yg + (size_t)row * kH + col, o[0], o[1]);
        put2<true>(Yg + (size_t)row * kH + col + 2, o[2], o[3]);
      } else {
        *reinterpret_cast<f32x4*>(Yg + (size_t)row * kH + col) = o;
      }
    }
  }
  return mask;
}

// Narrow products on the matrix pipe, weights straight from global memory (no LDS staging):
//   head_mfma:   out[r*stride + j] = sum_{c<256} X[r][c] W[c*J + j]      (W: [256][J], a network's head)
//   head_mfma_t: out[r*stride + j] = sum_{c<256} X[r][c] W[j*256 + c]    (W: J rows of 256)
// r < R (a multiple of 16), j < J; X in LDS with row stride kLda.  The output is cut into 16x16 tiles,
// dealt round-robin to the 4 wavefronts; a tile's 256-deep product is 64 v_mfma_f32_16x16x4_f32, its
// weights requested in one go (head_mfma: in two halves) ahead of the products.  Columns at or beyond J are neither read nor
// written.  The tile loop is controlled by a scalar (readfirstlane of the wavefront index): written on
// the per-lane value, the compiler wraps the matrix instructions in an EXEC-masked loop, and one build of
// that form produced wrong sums.
template <int R>
__device__ inline void head_mfma(const float* __restrict__ Xl, const float* __restrict__ W, int J, float* __restrict__ outl,
                                 int stride, int wave, int lane) {
  constexpr int RT = R / 16;
  const int c = lane & 15, kq = lane >> 4;
  const int tiles = RT * ((J + 15) >> 4);
  for (int tile = __builtin_amdgcn_readfirstlane(wave); tile < tiles; tile += kThreads / 64) {
    const int rt = tile % RT, col = 16 * (tile / RT) + c;
    const bool ok = col < J;
    const float* wp = W + (ok ? col : 0) + (size_t)(4 * kq) * J;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int h = 0; h < 2; ++h) {                    // two halves of 128 rows: 32 weight registers at a time
      float b[8][4];
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) b[i][j] = wp[(size_t)(16 * (8 * h + i) + j) * J];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(&Xl[(16 * rt + c) * kLda + 16 * (8 * h + i) + 4 * kq]);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = mfma16(a[j], ok ? b[i][j] : 0.0f, acc);
      }
    }
    if (ok) {
#pragma unroll
      for (int v = 0; v < 4; ++v) outl[(16 * rt + 4 * kq + v) * stride + col] = acc[v];
    }
  }
}

template <int R>
__device__ inline void head_mfma_t(const float* __restrict__ Xl, const float* __restrict__ W, int J, float* __restrict__ outl,
                                   int stride, int wave, int lane) {
  constexpr int RT = R / 16;
  const int c = lane & 15, kq = lane >> 4;
  const int tiles = RT * ((J + 15) >> 4);
  for (int tile = __builtin_amdgcn_readfirstlane(wave); tile < tiles; tile += kThreads / 64) {
    const int rt = tile % RT, col = 16 * (tile / RT) + c;
    const bool ok = col < J;
    const float* wp = W + (size_t)(ok ? col : 0) * kH + 4 * kq;
    f32x4 b[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) b[i] = *reinterpret_cast<const f32x4*>(wp + 16 * i);
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(&Xl[(16 * rt + c) * kLda + 16 * i + 4 * kq]);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = mfma16(a[j], ok ? b[i][j] : 0.0f, acc);
    }
    if (ok) {
#pragma unroll
      for (int v = 0; v < 4; ++v) outl[(16 * rt + 4 * kq + v) * stride + col] = acc[v];
    }
  }
}

// The same two products with the contraction split over the four wavefronts (64 deep each), for heads of at most
// 16 columns on 16 or 32 rows: dealt out as whole tiles only one or two wavefronts would work, each through 64
// MFMAs that wait for one another (2 us; 0.7 this way).  BY_ROWS: W as for head_mfma_t, else as for head_mfma.
// The partial tiles meet in LDS (red: [R / 16][4][16][16] floats) and are added in wavefront order.  Contains a
// workgroup barrier; the caller still places one before `outl` is read.
constexpr int kHeadRed = 2 * 4 * 256;                // floats of `red` for R <= 32
template <int R, bool BY_ROWS>
__device__ inline void head_mfma_split(const float* __restrict__ Xl, const float* __restrict__ W, int J,
                                       float* __restrict__ outl, int stride, int wave, int lane, float* __restrict__ red) {
  static_assert(R == 16 || R == 32, "wider tiles keep every wavefront busy as whole tiles");
  constexpr int RT = R / 16;
  const int c = lane & 15, kq = lane >> 4;
  const bool ok = c < J;
  const int k0 = 64 * wave + 4 * kq;                 // MFMA j of block i contracts k = k0 + 16 i + j
  f32x4 b[4];
  if (BY_ROWS) {
    const float* wp = W + (size_t)(ok ? c : 0) * kH + k0;
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = *reinterpret_cast<const f32x4*>(wp + 16 * i);
  } else {
    const float* wp = W + (ok ? c : 0) + (size_t)k0 * J;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) b[i][j] = wp[(size_t)(16 * i + j) * J];
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    f32x4 acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(&Xl[(16 * rt + c) * kLda + k0 + 16 * i]);
      acc0 = mfma16(a[0], ok ? b[i][0] : 0.0f, acc0);
      acc1 = mfma16(a[1], ok ? b[i][1] : 0.0f, acc1);
      acc0 = mfma16(a[2], ok ? b[i][2] : 0.0f, acc0);
      acc1 = mfma16(a[3], ok ? b[i][3] : 0.0f, acc1);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) red[((rt * 4 + wave) * 16 + 4 * kq + v) * 16 + c] = acc0[v] + acc1[v];
  }
  __syncthreads();
  const int row = (64 * wave + lane) >> 4;           // 256 threads: one element of each row tile
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const float* p = red + (rt * 4 * 16 + row) * 16 + c;
    const float sum = ((p[0] + p[256]) + p[512]) + p[768];
    if (ok) outl[(16 * rt + row) * stride + c] = sum;
  }
}

__device__ inline bool mask_bit16(uint64_t mask, int nt, int v) { return (mask >> (4 * nt + v)) & 1ull; }

// Thin products for 16 rows: out[r*stride + j] = sum_{c<256} X[r][c] V[j*256 + c], r < 16, j < J <= 8.
// Thread t works on row t >> 4 with the column groups 64 q + 4 (t & 15); the 16 lanes of a
// row are summed with lane shuffles.
__device__ inline void thin_dot16(const float* __restrict__ Xl, const float* __restrict__ V, int J,
                                  float* __restrict__ outl, int tid, int stride = kMaxAct) {
  const int p = tid & 15, r = tid >> 4;
  float s[kMaxAct];
#pragma unroll
  for (int j = 0; j < kMaxAct; ++j) s[j] = 0.0f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = 64 * q + 4 * p;
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
      v += __shfl_xor(v, 8);
      if (p == 0) outl[r * stride + j] = v;
    }
  }
}

}  // namespace pop
