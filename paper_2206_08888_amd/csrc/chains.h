// Fused forward/backward chains of one TD3 update step (Sec. 4.1 of the paper:
// every population member takes the ordinary TD3 update on its own batch).
//
// The batch of an agent is cut into row chunks of R = 16, 32 or 64 rows (the tile
// geometries below).  One
// workgroup owns one (agent or network, chunk) and walks the whole layer chain
// for its rows with the activations resident in LDS; only what the
// weight-gradient kernel needs later (layer inputs and pre-activation
// gradients) is written to global memory.  Rows of a batch interact only
// through the weight gradients, which are contracted over the full batch by a
// separate kernel, so chunks need no communication here.
//
//   target_chain : s' -> target actor -> smoothing noise -> twin target critics -> y
//   critic_chain : [s, a] -> critic k forward -> MSE seed gradient -> backward to
//              the pre-activation gradients of layers 2 and 1
//   actor_chain  : s -> actor -> a_pi -> critic 1 forward -> gradient w.r.t. the
//              action -> actor backward
//
// LDS economy: a hidden layer overwrites its own input tile (all wavefronts
// finish reading, barrier, then write) and ReLU patterns travel from the
// forward to the backward product as bit masks in registers, so one 256-wide
// tile per workgroup is enough.  Latency economy: everything a layer needs
// from memory (its first-layer weights, the first weight block of its hidden
// layer, its biases) is requested while the previous product is still on the
// matrix unit, and the small head vectors are staged in LDS when the kernel
// starts.
//
// The chains are device functions: k_chain.hip wraps each into a kernel of its own, and
// k_step.hip runs all of them, with the weight-gradient tiles, inside one launch per step.
#pragma once
#include "launch.h"
#include "mfma_tiles16.h"
#include "rng.h"

#ifndef POP_ONE_TRIP
#define POP_ONE_TRIP 1
#endif

namespace pop {

static_assert(kMaxAct == 8, "the action-gradient loops read dz3 rows as two 16-byte vectors");

namespace {

// LDS map (floats): input tile [R][xld] | activation tile [R][kLda] | NS x [R][8] scratch | vectors.
// KPAD: the first-layer product reads the input tile in blocks of KPAD columns.
template <int R_, int KPAD>
struct LdsMap {
  static constexpr int R = R_;
  int xld, buf, s0, s1, s2, vec;
  // NS: number of [R][8] scratch regions (s0, s1, s2, and for the SAC chains six more after them)
  __host__ __device__ LdsMap(int fan_in, int NS = 3) {
    xld = ((fan_in + KPAD - 1) / KPAD) * KPAD + 4;   // 4 * odd words: conflict-free 16-byte row reads
    buf = R * xld;
    s0 = buf + R * kLda;
    s1 = s0 + R * kMaxAct;
    s2 = s1 + R * kMaxAct;
    vec = s0 + NS * R * kMaxAct;
  }
  __host__ __device__ int s(int i) const { return s0 + i * R * kMaxAct; }
  __host__ size_t bytes(int vec_floats) const { return (size_t)(vec + vec_floats) * sizeof(float); }
};
template <int MT>
using Lds = LdsMap<32 * MT, 8>;

// what a two-hidden-layer network needs from memory before its products can start
template <int MT>
struct LayerPre {
  SmallW w1;                       // first-layer weights
  WeightBlock<MT, false> w2;       // block 0 of the hidden layer
  float b1[2], b2[2];              // biases of this lane's columns
  __device__ inline void load(const float* __restrict__ net, const NetLayout& L, int wave, int lane) {
    w1.load(net + L.w1, L.in, wave, lane);
    w2.load(net + L.w2, 0, wave, lane);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      b1[nt] = net[L.b1 + tile_col(wave, nt, lane)];
      b2[nt] = net[L.b2 + tile_col(wave, nt, lane)];
    }
  }
};

// Copy columns [c0, c0 + n) of R batch rows into the LDS input tile at columns
// [0, n), zero the remaining columns; rows at or beyond `valid` become zero.
template <int R>
__device__ inline void load_input(float* Xl, int xld, const float* rows, int row_stride, int c0, int n, int valid,
                                  int tid) {
  for (int e = tid; e < R * xld; e += kThreads) {
    const int r = e / xld, c = e - r * xld;
    Xl[e] = (c < n && r < valid) ? rows[(size_t)r * row_stride + c0 + c] : 0.0f;
  }
}

// The same for wide rows: wavefront w takes the rows w, w + 4, ..., its lanes consecutive columns
// (coalesced, no index division, every load independent of the others).
template <int R>
__device__ inline void load_input_wide(float* Xl, int xld, const float* rows, int row_stride, int c0, int n, int valid,
                                       int tid) {
  constexpr int RW = R / (kThreads / 64);            // rows per wavefront
  const int wave = tid >> 6, lane = tid & 63;
#pragma unroll 2
  for (int c = lane; c < xld; c += 64) {             // RW (x2) loads in flight per lane
    float v[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int r = wave + (kThreads / 64) * i;
      v[i] = rows[(size_t)(r < valid ? r : 0) * row_stride + c0 + (c < n ? c : 0)];
    }
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int r = wave + (kThreads / 64) * i;
      Xl[r * xld + c] = (r < valid && c < n) ? v[i] : 0.0f;
    }
  }
}

// Copies into LDS ahead of a chain.  The loads of a thread are requested eight at a time before the
// first of them is used: as a plain loop every element would wait out its own trip to memory.
__device__ inline void stage_vector(float* dst, const float* __restrict__ src, int n, int tid) {
  constexpr int U = 8;
  for (int e0 = tid; e0 < n; e0 += U * kThreads) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = e0 + u * kThreads;
      v[u] = src[e < n ? e : n - 1];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = e0 + u * kThreads;
      if (e < n) dst[e] = v[u];
    }
  }
}

// The same copy in two halves, for chain prologues: fetch() requests the values into registers, put() writes
// them to LDS.  A prologue calls every fetch() before the first put(), so that all it needs from memory is under
// way at once; as separate load-then-store loops each vector and the input tile wait out a trip to memory of their own
// (five in a row at the head of a target chain: 2.8 us).  One element per thread: n <= kThreads.
struct SmallVec {
  float v;
  __device__ inline void fetch(const float* __restrict__ src, int n, int tid) { v = src[tid < n ? tid : 0]; }
  __device__ inline void put(float* dst, int n, int tid) const { if (tid < n) dst[tid] = v; }
};

// The input tile of a chain (columns [c0, c0 + n) of R batch rows into columns [0, n) of the LDS tile, the rest
// zero) in the same two halves; for the narrow inputs (row stride of the tile at most kMaxIn + 4).
template <int R>
struct InputTile {
  static constexpr int IT = (R * (kMaxIn + 4) + kThreads - 1) / kThreads;
  float v[IT];
  __device__ inline void fetch(int xld, const float* __restrict__ rows, int row_stride, int c0, int n, int valid, int tid) {
#pragma unroll
    for (int i = 0; i < IT; ++i) {
      const int e = tid + i * kThreads;
      const int r = e / xld, c = e - r * xld;
      const bool in = e < R * xld && c < n && r < valid;
      const float x = rows[in ? (size_t)r * row_stride + c0 + c : (size_t)c0];
      v[i] = in ? x : 0.0f;
    }
  }
  __device__ inline void put(float* Xl, int xld, int tid) const {
#pragma unroll
    for (int i = 0; i < IT; ++i) {
      const int e = tid + i * kThreads;
      if (e < R * xld) Xl[e] = v[i];
    }
  }
};

// Stage a head weight W3[256][J] as J rows of 256 (so that the thin products read it with
// 16-byte LDS loads like any other row vector); thread c moves the J weights of hidden unit c.
static_assert(kThreads == kH, "stage_head: one thread per hidden unit");
__device__ inline void stage_head(float* dst, const float* __restrict__ src, int J, int tid) {
  constexpr int U = 8;
  const float* row = src + tid * J;
  for (int j0 = 0; j0 < J; j0 += U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = row[j0 + u < J ? j0 + u : J - 1];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (j0 + u < J) dst[(j0 + u) * kH + tid] = v[u];
  }
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// First layer from the input tile into `Yl` (+ optional global copy); returns the ReLU pattern.
template <int MT, bool THROUGH = false>
__device__ inline uint64_t first_layer(const float* Xs, int xld, const float* net, const NetLayout& L,
                                       const LayerPre<MT>& pre, float* Yl, float* Yg, int wave, int lane) {
  Acc<MT> acc;
  acc.zero();
  gemm_xw_small<MT>(Xs, xld, L.in, net + L.w1, pre.w1, wave, lane, acc);
  return relu_store<MT, THROUGH>(acc, pre.b1, Yl, Yg, wave, lane);
}

// Hidden layer in place on `buf`; `tail` is handed to the product (see gemm256).
template <int MT, bool THROUGH = false, bool FED = false, class Tail>
__device__ inline uint64_t hidden_layer(float* buf, const float* net, const NetLayout& L, LayerPre<MT>& pre,
                                        float* Yg, int wave, int lane, Tail tail) {
  Acc<MT> acc;
  acc.zero();
  const float bb[2] = {pre.b2[0], pre.b2[1]};
  gemm256<MT, false, 2, FED>(buf, kLda, net + L.w2, pre.w2, wave, lane, acc, tail);
  __syncthreads();                                   // every wavefront has read the input tile
  return relu_store<MT, THROUGH>(acc, bb, buf, Yg, wave, lane);
}

// dX = (dZ W^T) * mask written to global [rows][256]; column sums of the result
// (over this workgroup's rows) go to colsum_out[256].
template <int MT, bool THROUGH = false, bool FED = false>
__device__ inline void input_grad_to_global(const float* Zl, const float* W, WeightBlock<MT, true>& w0, uint64_t mask,
                                            float* __restrict__ dXg, float* __restrict__ colsum_out, int wave,
                                            int lane) {
  Acc<MT> acc;
  acc.zero();
  gemm256<MT, true, 2, FED>(Zl, kLda, W, w0, wave, lane, acc, NoTail());
  float cs[2] = {0.0f, 0.0f};
  const int col = tile_col(wave, 0, lane);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float z0 = mask_bit(mask, mt, 0, v) ? acc.t[mt][0][v] : 0.0f;
      const float z1 = mask_bit(mask, mt, 1, v) ? acc.t[mt][1][v] : 0.0f;
      put2<THROUGH>(dXg + (32 * mt + acc_row(v, lane)) * kH + col, z0, z1);
      cs[0] += z0;
      cs[1] += z1;
    }
  const float t0 = cs[0] + __shfl_xor(cs[0], 32), t1 = cs[1] + __shfl_xor(cs[1], 32);
  if (lane < 32) put2<THROUGH>(colsum_out + col, t0, t1);
}

// ---------------------------------------------------------------------------------------------
// Tile geometries of a chain: what the chains below need from a geometry G is
//   G::R, G::kPad, G::Pre (prefetch record with load()), G::WtBlock + G::load_wt (block 0 of a
//   transposed weight operand), first_layer, hidden_layer, input_grad_to_global,
//   input_grad_to_lds, thin (thin products on the vector ALU).
// FED: the 256-deep products issue their loads between the MFMAs (mfma_tiles.h) -- for kernels that run two
// workgroups per CU.
template <int MT, bool FED = false>
struct Rows32 {                                      // 32 MT rows on v_mfma_f32_32x32x2_f32 (mfma_tiles.h)
  static constexpr int R = 32 * MT, kPad = 8;
  using Pre = LayerPre<MT>;
  using WtBlock = WeightBlock<MT, true>;
  static constexpr int kStage = 0;                   // no LDS staging of weights (`stage` arguments are unused)
  __device__ static inline void load_wt(WtBlock& wt, const float* W, int wave, int lane) { wt.load(W, 0, wave, lane); }
  __device__ static inline void load_input(float* Xl, int xld, const float* rows, int row_stride, int c0, int n, int valid,
                                           int tid) {
    pop::load_input<R>(Xl, xld, rows, row_stride, c0, n, valid, tid);
  }
  template <bool THROUGH>
  __device__ static inline uint64_t first_layer(const float* Xs, int xld, const float* net, const NetLayout& L,
                                                const Pre& pre, float* Yl, float* Yg, int wave, int lane) {
    return pop::first_layer<MT, THROUGH>(Xs, xld, net, L, pre, Yl, Yg, wave, lane);
  }
  template <bool THROUGH, class Tail>
  __device__ static inline uint64_t hidden_layer(float* buf, const float* net, const NetLayout& L, Pre& pre, float* Yg,
                                                 int wave, int lane, Tail tail) {
    return pop::hidden_layer<MT, THROUGH, FED>(buf, net, L, pre, Yg, wave, lane, tail);
  }
  template <bool THROUGH>
  __device__ static inline void input_grad_to_global(const float* Zl, const float* W, WtBlock& w0, uint64_t mask,
                                                     float* dXg, float* colsum_out, int wave, int lane, float*) {
    pop::input_grad_to_global<MT, THROUGH, FED>(Zl, W, w0, mask, dXg, colsum_out, wave, lane);
  }
  // buf <- (buf W^T) * mask in place; tail() as in gemm256
  template <class Tail>
  __device__ static inline void input_grad_to_lds(float* buf, const float* W, WtBlock& wt, uint64_t mask, int wave,
                                                  int lane, Tail tail, float*) {
    Acc<MT> acc;
    acc.zero();
    gemm256<MT, true, 2, FED>(buf, kLda, W, wt, wave, lane, acc, tail);
    __syncthreads();                                 // every wavefront is done reading the operand
    const int col = tile_col(wave, 0, lane);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        *reinterpret_cast<f32x2*>(&buf[(32 * mt + acc_row(v, lane)) * kLda + col]) =
            f32x2{mask_bit(mask, mt, 0, v) ? acc.t[mt][0][v] : 0.0f, mask_bit(mask, mt, 1, v) ? acc.t[mt][1][v] : 0.0f};
  }
  __device__ static inline void thin(const float* Xl, const float* V, int J, float* outl, int tid, int stride = kMaxAct) {
    thin_dot<R>(Xl, V, J, outl, tid, stride);
  }
  // buf[row][col] = mask ? rowvec[row] * colvec[col] : 0  (mask as returned by hidden_layer)
  __device__ static inline void store_outer_masked(float* buf, uint64_t mask, const float* rowvec, const float* colvec,
                                                   int wave, int lane) {
    const int col = tile_col(wave, 0, lane);
    const f32x2 cv = *reinterpret_cast<const f32x2*>(&colvec[col]);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 32 * mt + acc_row(v, lane);
        const float rv = rowvec[row];
        *reinterpret_cast<f32x2*>(&buf[row * kLda + col]) =
            f32x2{mask_bit(mask, mt, 0, v) ? rv * cv[0] : 0.0f, mask_bit(mask, mt, 1, v) ? rv * cv[1] : 0.0f};
      }
  }
};

struct Rows16 {                                      // 16 rows on v_mfma_f32_16x16x4_f32 (mfma_tiles16.h)
  static constexpr int R = 16, kPad = 16;
  struct Pre {
    SmallW16 w1;
    WeightBlock16<false> w2;
    f32x4 b1, b2;                                    // biases of this lane's 4 columns
    __device__ inline void load(const float* __restrict__ net, const NetLayout& L, int wave, int lane) {
      w1.load(net + L.w1, L.in, wave, lane);
      w2.load(net + L.w2, 0, wave, lane);
      b1 = *reinterpret_cast<const f32x4*>(net + L.b1 + 64 * wave + 4 * (lane & 15));
      b2 = *reinterpret_cast<const f32x4*>(net + L.b2 + 64 * wave + 4 * (lane & 15));
    }
  };
  using WtBlock = WeightStage16;                     // the transposed products stage their weights through LDS
  static constexpr int kStage = kStage16;            // floats of LDS they need for that
  __device__ static inline void load_wt(WtBlock& wt, const float* W, int wave, int lane) { wt.load(W, 0, wave, lane); }
  __device__ static inline void load_input(float* Xl, int xld, const float* rows, int row_stride, int c0, int n, int valid,
                                           int tid) {
    pop::load_input<R>(Xl, xld, rows, row_stride, c0, n, valid, tid);
  }
  template <bool THROUGH>
  __device__ static inline uint64_t first_layer(const float* Xs, int xld, const float* net, const NetLayout& L,
                                                const Pre& pre, float* Yl, float* Yg, int wave, int lane) {
    Acc16 acc;
    acc.zero();
    gemm_xw_small16(Xs, xld, L.in, net + L.w1, pre.w1, wave, lane, acc);
    return relu_store16<THROUGH>(acc, pre.b1, Yl, Yg, wave, lane);
  }
  template <bool THROUGH, class Tail>
  __device__ static inline uint64_t hidden_layer(float* buf, const float* net, const NetLayout& L, Pre& pre, float* Yg,
                                                 int wave, int lane, Tail tail) {
    Acc16 acc;
    acc.zero();
    const f32x4 bb = pre.b2;
    gemm256_16<false>(buf, kLda, net + L.w2, pre.w2, wave, lane, acc, tail);
    __syncthreads();                                 // every wavefront has read the input tile
    return relu_store16<THROUGH>(acc, bb, buf, Yg, wave, lane);
  }
  template <bool THROUGH>
  __device__ static inline void input_grad_to_global(const float* Zl, const float* W, WtBlock& w0, uint64_t mask,
                                                     float* __restrict__ dXg, float* __restrict__ colsum_out, int wave,
                                                     int lane, float* stage) {
    Acc16 acc;
    acc.zero();
    gemm256_16_staged(Zl, kLda, W, w0, stage, wave, lane, acc, NoTail());
    const int c = lane & 15, kq = lane >> 4;
    float cs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int v = 0; v < 4; ++v) {                    // the lane's four columns are neighbours: two 8-byte stores per row
      float z[4];
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        z[nt] = mask_bit16(mask, nt, v) ? acc.t[nt][v] : 0.0f;
        cs[nt] += z[nt];
      }
      float* p = dXg + (4 * kq + v) * kH + 64 * wave + 4 * c;
      put2<THROUGH>(p, z[0], z[1]);
      put2<THROUGH>(p + 2, z[2], z[3]);
    }
    float tot[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      tot[nt] = cs[nt] + __shfl_xor(cs[nt], 16);
      tot[nt] += __shfl_xor(tot[nt], 32);
    }
    if (lane < 16) {
      put2<THROUGH>(colsum_out + 64 * wave + 4 * c, tot[0], tot[1]);
      put2<THROUGH>(colsum_out + 64 * wave + 4 * c + 2, tot[2], tot[3]);
    }
  }
  template <class Tail>
  __device__ static inline void input_grad_to_lds(float* buf, const float* W, WtBlock& wt, uint64_t mask, int wave,
                                                  int lane, Tail tail, float* stage) {
    Acc16 acc;
    acc.zero();
    gemm256_16_staged(buf, kLda, W, wt, stage, wave, lane, acc, tail);
    __syncthreads();
    const int c = lane & 15, kq = lane >> 4;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      f32x4 o;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) o[nt] = mask_bit16(mask, nt, v) ? acc.t[nt][v] : 0.0f;
      *reinterpret_cast<f32x4*>(&buf[(4 * kq + v) * kLda + 64 * wave + 4 * c]) = o;
    }
  }
  __device__ static inline void thin(const float* Xl, const float* V, int J, float* outl, int tid, int stride = kMaxAct) {
    thin_dot16(Xl, V, J, outl, tid, stride);
  }
  // The ReLU pattern first_layer / hidden_layer return, rebuilt from the layer's output Hg[16][256] in global memory
  __device__ static inline uint64_t mask_from_global(const float* __restrict__ Hg, int wave, int lane) {
    const int c = lane & 15, kq = lane >> 4;
    f32x4 h[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) h[v] = *reinterpret_cast<const f32x4*>(Hg + (4 * kq + v) * kH + 64 * wave + 4 * c);
    uint64_t mask = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
        if (h[v][nt] > 0.0f) mask |= 1ull << (4 * nt + v);
    return mask;
  }
  __device__ static inline void store_outer_masked(float* buf, uint64_t mask, const float* rowvec, const float* colvec,
                                                   int wave, int lane) {
    const int c = lane & 15, kq = lane >> 4;
    const f32x4 cv = *reinterpret_cast<const f32x4*>(&colvec[64 * wave + 4 * c]);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 4 * kq + v;
      const float rv = rowvec[row];
      f32x4 o;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) o[nt] = mask_bit16(mask, nt, v) ? rv * cv[nt] : 0.0f;
      *reinterpret_cast<f32x4*>(&buf[row * kLda + 64 * wave + 4 * c]) = o;
    }
  }
};

// The same tiles for first layers with a fan-in of several hundred (the SAC Humanoid shapes): only the
// first-layer product differs (software-pipelined beyond the prefetched rows).
// PF: weight blocks of 8 rows in flight; 8 where the registers allow it (the critic chain), else 4.
template <int MT, int PF = 4>
struct Rows32Deep : Rows32<MT> {
  using Pre = typename Rows32<MT>::Pre;
  __device__ static inline void load_input(float* Xl, int xld, const float* rows, int row_stride, int c0, int n, int valid,
                                           int tid) {
    load_input_wide<32 * MT>(Xl, xld, rows, row_stride, c0, n, valid, tid);
  }
  template <bool THROUGH>
  __device__ static inline uint64_t first_layer(const float* Xs, int xld, const float* net, const NetLayout& L,
                                                const Pre& pre, float* Yl, float* Yg, int wave, int lane) {
    Acc<MT> acc;
    acc.zero();
    gemm_xw_deep<MT, PF>(Xs, xld, L.in, net + L.w1, pre.w1, wave, lane, acc);
    return relu_store<MT, THROUGH>(acc, pre.b1, Yl, Yg, wave, lane);
  }
};

struct Rows16Deep : Rows16 {
  __device__ static inline void load_input(float* Xl, int xld, const float* rows, int row_stride, int c0, int n, int valid,
                                           int tid) {
    load_input_wide<16>(Xl, xld, rows, row_stride, c0, n, valid, tid);
  }
  template <bool THROUGH>
  __device__ static inline uint64_t first_layer(const float* Xs, int xld, const float* net, const NetLayout& L,
                                                const Pre& pre, float* Yl, float* Yg, int wave, int lane) {
    Acc16 acc;
    acc.zero();
    gemm_xw_deep16(Xs, xld, L.in, net + L.w1, pre.w1, wave, lane, acc);
    return relu_store16<THROUGH>(acc, pre.b1, Yl, Yg, wave, lane);
  }
};

}  // namespace

// Action dimensions beyond kMaxAct (up to kSacMaxAct): the chains are compiled a second time with scratch rows of
// AS = kSacMaxAct floats -- a block of kSacMaxAct / kMaxAct of the map's [R][8] regions -- and kWideScratch regions.
constexpr int kWideScratch = 3 * (kSacMaxAct / kMaxAct);
constexpr int vec_target_floats(int AS) { return AS + 2 * kH + 8 + kHeadRed; }
constexpr int vec_actor_floats_for(int AS) { return AS + kH + kHeadRed; }
constexpr int vec_critic_floats = kH + 8, vec_actor_floats = vec_actor_floats_for(kMaxAct);   // staged vectors of the critic / actor
                                                     // chain; behind them: the weight stage of the 16-row transposed products

// Thin product with any number of outputs, eight at a time (the register budget of one pass).
template <class G>
__device__ inline void thin_wide(const float* Xl, const float* V, int J, float* outl, int stride, int tid) {
  for (int j0 = 0; j0 < J; j0 += kMaxAct) G::thin(Xl, V + j0 * kH, J - j0 < kMaxAct ? J - j0 : kMaxAct, outl + j0, tid, stride);
}

// The longest time a workgroup waits for another one of the same launch is d.wait_limit, in 10 ns ticks of the
// constant-rate clock (50 ms unless the host sets another bound; a healthy wait is a fraction of a millisecond).

// Bellman targets handed from a target workgroup to critic workgroups of the same launch
// travel as one 64-bit word per row, (t + 1) << 32 | bits of y, written and read with
// single device-scope atomic accesses: value and "ready" tag can then never be seen apart,
// and nothing but per-location coherence of atomics is relied on (no fences, no L2-wide
// write-back or invalidate).  The reader polls its own row; the wait is bounded by the
// constant-rate clock, after which a bit in d.fault is raised, which the host
// reports at its next synchronisation, and the lane goes on so that the launch still drains.
__device__ inline void publish_y(const PopDev& d, size_t row, uint32_t t, float y) {
  const uint64_t word = ((uint64_t)(t + 1u) << 32) | (uint64_t)__float_as_uint(y);
  __hip_atomic_store(d.y_tagged + row, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float await_y(const PopDev& d, size_t row, uint32_t t) {
  const uint64_t t0 = wall_clock64();
  uint64_t word;
  while (((word = __hip_atomic_load(d.y_tagged + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 32) != t + 1u) {
    __builtin_amdgcn_s_sleep(4);
    if (wall_clock64() - t0 > d.wait_limit) {
      __hip_atomic_store(d.fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      break;
    }
  }
  return __uint_as_float((uint32_t)word);
}

// Bulk results (activation tiles, partial sums, updated weights) handed to later workgroups
// of the same launch.  The producers of a unit write them with put<true> (written through
// to memory), wait until the memory system has acknowledged all of their own stores
// (s_waitcnt vmcnt(0) in every wavefront, then the workgroup barrier) and only then count
// themselves in with a device-scope atomic.  A consumer lets one lane poll the count, then
// takes a device-scope acquire (drops whatever its L1 / L2 may still hold of those
// addresses from an earlier step), and a barrier passes that on to its workgroup.
// A device-scope release fence in the producer would give the same ordering by the book,
// but it writes back every dirty line of the XCD's L2 -- all the Adam state other
// workgroups are streaming out -- and was measured at +40 % step time at P = 80.
// Counts start at zero in every launch: there are two sets of counters, a launch counts in
// one (d.sync_half, alternated by the host from launch to launch) and clears the other for
// its successor.  Consumers always have higher
// block indices than their producers, and workgroups are dispatched in index order, so a
// wait only ever concerns workgroups already dispatched.
__device__ inline int parity_base(const PopDev& d, uint32_t, int n) { return d.sync_half * n; }
__device__ inline void signal_count(uint32_t* count, int tid) {
  __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): this wavefront's stores are acknowledged
  __syncthreads();
  if (tid == 0) __hip_atomic_fetch_add(count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void wait_count(const PopDev& d, const uint32_t* count, uint32_t want) {   // one lane
  const uint64_t t0 = wall_clock64();
  while (__hip_atomic_load(count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < want) {
    __builtin_amdgcn_s_sleep(8);
    if (wall_clock64() - t0 > d.wait_limit) {
      __hip_atomic_store(d.fault + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      break;
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// ---------------------------------------------------------------------------------------------
// Target chain.  One workgroup per (agent, chunk).
//   a~ = clip(pi'(s') + clip(sigma eps, -c, c), -1, 1), eps = normal e = b A + j of stream 1
//   y  = r + gamma (1 - d) min(Q1'(s', a~), Q2'(s', a~))
// AS: row stride of the head scratch (kMaxAct, or kSacMaxAct for action dimensions beyond kMaxAct).
template <class G, int AS = kMaxAct>
__device__ __forceinline__ void target_chain(const PopDev& d, uint32_t t, int agent, int chunk, float* lds) {
  constexpr int R = G::R, RG = AS / kMaxAct;
  const LdsMap<G::R, G::kPad> L(d.D, AS == kMaxAct ? 3 : kWideScratch);
  float* Xs = lds;
  float* buf = lds + L.buf;
  float* head = lds + L.s0;                          // [R][AS]
  float* qmin = lds + L.s(RG);
  float* v_ab3 = lds + L.vec;                        // [AS]
  float* v_cw3 = v_ab3 + AS;                         // [2][256]
  float* v_cb3 = v_cw3 + 2 * kH;                     // [2]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = chunk * R;
  const float* ta = net_ptr(d, d.target, agent, 0);
  const float* tc0 = net_ptr(d, d.target, agent, 1);
  const float* tc1 = net_ptr(d, d.target, agent, 2);
  POP_MARK(29);
  typename G::Pre pre;
  pre.load(ta, d.actor, wave, lane);
  const HpDev hp = d.hp[agent];
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  // The smoothing noise of this chunk depends on nothing the chain computes (counter RNG: agent seed, step,
  // element), so it is drawn here, while the prologue's loads are on their way, and added after the head.
  constexpr int kNoisePerThread = (R * AS + kThreads - 1) / kThreads;
  float noise[kNoisePerThread];
  auto draw_noise = [&]() {
#pragma unroll
    for (int i = 0; i < kNoisePerThread; ++i) {
      const int e = tid + i * kThreads;
      noise[i] = 0.0f;
      if (e < R * d.A) {
        const int r = e / d.A, j = e - r * d.A;
        const uint32_t el = (uint32_t)((r0 + r) * d.A + j);
        const U4 blk = philox4x32_10(hp.seed_lo, hp.seed_hi, el >> 2, t, kStreamSmooth, 0u);
        float n4[4];
        normals4(blk, n4);
        const float n = (el & 2u) ? ((el & 1u) ? n4[3] : n4[2]) : ((el & 1u) ? n4[1] : n4[0]);
        noise[i] = fminf(fmaxf(hp.policy_noise * n, -hp.noise_clip), hp.noise_clip);
      }
    }
  };
  if (POP_ONE_TRIP && d.D <= kMaxIn) {               // everything the chain needs from memory before its first product: one trip
    SmallVec ab3, cw3a, cw3b;
    InputTile<R> xin;
    ab3.fetch(ta + d.actor.b3, d.A, tid);
    cw3a.fetch(tc0 + d.critic.w3, kH, tid);
    cw3b.fetch(tc1 + d.critic.w3, kH, tid);
    const float cb3 = (tid == 0 ? tc0 : tc1)[d.critic.b3];
    xin.fetch(L.xld, rows, d.row, d.D + 2, d.O, R, tid);
    __builtin_amdgcn_sched_barrier(0);                 // the loads go out first, the noise is drawn under them
    draw_noise();
    POP_MARK(30);
    ab3.put(v_ab3, d.A, tid);
    cw3a.put(v_cw3, kH, tid);
    cw3b.put(v_cw3 + kH, kH, tid);
    if (tid < 2) v_cb3[tid] = cb3;
    xin.put(Xs, L.xld, tid);
  } else {
    draw_noise();
    stage_vector(v_ab3, ta + d.actor.b3, d.A, tid);
    stage_vector(v_cw3, tc0 + d.critic.w3, kH, tid);
    stage_vector(v_cw3 + kH, tc1 + d.critic.w3, kH, tid);
    if (tid < 2) v_cb3[tid] = (tid == 0 ? tc0 : tc1)[d.critic.b3];
    POP_MARK(30);
    G::load_input(Xs, L.xld, rows, d.row, d.D + 2, d.O, R, tid);
  }
  __syncthreads();
  POP_MARK(31);

  G::template first_layer<false>(Xs, L.xld, ta, d.actor, pre, buf, nullptr, wave, lane);
  __syncthreads();
  POP_MARK(32);
  G::template hidden_layer<false>(buf, ta, d.actor, pre, nullptr, wave, lane, [&]() { pre.load(tc0, d.critic, wave, lane); });
  __syncthreads();
  POP_MARK(33);
  if (R <= 32 && (AS == kMaxAct || d.A <= 16)) head_mfma_split<R <= 32 ? R : 16, false>(buf, ta + d.actor.w3, d.A, head, AS, wave, lane, v_cb3 + 8);
  else head_mfma<R>(buf, ta + d.actor.w3, d.A, head, AS, wave, lane);   // the head's weights straight from global memory
  __syncthreads();
  POP_MARK(34);
#pragma unroll
  for (int i = 0; i < kNoisePerThread; ++i) {
    const int e = tid + i * kThreads;
    if (e < R * d.A) {
      const int r = e / d.A, j = e - r * d.A;
      const float mu = tanhf(head[r * AS + j] + v_ab3[j]);
      const float at = fminf(fmaxf(mu + noise[i], -1.0f), 1.0f);
      Xs[r * L.xld + d.O + j] = at;
      d.atilde[((size_t)agent * d.B + r0 + r) * d.A + j] = at;
    }
  }
  __syncthreads();
  POP_MARK(35);

#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const float* tc = k == 0 ? tc0 : tc1;
    G::template first_layer<false>(Xs, L.xld, tc, d.critic, pre, buf, nullptr, wave, lane);
    __syncthreads();
    POP_MARK(36 + 4 * k);
    G::template hidden_layer<false>(buf, tc, d.critic, pre, nullptr, wave, lane,
                           [&]() { if (k == 0) pre.load(tc1, d.critic, wave, lane); });
    __syncthreads();
    POP_MARK(37 + 4 * k);
    G::thin(buf, v_cw3 + k * kH, 1, head, tid);
    __syncthreads();
    POP_MARK(38 + 4 * k);
    if (tid < R) {
      const float q = head[tid * kMaxAct] + v_cb3[k];
      qmin[tid] = k == 0 ? q : fminf(qmin[tid], q);
    }
    __syncthreads();
  }
  if (tid < R) {
    const float rew = rows[(size_t)tid * d.row + d.D];
    const float done = rows[(size_t)tid * d.row + d.D + 1];
    const float yv = rew + hp.gamma * (1.0f - done) * qmin[tid];
    d.y[(size_t)agent * d.B + r0 + tid] = yv;
    publish_y(d, (size_t)agent * d.B + r0 + tid, t, yv);   // for critic workgroups of the same launch
  }
  POP_MARK(45);
}


// ---------------------------------------------------------------------------------------------
// The actor's own forward pass (s -> h1 -> h2 -> a_pi) for the rows of a critic workgroup, run by that workgroup
// while it waits for its Bellman targets: it depends on nothing of the step but the batch, and the actor launch that
// follows the critics' weight step then starts at the critic (actor_chain<.., AHEAD>).  Xs: the critic's input tile
// [s, a] -- the action columns meet the zero rows that pad the actor's first-layer weights; `area`: LDS of
// ahead_floats<R>() floats that the critic chain does not use.  Writes aH1, aH2 and api.
template <int R>
constexpr int ahead_floats() { return R * kLda + R * kMaxAct + kHeadRed; }
constexpr int kAheadBase = 8 + 2 * kH + 8 + kHeadRed;   // floats behind the LDS map that the chains of the launch use for their vectors
template <class G>
__device__ __forceinline__ void actor_forward_ahead(const PopDev& d, int agent, int r0, const float* Xs, int xld, float* area) {
  constexpr int R = G::R;
  static_assert(R == 32, "built for the 32-row critic workgroups");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  float* buf2 = area;
  float* head = buf2 + R * kLda;
  float* red = head + R * kMaxAct;
  const float* an = net_ptr(d, d.theta, agent, 0);
  typename G::Pre pa;
  POP_MARK(56);
  pa.load(an, d.actor, wave, lane);
  const size_t act_off = ((size_t)agent * d.B + r0) * kH;
  G::template first_layer<false>(Xs, xld, an, d.actor, pa, buf2, d.aH1 + act_off, wave, lane);
  __syncthreads();
  POP_MARK(57);
  G::template hidden_layer<false>(buf2, an, d.actor, pa, d.aH2 + act_off, wave, lane, NoTail());
  __syncthreads();
  POP_MARK(58);
  head_mfma_split<R, false>(buf2, an + d.actor.w3, d.A, head, kMaxAct, wave, lane, red);
  __syncthreads();
  POP_MARK(59);
  float* out = d.api + ((size_t)agent * d.B + r0) * d.A;
  for (int e = tid; e < R * d.A; e += kThreads) {
    const int r = e / d.A, j = e - r * d.A;
    out[e] = tanhf(head[r * kMaxAct + j] + an[d.actor.b3 + j]);
  }
}

// ---------------------------------------------------------------------------------------------
// Critic forward + backward.  One workgroup per (critic network, chunk); network = 2 agent + k.
//   L = (1/B) sum_b (Q_k(s_b, a_b) - y_b)^2 ;  dq = 2 (q - y) / B
//   dz2 = (dq W3^T) * [h2 > 0] ;  dz1 = (dz2 W2^T) * [h1 > 0]
// Outputs for the weight-gradient kernel: h1, dz2, dz1 (global), and the chunk's
// partial sums of dW3, db3, db2, db1 and of the loss.
// WAIT: the targets come from target workgroups of the same launch; the lanes that need
// them poll for their rows right before the loss.  SIGNAL: count this chunk as finished
// for the weight-gradient workgroups of the same launch.  AHEAD: the workgroups of critic 2 run the actor's forward
// pass for their rows before they wait (d.actor_ahead, steps with an actor update).
template <class G, bool WAIT, bool SIGNAL, bool AHEAD = false>
__device__ __forceinline__ void critic_chain(const PopDev& d, uint32_t t, int net, int chunk, float* lds) {
  constexpr int R = G::R;
  const LdsMap<G::R, G::kPad> L(d.D);
  float* Xs = lds;
  float* buf = lds + L.buf;
  float* head = lds + L.s0;
  float* dq = lds + L.s1;
  float* v_w3 = lds + L.vec;                         // [256]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int agent = net >> 1, k = net & 1, r0 = chunk * R;
  const float* cn = net_ptr(d, d.theta, agent, 1 + k);
  typename G::Pre pre;
  pre.load(cn, d.critic, wave, lane);
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  const size_t act_off = ((size_t)net * d.B + r0) * kH;
  float* part = d.cpart + ((size_t)net * d.cstride + chunk) * kCPart;
  float yv = 0.0f, b3 = 0.0f;
  if (POP_ONE_TRIP && d.D <= kMaxIn) {               // one trip to memory for all of the prologue
    SmallVec w3;
    InputTile<R> xin;
    w3.fetch(cn + d.critic.w3, kH, tid);
    xin.fetch(L.xld, rows, d.row, 0, d.D, R, tid);
    if (tid < R) {
      if (!WAIT) yv = d.y[(size_t)agent * d.B + r0 + tid];
      b3 = cn[d.critic.b3];
    }
    w3.put(v_w3, kH, tid);
    xin.put(Xs, L.xld, tid);
  } else {
    stage_vector(v_w3, cn + d.critic.w3, kH, tid);
    G::load_input(Xs, L.xld, rows, d.row, 0, d.D, R, tid);
    if (tid < R) {
      if (!WAIT) yv = d.y[(size_t)agent * d.B + r0 + tid];
      b3 = cn[d.critic.b3];
    }
  }
  POP_MARK(0);
  __syncthreads();
  POP_MARK(1);

  const uint64_t mask1 = G::template first_layer<SIGNAL>(Xs, L.xld, cn, d.critic, pre, buf, d.cH1 + act_off, wave, lane);
  __syncthreads();
  POP_MARK(2);
  typename G::WtBlock wt;                          // block 0 of W2 for the input-gradient product
  G::template hidden_layer<false>(buf, cn, d.critic, pre, nullptr, wave, lane, [&]() { G::load_wt(wt, cn + d.critic.w2, wave, lane); });
  __syncthreads();
  POP_MARK(3);
  G::thin(buf, v_w3, 1, head, tid);
  if constexpr (AHEAD) {
    if (k == 1 && d.actor_ahead && t % (uint32_t)d.hp[agent].policy_delay == 0u)
      actor_forward_ahead<G>(d, agent, r0, Xs, L.xld, lds + L.vec + kAheadBase);
  }
  if (WAIT && tid < R) yv = await_y(d, (size_t)agent * d.B + r0 + tid, t);   // same lane uses it below
  __syncthreads();
  POP_MARK(4);
  if (tid < 64) {                                   // R <= 64: one wavefront covers the chunk
    float err = 0.0f, g = 0.0f;
    if (tid < R) {
      err = head[tid * kMaxAct] + b3 - yv;
      g = 2.0f * err / (float)(d.B * d.share);         // share > 1: the critic loss is the mean over the population
      dq[tid] = g;
    }
    const float sq = wave_sum(err * err);
    const float sdq = wave_sum(g);
    if (tid == 0) { put<SIGNAL>(part + kCP_loss, sq / (float)(d.B * d.share)); put<SIGNAL>(part + kCP_db3, sdq); }
  }
  __syncthreads();
  {                                                 // one thread per hidden unit, 8 rows at a time
    const int c = tid;
    const float w3 = v_w3[c];
    float gw3 = 0.0f, gb2 = 0.0f;
    float* zg = d.cdZ2 + act_off + c;
#pragma unroll 1
    for (int rb = 0; rb < R; rb += 8) {
      float h[8], g[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { h[i] = buf[(rb + i) * kLda + c]; g[i] = dq[rb + i]; }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        gw3 += h[i] * g[i];
        const float z = h[i] > 0.0f ? g[i] * w3 : 0.0f;
        buf[(rb + i) * kLda + c] = z;
        put<SIGNAL>(zg + (rb + i) * kH, z);
        gb2 += z;
      }
    }
    put<SIGNAL>(part + kCP_dW3 + c, gw3);
    put<SIGNAL>(part + kCP_db2 + c, gb2);
  }
  POP_MARK(5);
  __syncthreads();
  POP_MARK(6);
  G::template input_grad_to_global<SIGNAL>(buf, cn + d.critic.w2, wt, mask1, d.cdZ1 + act_off, part + kCP_db1, wave, lane,
                                           lds + L.vec + vec_critic_floats);
  POP_MARK(7);
  if (SIGNAL) signal_count(d.done_c + parity_base(d, t, 2 * d.P) + net, tid);
}



// ---------------------------------------------------------------------------------------------
// Actor chain (steps with t % policy_delay == 0).  One workgroup per (agent, chunk).
//   L = -(1/B) sum_b Q1(s_b, pi(s_b)) through the critic updated earlier in this step.
//   Critic 1: dz2c = -(1/B) W3c^T * [c2 > 0]; dz1c = (dz2c W2c^T) * [c1 > 0];
//             da = dz1c W1c[O:O+A, :]^T
//   Actor:    dz3 = da (1 - a_pi^2); dz2 = (dz3 W3^T) * [h2 > 0]; dz1 = (dz2 W2^T) * [h1 > 0]
// The actor's second hidden layer has to survive the critic pass: it is parked in
// global memory (L2) and fetched back into registers under the critic's last product.
// WAIT: the critic update of this step runs in the same launch; the actor's own forward
// pass goes ahead, everything that reads critic 1 waits until all of its weight-gradient
// workgroups are done.  SIGNAL: count this chunk as finished for the actor's weight-gradient
// workgroups.  AHEAD: the forward pass was run by critic workgroups of the launch before (actor_forward_ahead): the
// chain takes a_pi and the first layer's ReLU pattern from what they wrote and starts at the critic.
// AS: row stride of the head scratch blocks, as in target_chain.
template <class G, bool WAIT, bool AHEAD = false, int AS = kMaxAct>
__device__ __forceinline__ void actor_chain(const PopDev& d, uint32_t t, int agent, int chunk, float* lds, int critic_roles) {
  constexpr int R = G::R, RG = AS / kMaxAct;
  const LdsMap<G::R, G::kPad> L(d.D, AS == kMaxAct ? 3 : kWideScratch);
  float* Xs = lds;
  float* buf = lds + L.buf;
  float* head = lds + L.s0;                          // three blocks of [R][AS]
  float* api = lds + L.s(RG);
  float* dz3 = lds + L.s(2 * RG);
  const int A = d.A;
  float* v_ab3 = lds + L.vec;                        // [AS] actor head bias
  float* v_cw3 = v_ab3 + AS;                         // [256] critic head
  float* stage = lds + L.vec + vec_actor_floats_for(AS);   // weight stage of the 16-row transposed products
  // the actor's head and the critic's first-layer rows of the action inputs are matrix-pipe operands read
  // straight from global memory (head_mfma, head_mfma_t)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = chunk * R;
  const HpDev hp = d.hp[agent];
  if (t % (uint32_t)hp.policy_delay != 0u) return;
  const float* an = net_ptr(d, d.theta, agent, 0);
  const float* cn = net_ptr(d, d.theta, agent, 1);
  POP_MARK(8);
  typename G::Pre pre;
  pre.load(AHEAD ? cn : an, AHEAD ? d.critic : d.actor, wave, lane);
  const float* rows = batch_rows(d, t, agent) + (size_t)r0 * d.row;
  const size_t act_off = ((size_t)agent * d.B + r0) * kH;
  float* part = d.apart + ((size_t)agent * (d.B / R) + chunk) * kAPart;
  float cb3 = 0.0f;
  auto stage_critic = [&]() {
    stage_vector(v_cw3, cn + d.critic.w3, kH, tid);
    cb3 = cn[d.critic.b3];
  };
  uint64_t mask_a1 = 0;
  if constexpr (AHEAD) {
    static_assert(!WAIT && AS == kMaxAct, "the forward pass ahead belongs to the separate launches of the narrow shapes");
    // one trip to memory: the critic's head, the input tile [s, a_pi] (a_pi from the forward pass ahead), h1's pattern
    constexpr int IT = InputTile<R>::IT;
    SmallVec cw3;
    float xv[IT];
    cw3.fetch(cn + d.critic.w3, kH, tid);
    cb3 = cn[d.critic.b3];
    const float* ag = d.api + ((size_t)agent * d.B + r0) * A;
#pragma unroll
    for (int i = 0; i < IT; ++i) {
      const int e = tid + i * kThreads;
      const int r = e / L.xld, c = e - r * L.xld;
      const bool in = e < R * L.xld && c < d.D;
      const float* p = !in ? rows : c < d.O ? rows + (size_t)r * d.row + c : ag + r * A + (c - d.O);
      const float x = *p;
      xv[i] = in ? x : 0.0f;
    }
    mask_a1 = G::mask_from_global(d.aH1 + act_off, wave, lane);
    cw3.put(v_cw3, kH, tid);
#pragma unroll
    for (int i = 0; i < IT; ++i) {
      const int e = tid + i * kThreads;
      const int r = e / L.xld, c = e - r * L.xld;
      if (e < R * L.xld) {
        Xs[e] = xv[i];
        if (c >= d.O && c < d.D) api[r * kMaxAct + (c - d.O)] = xv[i];
      }
    }
    __syncthreads();
  } else {
  if (POP_ONE_TRIP && d.D <= kMaxIn) {               // one trip to memory for all of the prologue
    SmallVec ab3, cw3;
    InputTile<R> xin;
    ab3.fetch(an + d.actor.b3, A, tid);
    if (!WAIT) { cw3.fetch(cn + d.critic.w3, kH, tid); cb3 = cn[d.critic.b3]; }
    xin.fetch(L.xld, rows, d.row, 0, d.O, R, tid);
    ab3.put(v_ab3, A, tid);
    if (!WAIT) cw3.put(v_cw3, kH, tid);
    xin.put(Xs, L.xld, tid);
  } else {
    stage_vector(v_ab3, an + d.actor.b3, A, tid);
    if (!WAIT) stage_critic();
    G::load_input(Xs, L.xld, rows, d.row, 0, d.O, R, tid);
  }
  __syncthreads();

  mask_a1 = G::template first_layer<WAIT>(Xs, L.xld, an, d.actor, pre, buf, d.aH1 + act_off, wave, lane);
  __syncthreads();
  G::template hidden_layer<false>(buf, an, d.actor, pre, d.aH2 + act_off, wave, lane,
                         [&]() { if (!WAIT) pre.load(cn, d.critic, wave, lane); });
  __syncthreads();
  if (R <= 32 && (AS == kMaxAct || A <= 16)) head_mfma_split<R <= 32 ? R : 16, false>(buf, an + d.actor.w3, A, head, AS, wave, lane, v_cw3 + kH);
  else head_mfma<R>(buf, an + d.actor.w3, A, head, AS, wave, lane);
  __syncthreads();
  for (int e = tid; e < R * A; e += kThreads) {
    const int r = e / A, j = e - r * A;
    const float a = tanhf(head[r * AS + j] + v_ab3[j]);
    api[r * AS + j] = a;
    Xs[r * L.xld + d.O + j] = a;
  }
  __syncthreads();
  }

  // critic 1 on [s, a_pi]
  POP_MARK(9);
  if (WAIT) {
    if (tid == 0) wait_count(d, d.done_wc + parity_base(d, t, 2 * d.P) + 2 * agent, (uint32_t)critic_roles);
    __syncthreads();
    stage_critic();
    pre.load(cn, d.critic, wave, lane);
    __syncthreads();
  }
  POP_MARK(10);
  const uint64_t mask_c1 = G::template first_layer<false>(Xs, L.xld, cn, d.critic, pre, buf, nullptr, wave, lane);
  __syncthreads();
  typename G::WtBlock wt;
  G::template hidden_layer<false>(buf, cn, d.critic, pre, nullptr, wave, lane, [&]() { G::load_wt(wt, cn + d.critic.w2, wave, lane); });
  __syncthreads();
  POP_MARK(11);
  G::thin(buf, v_cw3, 1, head, tid);     // q, for the loss value only
  __syncthreads();
  if (tid < 64) {
    const float q = tid < R ? head[tid * kMaxAct] + cb3 : 0.0f;
    const float s = wave_sum(q);
    if (tid == 0) put<WAIT>(part + kAP_loss, -s / (float)d.B);
  }
  {
    const int c = tid;
    const float seed = -v_cw3[c] / (float)d.B;
#pragma unroll 1
    for (int rb = 0; rb < R; rb += 8) {
      float h[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) h[i] = buf[(rb + i) * kLda + c];
#pragma unroll
      for (int i = 0; i < 8; ++i) buf[(rb + i) * kLda + c] = h[i] > 0.0f ? seed : 0.0f;
    }
  }
  __syncthreads();
  f32x4 h2r[R / 4];                                  // this thread's share of the parked h2 tile
  {
    const float* h2g = d.aH2 + act_off;
    G::input_grad_to_lds(buf, cn + d.critic.w2, wt, mask_c1, wave, lane, [&]() {
#pragma unroll
      for (int i = 0; i < R / 4; ++i)
        h2r[i] = *reinterpret_cast<const f32x4*>(h2g + (4 * i + (tid >> 6)) * kH + 4 * (tid & 63));
    }, stage);                                       // buf = dz1 of the critic
  }
  __syncthreads();
  POP_MARK(12);
  if (R <= 32 && (AS == kMaxAct || A <= 16)) head_mfma_split<R <= 32 ? R : 16, true>(buf, cn + d.critic.w1 + d.O * kH, A, head, AS, wave, lane, v_cw3 + kH);   // da
  else head_mfma_t<R>(buf, cn + d.critic.w1 + d.O * kH, A, head, AS, wave, lane);
  G::load_wt(wt, an + d.actor.w2, wave, lane);       // block 0 of the actor's input-gradient product
  __syncthreads();
  for (int e = tid; e < R * AS; e += kThreads) {
    const int j = e % AS;
    const float a = j < A ? api[e] : 0.0f;
    dz3[e] = j < A ? head[e] * (1.0f - a * a) : 0.0f;     // unused columns are kept at zero
  }
#pragma unroll
  for (int i = 0; i < R / 4; ++i)                    // h2 of the actor back into the tile
    *reinterpret_cast<f32x4*>(&buf[(4 * i + (tid >> 6)) * kLda + 4 * (tid & 63)]) = h2r[i];
  __syncthreads();
  if (tid < A) {
    float s = 0.0f;
    for (int r = 0; r < R; ++r) s += dz3[r * AS + tid];
    put<WAIT>(part + kAP_db3 + tid, s);
  }
  {                                                  // actor head backward, one thread per hidden unit
    const int c = tid;
    constexpr int RB = AS == kMaxAct ? 4 : 2;        // rows in flight (the wide rows cost three times the registers)
    float w3[AS], gw3[AS];
#pragma unroll
    for (int j = 0; j < AS; ++j) { w3[j] = (an + d.actor.w3)[c * A + (j < A ? j : 0)]; gw3[j] = 0.0f; }
#pragma unroll
    for (int j = 0; j < AS; ++j) w3[j] = j < A ? w3[j] : 0.0f;
    float gb2 = 0.0f;
    float* zg = d.adZ2 + act_off + c;
#pragma unroll 1
    for (int rb = 0; rb < R; rb += RB) {
      float h[RB];
      f32x4 g[RB][AS / 4];
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        h[i] = buf[(rb + i) * kLda + c];
#pragma unroll
        for (int q = 0; q < AS / 4; ++q) g[i][q] = *reinterpret_cast<const f32x4*>(&dz3[(rb + i) * AS + 4 * q]);   // columns >= A hold zeros
      }
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        float dh = 0.0f;
#pragma unroll
        for (int j = 0; j < AS; ++j) {
          const float gj = g[i][j >> 2][j & 3];
          gw3[j] += h[i] * gj;
          dh += gj * w3[j];
        }
        const float z = h[i] > 0.0f ? dh : 0.0f;
        buf[(rb + i) * kLda + c] = z;
        put<WAIT>(zg + (rb + i) * kH, z);
        gb2 += z;
      }
    }
#pragma unroll
    for (int j = 0; j < AS; ++j)
      if (j < A) put<WAIT>(part + kAP_dW3 + j * kH + c, gw3[j]);
    put<WAIT>(part + kAP_db2 + c, gb2);
  }
  __syncthreads();
  POP_MARK(13);
  G::template input_grad_to_global<WAIT>(buf, an + d.actor.w2, wt, mask_a1, d.adZ1 + act_off, part + kAP_db1, wave, lane, stage);
  POP_MARK(14);
  if (WAIT) signal_count(d.done_a + parity_base(d, t, d.P) + agent, tid);
}

// floats of staged vectors behind the LDS map of each chain
inline int vec_target(const PopDev& d) { return vec_target_floats(d.A > kMaxAct ? kSacMaxAct : kMaxAct); }
inline int vec_critic(const PopDev&) { return vec_critic_floats; }
inline int vec_actor(const PopDev& d) { return vec_actor_floats_for(d.A > kMaxAct ? kSacMaxAct : kMaxAct); }
inline int vec_act(const PopDev& d) { return kH * d.actor.out + kMaxHead; }
constexpr int kActScratch = 2 * (kSacMaxAct / kMaxAct);   // acting: two head blocks of [32][kSacMaxAct]

}  // namespace pop
