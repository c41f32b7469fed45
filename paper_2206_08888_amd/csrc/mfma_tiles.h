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

__device__ inline f32x16 mfma32(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ inline int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

template <int MT>
struct Acc {
  f32x16 t[MT][2];
  __device__ inline void zero() {
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
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
        f(32 * mt + acc_row(v, lane), 64 * wave + 32 * nt + (lane & 31), acc.t[mt][nt][v]);
}

// acc[r][c] += sum_{k<K} X[r][k] W[k][c]   (forward product x W)
//   X: LDS, row stride ldx, rows [0, 32 MT), columns >= K up to the next
//      multiple of 8 must hold finite values (they meet zero weights);
//   W: global, row-major [K][256].
template <int MT, bool FULLK>
__device__ inline void gemm_xw(const float* __restrict__ Xl, int ldx, int K, const float* __restrict__ W,
                               int wave, int lane, Acc<MT>& acc) {
  const int half = lane >> 5, l32 = lane & 31;
  const float* wcol = W + 64 * wave + l32;
  const int K8 = (K + 7) & ~7;
  float bc[2][4], bn[2][4];
  auto load_b = [&](int k0, float (&b)[2][4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + 4 * half + j;
      const bool ok = FULLK || k < K;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) b[nt][j] = ok ? wcol[(size_t)k * kH + 32 * nt] : 0.0f;
    }
  };
  load_b(0, bc);
#pragma unroll 2
  for (int k0 = 0; k0 < K8; k0 += 8) {
    if (k0 + 8 < K8) load_b(k0 + 8, bn);
    f32x4 a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      a[mt] = *reinterpret_cast<const f32x4*>(&Xl[(32 * mt + l32) * ldx + k0 + 4 * half]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc.t[mt][nt] = mfma32(a[mt][j], bc[nt][j], acc.t[mt][nt]);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int j = 0; j < 4; ++j) bc[nt][j] = bn[nt][j];
  }
}

// acc[r][k] += sum_{n<256} Z[r][n] W[k][n]   (input-gradient product dz W^T)
//   Z: LDS, row stride kLda; W: global, row-major [256][256].
template <int MT>
__device__ inline void gemm_zwt(const float* __restrict__ Zl, const float* __restrict__ W, int wave, int lane,
                                Acc<MT>& acc) {
  const int half = lane >> 5, l32 = lane & 31;
  const float* wrow = W + (size_t)(64 * wave + l32) * kH + 4 * half;
  f32x4 bc[2], bn[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) bc[nt] = *reinterpret_cast<const f32x4*>(wrow + (size_t)32 * nt * kH);
#pragma unroll 2
  for (int n0 = 0; n0 < kH; n0 += 8) {
    if (n0 + 8 < kH) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
        bn[nt] = *reinterpret_cast<const f32x4*>(wrow + (size_t)32 * nt * kH + n0 + 8);
    }
    f32x4 a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      a[mt] = *reinterpret_cast<const f32x4*>(&Zl[(32 * mt + l32) * kLda + n0 + 4 * half]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc.t[mt][nt] = mfma32(a[mt][j], bc[nt][j], acc.t[mt][nt]);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) bc[nt] = bn[nt];
  }
}

// One hidden layer: Y = relu(X W + b) written to LDS (row stride kLda) and,
// when Yg != nullptr, to global memory as [rows][256].
template <int MT, bool FULLK>
__device__ inline void layer_relu(const float* __restrict__ Xl, int ldx, int K, const float* __restrict__ W,
                                  const float* __restrict__ bias, float* __restrict__ Yl,
                                  float* __restrict__ Yg, int wave, int lane) {
  Acc<MT> acc;
  acc.zero();
  gemm_xw<MT, FULLK>(Xl, ldx, K, W, wave, lane, acc);
  float bb[2];
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) bb[nt] = bias[64 * wave + 32 * nt + (lane & 31)];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 32 * mt + acc_row(v, lane);
        const int col = 64 * wave + 32 * nt + (lane & 31);
        const float h = fmaxf(acc.t[mt][nt][v] + bb[nt], 0.0f);
        Yl[row * kLda + col] = h;
        if (Yg) Yg[(size_t)row * kH + col] = h;
      }
}

// Thin products on the vector ALU (heads with 1..8 outputs, action gradient):
// out[r*kMaxAct + j] = sum_{c<256} X[r][c] V_j[c],  r < R, j < J.
// Thread t works on rows (t >> 3) + 32 i with column groups 32 q + 4 (t & 7);
// 8 neighbouring lanes share a row and are summed with lane shuffles.
// STRIDED: V_j[c] = V[c * J + j] (a head weight W3[256][J]);
// otherwise V_j[c] = V[j * 256 + c] (J rows of a [.., 256] matrix).
template <int R, bool STRIDED>
__device__ inline void thin_dot(const float* __restrict__ Xl, const float* __restrict__ V, int J,
                                float* __restrict__ outl, int tid) {
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
          if (STRIDED) {
            s[j] += x[0] * V[(c + 0) * J + j] + x[1] * V[(c + 1) * J + j] + x[2] * V[(c + 2) * J + j] +
                    x[3] * V[(c + 3) * J + j];
          } else {
            const f32x4 w = *reinterpret_cast<const f32x4*>(&V[(size_t)j * kH + c]);
            s[j] += x[0] * w[0] + x[1] * w[1] + x[2] * w[2] + x[3] * w[3];
          }
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
        if (p == 0) outl[r * kMaxAct + j] = v;
      }
    }
  }
}

// 32x32 tile of a weight gradient: C[m][n] = sum_{b<B} A[b*lda + m0 + m] Z[b*ldz + n0 + n],
// both operands in global memory, rows m0 + m >= M masked to zero.  B % 16 == 0.
__device__ inline f32x16 wgrad_tile(const float* __restrict__ A, int lda, int M, int m0,
                                    const float* __restrict__ Z, int ldz, int n0, int B, int lane) {
  const int half = lane >> 5, l32 = lane & 31;
  const bool mok = (m0 + l32) < M;
  const float* ap = A + (size_t)half * lda + m0 + l32;
  const float* zp = Z + (size_t)half * ldz + n0 + l32;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  float ac[8], zc[8], an[8], zn[8];
  auto load = [&](int b0, float (&a)[8], float (&z)[8]) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      a[u] = mok ? ap[(size_t)(b0 + 2 * u) * lda] : 0.0f;
      z[u] = zp[(size_t)(b0 + 2 * u) * ldz];
    }
  };
  load(0, ac, zc);
#pragma unroll 2
  for (int b0 = 0; b0 < B; b0 += 16) {
    if (b0 + 16 < B) load(b0 + 16, an, zn);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc = mfma32(ac[u], zc[u], acc);
#pragma unroll
    for (int u = 0; u < 8; ++u) { ac[u] = an[u]; zc[u] = zn[u]; }
  }
  return acc;
}

}  // namespace pop
