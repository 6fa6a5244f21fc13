// Device building blocks for the fp32 MFMA contractions (gfx950, wave64).
//
// All dense products of the pass are tiled the same way: a workgroup of 256
// threads (4 wavefronts in a 2 x 2 arrangement) owns a 128 x 128 output tile,
// each wavefront a 64 x 64 quarter held as 2 x 2 accumulators of
// v_mfma_f32_32x32x2_f32.  Operands are staged through LDS in k-chunks.
//
// Register layout of one 32 x 32 accumulator (16 VGPRs per lane):
//   value v of lane l is element (row, col) = (8*(v/4) + 4*(l/32) + v%4, l%32).
// Operand layout: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32].
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int TILE = 128;      // output tile edge
constexpr int WG_THREADS = 256;

struct Acc2x2 {
  floatx16 t[2][2];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) t[a][b][v] = 0.0f;
  }
};

// The 128 x 128 tile is a 4 x 4 array of 32 x 32 MFMA sub-tiles; wave (wm, wn) owns the
// sub-tiles (wm + 2 tm, wn + 2 tn).  Two sub-tiles of a wave are therefore 64 floats apart
// in a k-major LDS row, which is what lets one ds_read2st64_b32 with immediate offsets fetch
// both operands of a k-step: address arithmetic on the vector ALU between MFMA groups
// (measured: about 32 idle MFMA cycles per group of four) is avoided.
// Row (within the 128-tile) of accumulator value v of sub-tile tm for this lane.
__device__ __forceinline__ int acc_row(int wm, int tm, int v, int lane) {
  return wm * 32 + tm * 64 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}
__device__ __forceinline__ int acc_col(int wn, int tn, int lane) {
  return wn * 32 + tn * 64 + (lane & 31);
}

// One k-chunk of KT (even) steps.  Both operands are k-major in LDS:
// sP[k][128] holds A[m][k] at sP[k*128 + m], sQ[k][128] holds B[k][n].
template <int KT>
__device__ __forceinline__ void mma_chunk_kmajor(const float* __restrict__ sP,
                                                 const float* __restrict__ sQ, int wm, int wn,
                                                 int lane, Acc2x2& acc) {
  const int kl = lane >> 5, ml = lane & 31;
  const float* p = sP + kl * TILE + wm * 32 + ml;   // + 2*kk*TILE per step: immediate offsets
  const float* q = sQ + kl * TILE + wn * 32 + ml;
  // operands of step kk+1 are read while the MFMAs of step kk run; the scheduling
  // barriers keep the compiler from sinking the reads below the MFMAs again
  float a0[2], a1[2], b0[2], b1[2];
  a0[0] = p[0]; a1[0] = p[64]; b0[0] = q[0]; b1[0] = q[64];
#pragma unroll
  for (int kk = 0; kk < KT / 2; ++kk) {
    const int cur = kk & 1, nxt = cur ^ 1;
    if (kk + 1 < KT / 2) {
      a0[nxt] = p[2 * (kk + 1) * TILE];
      a1[nxt] = p[2 * (kk + 1) * TILE + 64];
      b0[nxt] = q[2 * (kk + 1) * TILE];
      b1[nxt] = q[2 * (kk + 1) * TILE + 64];
    }
    __builtin_amdgcn_sched_barrier(0);
    acc.t[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[cur], b0[cur], acc.t[0][0], 0, 0, 0);
    acc.t[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[cur], b1[cur], acc.t[0][1], 0, 0, 0);
    acc.t[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[cur], b0[cur], acc.t[1][0], 0, 0, 0);
    acc.t[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[cur], b1[cur], acc.t[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Row-major operand chunk in LDS: s[idx][RM_LD] holds value (idx, k) at s[idx*RM_LD + k],
// idx = m for the A operand or n for a transposed B operand.  RM_LD = 33 keeps both the
// scalar stores of a float4-per-thread fill and the MFMA operand reads free of bank conflicts.
constexpr int RM_KT = 32;
constexpr int RM_LD = 33;

// Fill a row-major chunk: 128 rows x 32 k-values from src[row*ld + k], all in bounds,
// ld % 4 == 0 and src 16-byte aligned.
__device__ __forceinline__ void fill_rowmajor(float* __restrict__ s, const float* __restrict__ src,
                                              int64_t ld, int tid) {
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int f = tid + p * WG_THREADS;
    int row = f >> 3, k4 = f & 7;
    float4 v = *reinterpret_cast<const float4*>(src + (int64_t)row * ld + 4 * k4);
    float* d = s + row * RM_LD + 4 * k4;
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
  }
}

// Fill a k-major chunk: 32 k-rows x 128 values from src[k*ld + idx].
__device__ __forceinline__ void fill_kmajor32(float* __restrict__ s, const float* __restrict__ src,
                                              int64_t ld, int tid) {
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int f = tid + p * WG_THREADS;
    int k = f >> 5, c4 = f & 31;
    float4 v = *reinterpret_cast<const float4*>(src + (int64_t)k * ld + 4 * c4);
    *reinterpret_cast<float4*>(s + k * TILE + 4 * c4) = v;
  }
}

// One 32-deep k-chunk with A row-major in LDS and B either row-major (B_KMAJOR = false,
// i.e. the product A * B^T of two row-major tiles) or k-major.
template <bool B_KMAJOR>
__device__ __forceinline__ void mma_chunk_rowmajor_a(const float* __restrict__ sA,
                                                     const float* __restrict__ sB, int wm, int wn,
                                                     int lane, Acc2x2& acc) {
  const int kl = lane >> 5, ml = lane & 31;
#pragma unroll
  for (int kk = 0; kk < RM_KT / 2; ++kk) {
    const int k = 2 * kk + kl;
    float a0 = sA[(wm * 32 + ml) * RM_LD + k];
    float a1 = sA[(wm * 32 + 64 + ml) * RM_LD + k];
    float b0, b1;
    if (B_KMAJOR) {
      b0 = sB[k * TILE + wn * 32 + ml];
      b1 = sB[k * TILE + wn * 32 + 64 + ml];
    } else {
      b0 = sB[(wn * 32 + ml) * RM_LD + k];
      b1 = sB[(wn * 32 + 64 + ml) * RM_LD + k];
    }
    acc.t[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc.t[0][0], 0, 0, 0);
    acc.t[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc.t[0][1], 0, 0, 0);
    acc.t[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc.t[1][0], 0, 0, 0);
    acc.t[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc.t[1][1], 0, 0, 0);
  }
}

}  // namespace lq
