// Column kernel of lq_quantize_layer (Algorithm 1 lines 11-18): one lane owns one row
// and keeps that row's B weights of the current block in registers; for every column
// it quantizes against the row's grid (line 13 / 15), forms E = (w - q) / U_jj (line 16)
// and subtracts E * U[j, j+1:] from its remaining registers (line 17).  The B x B block
// of U is read from LDS at wave-uniform addresses.  E is written transposed ([B x r]) for
// the trailing MFMA update.  Instantiated per block width in separate translation units.
#pragma once

#include "lq_common.h"

namespace lq {

constexpr int QT = 256;  // threads (= rows) per workgroup of the column kernel

struct ColArgs {
  float* W; int64_t ldw;
  int64_t r, c;
  int64_t i0;           // first column of the block
  int nb;               // columns in this block (<= B)
  const float* U; int64_t ldu;
  const float* grid;    // nu: [r x K]; aff: [r x ngroups x 2]
  int group; int ngroups;
  uint8_t* codes;
  float* Et; int64_t rpad;
  float* row_loss;      // may be null
  int first;            // 1 for the first block (row_loss starts from zero)
  int vecw;             // W rows may be read / written as float4
};

// Nearest point of an ascending grid; ties go to the lower point.
template <int K>
__device__ __forceinline__ void quant_nu(float w, const float (&g)[K], const float (&mid)[K - 1],
                                         float& q, int& code) {
  q = g[0];
  code = 0;
#pragma unroll
  for (int m = 1; m < K; ++m) {
    bool up = w > mid[m - 1];
    q = up ? g[m] : q;
    code += up ? 1 : 0;
  }
}

template <int B, int BITS, bool AFF>
__global__ __launch_bounds__(QT) void column_block_kernel(ColArgs a) {
  constexpr int K = 1 << BITS;
  extern __shared__ __align__(16) float smq[];
  float* sU = smq;            // [B][B], zero outside the stored upper triangle / the block
  float* sRinv = smq + B * B; // [B]  1 / U_jj

  const int tid = threadIdx.x;
  const int64_t row = (int64_t)blockIdx.x * QT + tid;
  const bool valid = row < a.r;
  const int nb = a.nb;

  for (int f = tid; f < B * B; f += QT) {
    int j = f / B, jj = f - j * B;
    float v = 0.0f;
    if (j < nb && jj < nb && jj >= j) v = a.U[(a.i0 + j) * a.ldu + a.i0 + jj];
    sU[f] = v;
  }
  for (int j = tid; j < B; j += QT) sRinv[j] = (j < nb) ? 1.0f / a.U[(a.i0 + j) * a.ldu + a.i0 + j] : 0.0f;

  float w[B];
  const float* wrow = a.W + (valid ? row : 0) * a.ldw + a.i0;
  if (a.vecw && nb == B) {
#pragma unroll
    for (int q4 = 0; q4 < B / 4; ++q4) {
      float4 v = valid ? *reinterpret_cast<const float4*>(wrow + 4 * q4) : make_float4(0.f, 0.f, 0.f, 0.f);
      w[4 * q4 + 0] = v.x; w[4 * q4 + 1] = v.y; w[4 * q4 + 2] = v.z; w[4 * q4 + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < B; ++j) w[j] = (valid && j < nb) ? wrow[j] : 0.0f;
  }

  float g[K], mid[K - 1];
  float S = 1.0f, Z = 0.0f, invS = 1.0f;
  if (!AFF) {
#pragma unroll
    for (int m = 0; m < K; ++m) g[m] = valid ? a.grid[row * K + m] : 0.0f;
#pragma unroll
    for (int m = 0; m < K - 1; ++m) mid[m] = 0.5f * (g[m] + g[m + 1]);
  }
  __syncthreads();

  uint32_t pk[B / 4];
#pragma unroll
  for (int q4 = 0; q4 < B / 4; ++q4) pk[q4] = 0u;
  float loss = 0.0f;
  const float qmax = (float)(K - 1);

#pragma unroll
  for (int j = 0; j < B; ++j) {
    if (j < nb) {
      float q;
      int code;
      const float wj = w[j];
      if (AFF) {
        const int64_t col = a.i0 + j;
        if (j == 0 || (col % a.group) == 0) {
          const float* sz = a.grid + ((valid ? row : 0) * a.ngroups + col / a.group) * 2;
          S = sz[0];
          Z = sz[1];
          invS = 1.0f / S;
        }
        // Section 2.1: w_int = clip(round(w / S) + Z, 0, 2^b - 1); quant = (w_int - Z) S
        float wi = fminf(fmaxf(rintf(wj * invS) + Z, 0.0f), qmax);
        code = (int)wi;
        q = (wi - Z) * S;
      } else {
        quant_nu<K>(wj, g, mid, q, code);
      }
      const float e = (wj - q) * sRinv[j];
      w[j] = q;
      pk[j >> 2] |= (uint32_t)code << (8 * (j & 3));
      loss = fmaf(0.5f * e, e, loss);
      if (valid) a.Et[(int64_t)j * a.rpad + row] = e;
      const float* urow = sU + j * B;
#pragma unroll
      for (int jj = j + 1; jj < B; ++jj) w[jj] = fmaf(-e, urow[jj], w[jj]);
    }
  }

  if (valid) {
    float* wout = a.W + row * a.ldw + a.i0;
    uint8_t* cout = a.codes + row * a.c + a.i0;
    if (a.vecw && nb == B) {
#pragma unroll
      for (int q4 = 0; q4 < B / 4; ++q4)
        *reinterpret_cast<float4*>(wout + 4 * q4) =
            make_float4(w[4 * q4], w[4 * q4 + 1], w[4 * q4 + 2], w[4 * q4 + 3]);
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j)
        if (j < nb) wout[j] = w[j];
    }
    if (nb == B && ((a.c | a.i0) % 4) == 0) {
#pragma unroll
      for (int q4 = 0; q4 < B / 4; ++q4) reinterpret_cast<uint32_t*>(cout)[q4] = pk[q4];
    } else {
#pragma unroll
      for (int j = 0; j < B; ++j)
        if (j < nb) cout[j] = (uint8_t)((pk[j >> 2] >> (8 * (j & 3))) & 0xffu);
    }
    if (a.row_loss) a.row_loss[row] = (a.first ? 0.0f : a.row_loss[row]) + loss;
  }
}

template <int B>
lq_status launch_column(const ColArgs& a, const lq_params* P, hipStream_t st) {
  const size_t lds = (size_t)(B * B + B) * sizeof(float);
  dim3 grid((unsigned)lq::ceil_div(a.r, QT)), block(QT);
#define LQ_COL(BITS, AFF)                                                                          \
  do {                                                                                             \
    static bool done = false;                                                                      \
    if (!done) {                                                                                   \
      LQ_CHECK_HIP(hipFuncSetAttribute((const void*)column_block_kernel<B, BITS, AFF>,             \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));     \
      done = true;                                                                                 \
    }                                                                                              \
    hipLaunchKernelGGL((column_block_kernel<B, BITS, AFF>), grid, block, lds, st, a);              \
  } while (0)
  const bool aff = P->mode == LQ_GRID_AFFINE;
  if (P->bits == 2) { if (aff) LQ_COL(2, true); else LQ_COL(2, false); }
  else if (P->bits == 3) { if (aff) LQ_COL(3, true); else LQ_COL(3, false); }
  else { if (aff) LQ_COL(4, true); else LQ_COL(4, false); }
#undef LQ_COL
  LQ_CHECK_LAUNCH("column_block_kernel");
  return LQ_OK;
}


lq_status launch_column_128(const ColArgs& a, const lq_params* P, hipStream_t st);
lq_status launch_column_64(const ColArgs& a, const lq_params* P, hipStream_t st);
lq_status launch_column_32(const ColArgs& a, const lq_params* P, hipStream_t st);

}  // namespace lq
