// lq_matmul_packed: Y = X W_hat^T for a batch of input vectors, straight from the stored form
// of a quantized layer (packed b-bit codes + binary16 tables) -- the batched form of the
// decoding-time product that the paper's appendix on inference efficiency builds a kernel
// for.  lq_matvec_packed walks the codes once per 4 vectors on the vector ALU; here a weight
// is decoded once per 32 or 64 vectors into an fp32 tile in LDS and the products run on the
// fp32 matrix cores (v_mfma_f32_32x32x2_f32), fp32 accumulation in a fixed order.
//
// A workgroup (4 wavefronts) owns 128 rows of W_hat and 32 MT input vectors (MT = 1 or 2) and
// walks the columns in stages of 64:
//   * decode: thread (row, unit) loads one unit of 32 codes (16 / 12 / 8 bytes), turns each
//     code into its weight -- table lookup in LDS (non-uniform) or fma(code, S, -Z S) with the
//     unit's group pair (affine) -- and writes the 32 floats into the row of the LDS tile;
//   * the X tile is copied as it lies in memory (vectors are rows);
//   * both tiles have odd row strides (65 floats), so the MFMA operand reads -- lane l takes
//     element (row l % 32, column 2 kk + l / 32) -- hit 32 distinct banks, and the k loop holds
//     nothing but LDS reads with immediate offsets and MFMAs;
//   * wavefront w multiplies the X tile with rows 32 w .. 32 w + 31 of the weight tile; its
//     accumulators are Y[vector][row] with the row index along the lanes, so the final stores
//     are 128-byte runs of a vector's outputs.
// The loads of the next stage (codes, group pairs, X) are issued before the current stage's
// MFMA loop.  Two or three workgroups share a compute unit, so one decodes while another
// multiplies.  Layers with few rows take a second kernel (32 rows per workgroup, the columns
// split over its wavefronts) that fills the chip where r / 128 workgroups would not.
#include <hip/hip_fp16.h>

#include "lq_common.h"
#include "lq_mfma.h"
#include "lq_unpack.h"

namespace {

using lq::floatx16;
using lq::UNIT;

constexpr int NT = 256;
constexpr int KS = 64;          // columns per stage (two units)
constexpr int WROWS = 128;      // rows of W_hat per workgroup
constexpr int LDT = KS + 1;     // row stride of the LDS tiles

struct MmArgs {
  const uint8_t* packed; int64_t packed_ld;
  const uint16_t* table;
  const float* x;      // [nb x c]
  float* y;            // [nb x r]
  int64_t r; int c; int64_t nb;
  int group; int ngroups;
};

template <int BITS, bool AFF, int J>
__device__ __forceinline__ void decode_unit(const uint32_t (&w)[BITS], const float* lut, float S, float ZS,
                                            bool valid, float* dst) {
  if constexpr (J < UNIT) {
    const uint32_t code = lq::unit_code<BITS, J>(w);
    // Section 2.1: table[code], or (w_int - Z) S
    float v = AFF ? fmaf((float)code, S, -ZS) : lut[code];
    dst[J] = valid ? v : 0.0f;
    decode_unit<BITS, AFF, J + 1>(w, lut, S, ZS, valid, dst);
  }
}

template <int BITS, bool AFF, int MT>
__global__ __launch_bounds__(NT, 2) void matmul_packed_kernel(MmArgs a) {
  constexpr int K = 1 << BITS;
  constexpr int UB = UNIT * BITS / 8;                  // bytes per unit
  constexpr int XROWS = 32 * MT;
  constexpr int XQ = XROWS * (KS / 4) / NT;            // float4 loads of the X tile per thread
  __shared__ float sW[WROWS * LDT];
  __shared__ float sX[XROWS * LDT];
  __shared__ float sLut[AFF ? 1 : WROWS * K];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ml = lane & 31, hl = lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.x * WROWS;
  const int64_t n0 = (int64_t)blockIdx.y * XROWS;
  const int nunits = a.c / UNIT;

  // decode assignment: thread -> (row of the tile, first or second unit of the stage); rows
  // past r read row r - 1 (their results are never stored)
  const int drow = tid >> 1, dunit = tid & 1;
  int64_t grow = row0 + drow;
  grow = grow < a.r ? grow : a.r - 1;
  const uint8_t* prow = a.packed + grow * a.packed_ld;

  if (!AFF) {
    for (int i = tid; i < WROWS * K; i += NT) {
      int64_t rr = row0 + i / K;
      rr = rr < a.r ? rr : a.r - 1;
      sLut[i] = __half2float(__ushort_as_half(a.table[rr * K + i % K]));
    }
  }

  uint32_t wreg[BITS];
  uint32_t szreg = 0;
  float4 xreg[XQ];
  bool uok = false;
  auto prefetch = [&](int k0) {
    const int u = k0 / UNIT + dunit;
    uok = u < nunits;
    const int uu = uok ? u : nunits - 1;
    lq::load_unit<BITS>(prow + (int64_t)uu * UB, wreg);
    // affine: binary16 S | int16 Z << 16 of the unit's group
    if (AFF) szreg = *reinterpret_cast<const uint32_t*>(a.table + (grow * a.ngroups + (uu * UNIT) / a.group) * 2);
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
      const int idx = tid + q * NT;
      const int n = idx / (KS / 4), k4 = idx % (KS / 4);
      const int64_t gn = n0 + n;
      const int kcol = k0 + 4 * k4;
      xreg[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (gn < a.nb && kcol < a.c) xreg[q] = *reinterpret_cast<const float4*>(a.x + gn * a.c + kcol);
    }
  };

  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.0f;

  prefetch(0);
  for (int k0 = 0; k0 < a.c; k0 += KS) {
    __syncthreads();                 // the previous stage's operand reads are done (first pass: the table is in LDS)
    {
      float S = 1.0f, ZS = 0.0f;
      if (AFF) {
        S = __half2float(__ushort_as_half((uint16_t)(szreg & 0xffffu)));
        ZS = (float)(int16_t)(szreg >> 16) * S;
      }
      decode_unit<BITS, AFF, 0>(wreg, sLut + (AFF ? 0 : drow * K), S, ZS, uok, sW + drow * LDT + dunit * UNIT);
#pragma unroll
      for (int q = 0; q < XQ; ++q) {
        const int idx = tid + q * NT;
        const int n = idx / (KS / 4), k4 = idx % (KS / 4);
        float* d = sX + n * LDT + 4 * k4;
        d[0] = xreg[q].x; d[1] = xreg[q].y; d[2] = xreg[q].z; d[3] = xreg[q].w;
      }
    }
    __syncthreads();
    if (k0 + KS < a.c) prefetch(k0 + KS);
    const float* pb = sW + (32 * wave + ml) * LDT + hl;
    const float* pa = sX + ml * LDT + hl;
#pragma unroll
    for (int kk = 0; kk < KS / 2; ++kk) {
      const float b = pb[2 * kk];
#pragma unroll
      for (int m = 0; m < MT; ++m)
        acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[m * 32 * LDT + 2 * kk], b, acc[m], 0, 0, 0);
    }
  }

  const int64_t row = row0 + 32 * wave + ml;
  if (row < a.r) {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t n = n0 + 32 * m + 8 * (v >> 2) + 4 * hl + (v & 3);
        if (n < a.nb) a.y[n * a.r + row] = acc[m][v];
      }
    }
  }
}

// Layers with few rows: the 128-row tiling above gives r / 128 workgroups per 64 vectors, far
// fewer than the chip has compute units.  Here a workgroup owns 32 rows of W_hat and 32 MT
// vectors, and its four wavefronts split the columns: wavefront w takes the 64-column chunks
// w, w + 4, w + 8, ... and runs the whole decode -> LDS -> MFMA pipeline on tiles of its own (no
// workgroup barrier inside the loop: a wavefront's LDS accesses are served in order).  The four
// partial results are added in wavefront order at the end, so the sums are again fixed.
template <int BITS, bool AFF, int MT>
__global__ __launch_bounds__(NT) void matmul_packed_rows32_kernel(MmArgs a) {
  constexpr int K = 1 << BITS;
  constexpr int UB = UNIT * BITS / 8;
  constexpr int XROWS = 32 * MT;
  constexpr int XQ = XROWS * (KS / 4) / 64;            // float4 loads of a wavefront's X tile per lane
  constexpr int WTILE = 32 * LDT;                      // floats
  constexpr int XTILE = XROWS * LDT;
  extern __shared__ __align__(16) float dyn[];         // [4][WTILE + XTILE], then the table (non-uniform)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ml = lane & 31, hl = lane >> 5;
  const int64_t row0 = (int64_t)blockIdx.x * 32;
  const int64_t n0 = (int64_t)blockIdx.y * XROWS;
  const int nunits = a.c / UNIT;
  float* sW = dyn + wave * (WTILE + XTILE);
  float* sX = sW + WTILE;
  float* sLut = dyn + 4 * (WTILE + XTILE);

  const int drow = lane >> 1, dunit = lane & 1;
  int64_t grow = row0 + drow;
  grow = grow < a.r ? grow : a.r - 1;
  const uint8_t* prow = a.packed + grow * a.packed_ld;

  if (!AFF) {
    for (int i = tid; i < 32 * K; i += NT) {
      int64_t rr = row0 + i / K;
      rr = rr < a.r ? rr : a.r - 1;
      sLut[i] = __half2float(__ushort_as_half(a.table[rr * K + i % K]));
    }
    __syncthreads();
  }

  uint32_t wreg[BITS];
  uint32_t szreg = 0;
  float4 xreg[XQ];
  bool uok = false;
  auto prefetch = [&](int k0) {
    const int u = k0 / UNIT + dunit;
    uok = u < nunits;
    const int uu = uok ? u : nunits - 1;
    lq::load_unit<BITS>(prow + (int64_t)uu * UB, wreg);
    if (AFF) szreg = *reinterpret_cast<const uint32_t*>(a.table + (grow * a.ngroups + (uu * UNIT) / a.group) * 2);
#pragma unroll
    for (int q = 0; q < XQ; ++q) {
      const int idx = lane + q * 64;
      const int n = idx / (KS / 4), k4 = idx % (KS / 4);
      const int64_t gn = n0 + n;
      const int kcol = k0 + 4 * k4;
      xreg[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (gn < a.nb && kcol < a.c) xreg[q] = *reinterpret_cast<const float4*>(a.x + gn * a.c + kcol);
    }
  };

  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.0f;

  const int kstep = 4 * KS;
  int k0 = wave * KS;
  if (k0 < a.c) prefetch(k0);
  for (; k0 < a.c; k0 += kstep) {
    {
      float S = 1.0f, ZS = 0.0f;
      if (AFF) {
        S = __half2float(__ushort_as_half((uint16_t)(szreg & 0xffffu)));
        ZS = (float)(int16_t)(szreg >> 16) * S;
      }
      decode_unit<BITS, AFF, 0>(wreg, sLut + (AFF ? 0 : drow * K), S, ZS, uok, sW + drow * LDT + dunit * UNIT);
#pragma unroll
      for (int q = 0; q < XQ; ++q) {
        const int idx = lane + q * 64;
        const int n = idx / (KS / 4), k4 = idx % (KS / 4);
        float* d = sX + n * LDT + 4 * k4;
        d[0] = xreg[q].x; d[1] = xreg[q].y; d[2] = xreg[q].z; d[3] = xreg[q].w;
      }
    }
    __builtin_amdgcn_wave_barrier();      // the tiles are this wavefront's own: ordering inside the wavefront is enough
    if (k0 + kstep < a.c) prefetch(k0 + kstep);
    const float* pb = sW + ml * LDT + hl;
    const float* pa = sX + ml * LDT + hl;
#pragma unroll
    for (int kk = 0; kk < KS / 2; ++kk) {
      const float b = pb[2 * kk];
#pragma unroll
      for (int m = 0; m < MT; ++m)
        acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[m * 32 * LDT + 2 * kk], b, acc[m], 0, 0, 0);
    }
    __builtin_amdgcn_wave_barrier();
  }

  // partial results of the four wavefronts -> LDS, added in wavefront order
  __syncthreads();
  float* red = dyn;                                    // [4][MT][16][64]
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wave * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
  __syncthreads();
  for (int o = tid; o < MT * 16 * 64; o += NT) {
    const int l = o & 63, v = (o >> 6) & 15, m = o >> 10;
    float sum = red[o];
#pragma unroll
    for (int w = 1; w < 4; ++w) sum += red[w * MT * 16 * 64 + o];
    const int64_t row = row0 + (l & 31);
    const int64_t n = n0 + 32 * m + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
    if (row < a.r && n < a.nb) a.y[n * a.r + row] = sum;
  }
}

template <int BITS, bool AFF, int MT>
constexpr size_t rows32_lds() {
  return (size_t)(4 * (32 * LDT + 32 * MT * LDT) + (AFF ? 0 : 32 * (1 << BITS))) * sizeof(float);
}

// fewer 128-row workgroups than this: the 32-row kernel fills the chip better (measured: for up
// to 32 vectors it still leads at 224 workgroups, for 64 it no longer does)
constexpr int64_t ROWS32_BELOW = 192;
constexpr int64_t ROWS32_BELOW_SMALL_BATCH = 320;

template <int BITS, bool AFF>
lq_status launch_mm(const MmArgs& a, hipStream_t st) {
  const unsigned gx = (unsigned)lq::ceil_div(a.r, WROWS);
  const int64_t vt = a.nb <= 32 ? 32 : 64;
  if ((int64_t)gx * lq::ceil_div(a.nb, vt) < (a.nb <= 32 ? ROWS32_BELOW_SMALL_BATCH : ROWS32_BELOW)) {
    static lq::DeviceOnce attr_once;
    if (lq::DeviceOnceGuard once(attr_once); once.first()) {
      LQ_CHECK_HIP(hipFuncSetAttribute((const void*)matmul_packed_rows32_kernel<BITS, AFF, 1>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)rows32_lds<BITS, AFF, 1>()));
      LQ_CHECK_HIP(hipFuncSetAttribute((const void*)matmul_packed_rows32_kernel<BITS, AFF, 2>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)rows32_lds<BITS, AFF, 2>()));
      once.done();
    }
    const unsigned gr = (unsigned)lq::ceil_div(a.r, 32);
    const size_t lds1 = rows32_lds<BITS, AFF, 1>(), lds2 = rows32_lds<BITS, AFF, 2>();
    if (a.nb <= 32)
      hipLaunchKernelGGL((matmul_packed_rows32_kernel<BITS, AFF, 1>), dim3(gr, 1), dim3(NT), lds1, st, a);
    else
      hipLaunchKernelGGL((matmul_packed_rows32_kernel<BITS, AFF, 2>), dim3(gr, (unsigned)lq::ceil_div(a.nb, 64)), dim3(NT), lds2, st, a);
    return LQ_OK;
  }
  if (a.nb <= 32) {
    hipLaunchKernelGGL((matmul_packed_kernel<BITS, AFF, 1>), dim3(gx, (unsigned)lq::ceil_div(a.nb, 32)), dim3(NT), 0, st, a);
  } else {
    hipLaunchKernelGGL((matmul_packed_kernel<BITS, AFF, 2>), dim3(gx, (unsigned)lq::ceil_div(a.nb, 64)), dim3(NT), 0, st, a);
  }
  return LQ_OK;
}

}  // namespace

extern "C" lq_status lq_matmul_packed(const uint8_t* packed, int64_t packed_ld, const uint16_t* table,
                                      int64_t r, int64_t c, const lq_params* P, const float* X,
                                      int64_t nb, float* Y, void* stream) {
  if (r < 0 || c < 1 || nb < 0) return lq::fail(LQ_ERR_INVALID_ARG, "lq_matmul_packed: r=%lld c=%lld nb=%lld", (long long)r, (long long)c, (long long)nb);
  lq_status stt = lq::check_params(P, c);
  if (stt != LQ_OK) return stt;
  if (r == 0 || nb == 0) return LQ_OK;
  if (!packed || !table || !X || !Y) return lq::fail(LQ_ERR_INVALID_ARG, "lq_matmul_packed: null pointer");
  const int64_t row_bytes = (c * P->bits + 7) / 8;
  if (packed_ld < row_bytes) return lq::fail(LQ_ERR_INVALID_ARG, "lq_matmul_packed: packed_ld too small");
  const int align = P->bits == 4 ? 16 : (P->bits == 2 ? 8 : 4);
  if (c % UNIT != 0 || c > (1 << 30))
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matmul_packed: c must be a multiple of %d", UNIT);
  if (packed_ld % align != 0 || !lq::aligned(packed, align) || !lq::aligned(X, 16) || !lq::aligned(table, 4))
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matmul_packed: packed rows must be %d-byte aligned, X 16-byte aligned", align);
  if (nb > 65535LL * 64) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matmul_packed: nb too large for one launch");
  const bool aff = P->mode == LQ_GRID_AFFINE;
  const int64_t g = (aff && P->group_size > 0) ? P->group_size : c;
  if (aff && g % UNIT != 0) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matmul_packed: affine groups must be multiples of %d columns", UNIT);
  MmArgs a;
  a.packed = packed; a.packed_ld = packed_ld; a.table = table;
  a.x = X; a.y = Y; a.r = r; a.c = (int)c; a.nb = nb;
  a.group = (int)g; a.ngroups = (int)(c / g);
  hipStream_t st = (hipStream_t)stream;
  lq_status rc;
  if (P->bits == 2) rc = aff ? launch_mm<2, true>(a, st) : launch_mm<2, false>(a, st);
  else if (P->bits == 3) rc = aff ? launch_mm<3, true>(a, st) : launch_mm<3, false>(a, st);
  else rc = aff ? launch_mm<4, true>(a, st) : launch_mm<4, false>(a, st);
  if (rc != LQ_OK) return rc;
  LQ_CHECK_LAUNCH("matmul_packed_kernel");
  return LQ_OK;
}
