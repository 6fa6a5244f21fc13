// lq_pack_layer / lq_unpack_layer: the stored form of a quantized layer.
//
// The paper's result tables count b bits per weight plus sixteen bits per grid point per
// row (non-uniform grids, Section 2.1: one set of 2^b points per row) or per scale and
// zero-point per group (affine grids): their "Bits" columns read 4.05 / 3.02 / 2.01 and 4.25
// at group size 128.  Layout: a row's codes are a little-endian bit stream (code j in bits
// [j b, (j + 1) b)), ceil(c b / 8) bytes per row; tables are IEEE binary16 (round to nearest
// even), the affine zero-point an int16.  Plain HBM-bound kernels: one thread handles eight
// codes, i.e. b whole bytes of the stream.
#include <hip/hip_fp16.h>

#include "lq_common.h"

namespace {

__device__ __forceinline__ uint16_t half_bits(float x) { return __half_as_ushort(__float2half_rn(x)); }
__device__ __forceinline__ float half_value(uint16_t h) { return __half2float(__ushort_as_half(h)); }

template <int BITS>
__global__ __launch_bounds__(256) void pack_codes_kernel(const uint8_t* __restrict__ codes, int64_t r,
                                                         int64_t c, uint8_t* __restrict__ packed,
                                                         int64_t packed_ld) {
  const int64_t groups = (c + 7) / 8;                       // groups of eight codes per row
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= r * groups) return;
  const int64_t row = t / groups, gi = t - row * groups;
  const uint8_t* src = codes + row * c + gi * 8;
  const int n = (int)((c - gi * 8 < 8) ? (c - gi * 8) : 8);
  uint32_t v = 0;
  if (n == 8 && ((reinterpret_cast<uintptr_t>(src) & 7) == 0)) {
    const uint64_t q = *reinterpret_cast<const uint64_t*>(src);
#pragma unroll
    for (int j = 0; j < 8; ++j) v |= (uint32_t)((q >> (8 * j)) & ((1u << BITS) - 1u)) << (BITS * j);
  } else {
    for (int j = 0; j < n; ++j) v |= ((uint32_t)src[j] & ((1u << BITS) - 1u)) << (BITS * j);
  }
  const int64_t row_bytes = (c * BITS + 7) / 8;
  uint8_t* dst = packed + row * packed_ld + gi * BITS;
  const int nbytes = (int)((row_bytes - gi * BITS < BITS) ? (row_bytes - gi * BITS) : BITS);
  for (int b = 0; b < nbytes; ++b) dst[b] = (uint8_t)(v >> (8 * b));
}

__global__ __launch_bounds__(256) void table_nu_kernel(const float* __restrict__ grid, int64_t n,
                                                       uint16_t* __restrict__ table) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) table[i] = half_bits(grid[i]);
}

__global__ __launch_bounds__(256) void table_aff_kernel(const float* __restrict__ grid, int64_t npairs,
                                                        uint16_t* __restrict__ table) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= npairs) return;
  table[2 * i] = half_bits(grid[2 * i]);
  const float z = fminf(fmaxf(rintf(grid[2 * i + 1]), -32768.0f), 32767.0f);
  table[2 * i + 1] = (uint16_t)(int16_t)(int)z;
}

template <int BITS, bool AFF>
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t* __restrict__ packed, int64_t packed_ld,
                                                     const uint16_t* __restrict__ table, int64_t r,
                                                     int64_t c, int group, int ngroups,
                                                     float* __restrict__ W, int64_t ldw,
                                                     uint8_t* __restrict__ codes) {
  constexpr int K = 1 << BITS;
  const int64_t groups = (c + 7) / 8;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= r * groups) return;
  const int64_t row = t / groups, gi = t - row * groups;
  const int64_t col0 = gi * 8;
  const int n = (int)((c - col0 < 8) ? (c - col0) : 8);
  const int64_t row_bytes = (c * BITS + 7) / 8;
  const uint8_t* src = packed + row * packed_ld + gi * BITS;
  const int nbytes = (int)((row_bytes - gi * BITS < BITS) ? (row_bytes - gi * BITS) : BITS);
  uint32_t v = 0;
  for (int b = 0; b < nbytes; ++b) v |= (uint32_t)src[b] << (8 * b);
  for (int j = 0; j < n; ++j) {
    const uint32_t code = (v >> (BITS * j)) & (K - 1);
    float w;
    if (AFF) {
      // Section 2.1: (w_int - Z) S with the group's stored scale and zero-point
      const uint16_t* sz = table + (row * ngroups + (col0 + j) / group) * 2;
      w = ((float)code - (float)(int16_t)sz[1]) * half_value(sz[0]);
    } else {
      w = half_value(table[row * K + code]);
    }
    W[row * ldw + col0 + j] = w;
    if (codes) codes[row * c + col0 + j] = (uint8_t)code;
  }
}

lq_status check_common(const char* who, int64_t r, int64_t c, const lq_params* P) {
  if (r < 0 || c < 1) return lq::fail(LQ_ERR_INVALID_ARG, "%s: r=%lld c=%lld", who, (long long)r, (long long)c);
  return lq::check_params(P, c);
}

}  // namespace

extern "C" int64_t lq_packed_row_bytes(int64_t c, int32_t bits) {
  if (c < 0 || bits < 1 || bits > 8) return -1;
  return (c * bits + 7) / 8;
}

extern "C" double lq_bits_per_weight(int64_t r, int64_t c, const lq_params* P) {
  (void)r;
  if (!P || c < 1 || lq::check_params(P, c) != LQ_OK) return -1.0;
  if (P->mode == LQ_GRID_NONUNIFORM) return (double)P->bits + 16.0 * (double)(1 << P->bits) / (double)c;
  const int64_t g = P->group_size > 0 ? P->group_size : c;
  return (double)P->bits + 32.0 / (double)g;
}

extern "C" lq_status lq_pack_layer(const uint8_t* codes, const float* grid, int64_t r, int64_t c,
                                   const lq_params* P, uint8_t* packed, int64_t packed_ld,
                                   uint16_t* table, void* stream) {
  lq_status st0 = check_common("lq_pack_layer", r, c, P);
  if (st0 != LQ_OK) return st0;
  if (r == 0) return LQ_OK;
  if (!codes || !grid || !packed || !table) return lq::fail(LQ_ERR_INVALID_ARG, "lq_pack_layer: null pointer");
  const int64_t row_bytes = (c * P->bits + 7) / 8;
  if (packed_ld < row_bytes) return lq::fail(LQ_ERR_INVALID_ARG, "lq_pack_layer: packed_ld %lld < %lld bytes per row", (long long)packed_ld, (long long)row_bytes);
  hipStream_t st = (hipStream_t)stream;
  const int64_t threads = r * ((c + 7) / 8);
  dim3 grid1((unsigned)lq::ceil_div(threads, 256)), block(256);
  if (lq::ceil_div(threads, 256) > 0x7fffffffLL) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_pack_layer: layer too large");
  switch (P->bits) {
    case 2: hipLaunchKernelGGL(pack_codes_kernel<2>, grid1, block, 0, st, codes, r, c, packed, packed_ld); break;
    case 3: hipLaunchKernelGGL(pack_codes_kernel<3>, grid1, block, 0, st, codes, r, c, packed, packed_ld); break;
    default: hipLaunchKernelGGL(pack_codes_kernel<4>, grid1, block, 0, st, codes, r, c, packed, packed_ld); break;
  }
  LQ_CHECK_LAUNCH("pack_codes_kernel");
  if (P->mode == LQ_GRID_NONUNIFORM) {
    const int64_t n = r * (1 << P->bits);
    hipLaunchKernelGGL(table_nu_kernel, dim3((unsigned)lq::ceil_div(n, 256)), block, 0, st, grid, n, table);
  } else {
    const int64_t g = P->group_size > 0 ? P->group_size : c;
    const int64_t n = r * (c / g);
    hipLaunchKernelGGL(table_aff_kernel, dim3((unsigned)lq::ceil_div(n, 256)), block, 0, st, grid, n, table);
  }
  LQ_CHECK_LAUNCH("table kernel");
  return LQ_OK;
}

extern "C" lq_status lq_unpack_layer(const uint8_t* packed, int64_t packed_ld, const uint16_t* table,
                                     int64_t r, int64_t c, const lq_params* P, float* W_hat,
                                     int64_t ldw, uint8_t* codes, void* stream) {
  lq_status st0 = check_common("lq_unpack_layer", r, c, P);
  if (st0 != LQ_OK) return st0;
  if (r == 0) return LQ_OK;
  if (!packed || !table || !W_hat) return lq::fail(LQ_ERR_INVALID_ARG, "lq_unpack_layer: null pointer");
  const int64_t row_bytes = (c * P->bits + 7) / 8;
  if (packed_ld < row_bytes || ldw < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_unpack_layer: leading dimension too small");
  hipStream_t st = (hipStream_t)stream;
  const int64_t threads = r * ((c + 7) / 8);
  if (lq::ceil_div(threads, 256) > 0x7fffffffLL) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_unpack_layer: layer too large");
  dim3 grid1((unsigned)lq::ceil_div(threads, 256)), block(256);
  const bool aff = P->mode == LQ_GRID_AFFINE;
  const int64_t g = (aff && P->group_size > 0) ? P->group_size : c;
  const int group = (int)g, ngroups = (int)(c / g);
#define LQ_UNPACK(B, A) hipLaunchKernelGGL((unpack_kernel<B, A>), grid1, block, 0, st, packed, packed_ld, table, r, c, group, ngroups, W_hat, ldw, codes)
  if (P->bits == 2) { if (aff) LQ_UNPACK(2, true); else LQ_UNPACK(2, false); }
  else if (P->bits == 3) { if (aff) LQ_UNPACK(3, true); else LQ_UNPACK(3, false); }
  else { if (aff) LQ_UNPACK(4, true); else LQ_UNPACK(4, false); }
#undef LQ_UNPACK
  LQ_CHECK_LAUNCH("unpack_kernel");
  return LQ_OK;
}
