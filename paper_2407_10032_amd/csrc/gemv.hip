// lq_matvec_packed: y = W_hat x straight from the stored form of a quantized layer (packed
// b-bit codes + binary16 tables), the decoding-time product of a quantized linear layer (the
// paper's appendix on inference efficiency describes a dedicated kernel for non-uniform
// grids; this is the gfx950 counterpart for the layout of lq_pack_layer).
//
// HBM bound by design: the packed codes are read exactly once, 16 / 12 / 8 bytes per lane
// and load (32 codes), coalesced; the input vector lives in registers (a lane always serves
// the same columns, for every row of its workgroup), the row's 2^b table values in LDS
// (a 16-entry table spans 16 banks: lookups are conflict-free).  A workgroup walks 8 or 16 rows;
// per row a wavefront reduces its lanes' partial sums by shuffles, the four wavefronts meet
// in LDS at the end.
#include <hip/hip_fp16.h>

#include "lq_common.h"

namespace {

constexpr int NT = 256;
constexpr int UNIT = 32;      // codes per lane and load

struct MvArgs {
  const uint8_t* packed; int64_t packed_ld;
  const uint16_t* table;
  const float* x;
  float* y;
  int64_t r; int c;
  int group; int ngroups;
};

template <int BITS>
__device__ __forceinline__ void load_unit(const uint8_t* p, uint32_t (&w)[BITS]) {
  if constexpr (BITS == 4) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if constexpr (BITS == 2) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    w[0] = v.x; w[1] = v.y;
  } else {
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    w[0] = q[0]; w[1] = q[1]; w[2] = q[2];
  }
}

// code j (0..31) of a unit held as BITS 32-bit words of the little-endian bit stream
template <int BITS, int J>
__device__ __forceinline__ uint32_t unit_code(const uint32_t (&w)[BITS]) {
  constexpr int pos = BITS * J, idx = pos / 32, sh = pos % 32;
  if constexpr (sh + BITS <= 32) return (w[idx] >> sh) & ((1u << BITS) - 1u);
  else return ((w[idx] >> sh) | (w[idx + 1] << (32 - sh))) & ((1u << BITS) - 1u);
}

template <int BITS, bool AFF, int J>
__device__ __forceinline__ void unit_fma(const uint32_t (&w)[BITS], const float (&x)[UNIT],
                                         const float* lut, float& acc) {
  if constexpr (J < UNIT) {
    const uint32_t code = unit_code<BITS, J>(w);
    const float v = AFF ? (float)code : lut[code];
    acc = fmaf(v, x[J], acc);
    unit_fma<BITS, AFF, J + 1>(w, x, lut, acc);
  }
}

// Affine grids at 2 and 4 bits: sum_j code_j x_j of a unit with the codes spread to one per
// byte by a mask (one mask per 4 codes), so that the byte-to-float conversion does the
// extraction: two instructions per weight instead of three.
template <int BITS>
__device__ __forceinline__ float unit_dot_bytes(const uint32_t (&w)[BITS], const float (&x)[UNIT]) {
  static_assert(BITS == 2 || BITS == 4, "codes that do not straddle bytes");
  constexpr int PER_BYTE = 8 / BITS;                 // codes per byte
  constexpr int PER_WORD = 32 / BITS;
  constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x01010101u;
  float dot = 0.0f;
#pragma unroll
  for (int i = 0; i < BITS; ++i) {
#pragma unroll
    for (int s = 0; s < PER_BYTE; ++s) {
      uint32_t m = (w[i] >> (BITS * s)) & MASK;        // byte b holds code PER_BYTE * b + s of the word
      asm volatile("" : "+v"(m));                      // keep the mask: the compiler would go back to bit-field extracts
#pragma unroll
      for (int b = 0; b < 4; ++b)
        dot = fmaf((float)((m >> (8 * b)) & 0xffu), x[PER_WORD * i + PER_BYTE * b + s], dot);
    }
  }
  return dot;
}

// RB rows per workgroup: 16 for layers with many rows (the input vector is re-read per
// workgroup), 8 where that leaves too few workgroups to fill the chip.
template <int BITS, bool AFF, int U, int RB>
__global__ __launch_bounds__(NT) void matvec_packed_kernel(MvArgs a) {
  constexpr int K = 1 << BITS;
  constexpr int UB = UNIT * BITS / 8;                  // bytes per unit
  __shared__ float sLut[RB][K];
  __shared__ float sPart[RB][NT / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row0 = (int64_t)blockIdx.x * RB;
  const int nunits = a.c / UNIT;

  // Units past the end of the row read the row's last unit and count as zero, rows past r
  // read row r - 1 and are discarded: no divergent branches around the loads.
  bool uval[U];
  int uidx[U], gidx[U];
#pragma unroll
  for (int i = 0; i < U; ++i) {
    const int u = tid + i * NT;
    uval[i] = u < nunits;
    uidx[i] = uval[i] ? u : nunits - 1;
    gidx[i] = AFF ? (uidx[i] * UNIT) / a.group : 0;
  }

  // Rows in batches of RG, double buffered: the loads of the next batch are in flight while
  // the current one is looked up and accumulated.
  constexpr int RG = 4 / U;
  static_assert(RB % (2 * RG) == 0, "row batches");
  auto load_batch = [&](int rb0, uint32_t (&w)[RG][U][BITS], uint32_t (&sz)[RG][U]) {
#pragma unroll
    for (int q = 0; q < RG; ++q) {
      int64_t row = row0 + rb0 + q;
      row = row < a.r ? row : a.r - 1;
#pragma unroll
      for (int i = 0; i < U; ++i) {
        load_unit<BITS>(a.packed + row * a.packed_ld + (int64_t)uidx[i] * UB, w[q][i]);
        // affine: binary16 S | int16 Z << 16 of the unit's group
        if (AFF) sz[q][i] = *reinterpret_cast<const uint32_t*>(a.table + (row * a.ngroups + gidx[i]) * 2);
        if (!uval[i]) {
#pragma unroll
          for (int b = 0; b < BITS; ++b) w[q][i][b] = 0u;
        }
      }
    }
  };
  // everything the first batch needs is requested at once: codes, tables, x
  uint32_t wa[RG][U][BITS], wb[RG][U][BITS];
  uint32_t sa[RG][U], sb[RG][U];
  load_batch(0, wa, sa);
  static_assert(RB * K <= NT, "one table entry per thread");
  uint16_t tab = 0;
  if (!AFF && tid < RB * K) {
    int64_t row = row0 + tid / K;
    row = row < a.r ? row : a.r - 1;
    tab = a.table[row * K + tid % K];
  }
  // this lane's columns of x, and their sums (affine: the zero-point term)
  float x[U][UNIT];
  float xsum[U];
#pragma unroll
  for (int i = 0; i < U; ++i) {
    xsum[i] = 0.0f;
#pragma unroll
    for (int q4 = 0; q4 < UNIT / 4; ++q4) {
      float4 v = *reinterpret_cast<const float4*>(a.x + (int64_t)uidx[i] * UNIT + 4 * q4);
      if (!uval[i]) v = make_float4(0.f, 0.f, 0.f, 0.f);
      x[i][4 * q4 + 0] = v.x; x[i][4 * q4 + 1] = v.y; x[i][4 * q4 + 2] = v.z; x[i][4 * q4 + 3] = v.w;
      xsum[i] += (v.x + v.y) + (v.z + v.w);
    }
  }
  if (!AFF && tid < RB * K) sLut[tid / K][tid % K] = __half2float(__ushort_as_half(tab));
  __syncthreads();

  auto use_batch = [&](int rb0, const uint32_t (&w)[RG][U][BITS], const uint32_t (&sz)[RG][U]) {
#pragma unroll
    for (int q = 0; q < RG; ++q) {
      const int rb = rb0 + q;
      int64_t row = row0 + rb;
      row = row < a.r ? row : a.r - 1;
      float acc = 0.0f;
#pragma unroll
      for (int i = 0; i < U; ++i) {
        if (AFF) {
          // Section 2.1: (w_int - Z) S, with the unit's group pair: S (sum code x - Z sum x)
          const float S = __half2float(__ushort_as_half((uint16_t)(sz[q][i] & 0xffffu)));
          const float Z = (float)(int16_t)(sz[q][i] >> 16);
          float dot = 0.0f;
          if constexpr (BITS == 3) unit_fma<BITS, true, 0>(w[q][i], x[i], nullptr, dot);
          else dot = unit_dot_bytes<BITS>(w[q][i], x[i]);
          acc = fmaf(S, dot - Z * xsum[i], acc);
        } else {
          unit_fma<BITS, false, 0>(w[q][i], x[i], sLut[rb], acc);
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
      if (lane == 0) sPart[rb][wave] = acc;
    }
  };
#pragma unroll
  for (int rb0 = 0; rb0 < RB; rb0 += 2 * RG) {
    load_batch(rb0 + RG, wb, sb);
    use_batch(rb0, wa, sa);
    if (rb0 + 2 * RG < RB) load_batch(rb0 + 2 * RG, wa, sa);
    use_batch(rb0 + RG, wb, sb);
  }
  __syncthreads();
  if (tid < RB && row0 + tid < a.r) {
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) s += sPart[tid][w];
    a.y[row0 + tid] = s;
  }
}

template <int BITS, bool AFF>
void launch_mv(const MvArgs& a, int U, hipStream_t st) {
  dim3 block(NT);
  if (a.r < 16 * 1024) {
    dim3 grid((unsigned)lq::ceil_div(a.r, 8));
    if (U <= 1) hipLaunchKernelGGL((matvec_packed_kernel<BITS, AFF, 1, 8>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((matvec_packed_kernel<BITS, AFF, 2, 8>), grid, block, 0, st, a);
  } else {
    dim3 grid((unsigned)lq::ceil_div(a.r, 16));
    if (U <= 1) hipLaunchKernelGGL((matvec_packed_kernel<BITS, AFF, 1, 16>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((matvec_packed_kernel<BITS, AFF, 2, 16>), grid, block, 0, st, a);
  }
}

}  // namespace

extern "C" lq_status lq_matvec_packed(const uint8_t* packed, int64_t packed_ld, const uint16_t* table,
                                      int64_t r, int64_t c, const lq_params* P, const float* X,
                                      int64_t nb, float* Y, void* stream) {
  if (r < 0 || c < 1 || nb < 0) return lq::fail(LQ_ERR_INVALID_ARG, "lq_matvec_packed: r=%lld c=%lld nb=%lld", (long long)r, (long long)c, (long long)nb);
  lq_status stt = lq::check_params(P, c);
  if (stt != LQ_OK) return stt;
  if (r == 0 || nb == 0) return LQ_OK;
  if (!packed || !table || !X || !Y) return lq::fail(LQ_ERR_INVALID_ARG, "lq_matvec_packed: null pointer");
  const int64_t row_bytes = (c * P->bits + 7) / 8;
  if (packed_ld < row_bytes) return lq::fail(LQ_ERR_INVALID_ARG, "lq_matvec_packed: packed_ld too small");
  const int align = P->bits == 4 ? 16 : (P->bits == 2 ? 8 : 4);
  if (c % UNIT != 0 || c > 2 * NT * UNIT)
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matvec_packed: c must be a multiple of %d and at most %d", UNIT, 2 * NT * UNIT);
  if (packed_ld % align != 0 || !lq::aligned(packed, align) || !lq::aligned(X, 16) || !lq::aligned(table, 4))
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matvec_packed: packed rows must be %d-byte aligned, X 16-byte aligned", align);
  const bool aff = P->mode == LQ_GRID_AFFINE;
  const int64_t g = (aff && P->group_size > 0) ? P->group_size : c;
  if (aff && g % UNIT != 0) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_matvec_packed: affine groups must be multiples of %d columns", UNIT);
  hipStream_t st = (hipStream_t)stream;
  const int U = (int)lq::ceil_div(c / UNIT, NT);
  for (int64_t n = 0; n < nb; ++n) {       // one pass over the codes per input vector
    MvArgs a;
    a.packed = packed; a.packed_ld = packed_ld; a.table = table;
    a.x = X + n * c; a.y = Y + n * r; a.r = r; a.c = (int)c;
    a.group = (int)g; a.ngroups = (int)(c / g);
    if (P->bits == 2) { if (aff) launch_mv<2, true>(a, U, st); else launch_mv<2, false>(a, U, st); }
    else if (P->bits == 3) { if (aff) launch_mv<3, true>(a, U, st); else launch_mv<3, false>(a, U, st); }
    else { if (aff) launch_mv<4, true>(a, U, st); else launch_mv<4, false>(a, U, st); }
    LQ_CHECK_LAUNCH("matvec_packed_kernel");
  }
  return LQ_OK;
}
