// lq_matvec_packed: y = W_hat x straight from the stored form of a quantized layer (packed
// b-bit codes + binary16 tables), the decoding-time product of a quantized linear layer (the
// paper's appendix on inference efficiency describes a dedicated kernel for non-uniform
// grids; this is the gfx950 counterpart for the layout of lq_pack_layer).
//
// The packed codes are read exactly once per pass, 16 / 12 / 8 bytes per lane and load (32
// codes), coalesced; the input vectors (up to 4 per pass) live in registers (a lane always
// serves the same columns, for every row of its workgroup), the row's 2^b table values in
// LDS (a 16-entry table spans 16 banks: lookups are conflict-free).  A workgroup walks 8 or
// 16 rows; per row a wavefront adds its lanes' partial sums with DPP adds, the four
// wavefronts meet in LDS at the end.  What limits it is instruction issue (one LDS lookup
// or 2.4 vector instructions per weight), not HBM.
#include <hip/hip_fp16.h>

#include "lq_common.h"
#include "lq_unpack.h"

namespace {

using lq::UNIT;
using lq::load_unit;
using lq::unit_code;

constexpr int NT = 256;

struct MvArgs {
  const uint8_t* packed; int64_t packed_ld;
  const uint16_t* table;
  const float* x;      // NBV input vectors, c apart
  float* y;            // NBV output vectors, r apart
  int64_t r; int c;
  int group; int ngroups;
};

// One unit of a row against the same 32 columns of NBV input vectors: a weight is decoded
// once and used NBV times.
template <int BITS, bool AFF, int NBV, int J>
__device__ __forceinline__ void unit_fma(const uint32_t (&w)[BITS], const float (&x)[NBV][UNIT],
                                         const float* lut, float (&acc)[NBV]) {
  if constexpr (J < UNIT) {
    const uint32_t code = unit_code<BITS, J>(w);
    const float v = AFF ? (float)code : lut[code];
#pragma unroll
    for (int n = 0; n < NBV; ++n) acc[n] = fmaf(v, x[n][J], acc[n]);
    unit_fma<BITS, AFF, NBV, J + 1>(w, x, lut, acc);
  }
}

// Sum over the 64 lanes of a wavefront, delivered in lane 63.  Data-parallel-primitive
// modifiers on the adds (quad permutes, row shifts, row broadcasts) instead of shuffles: the
// latter go through the LDS crossbar and, with a wait each, cost more than a row's products.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  // lanes without a source read 0.0f (the `old` operand)
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_lane63(float v) {
  v = dpp_add<0xb1, 0xf>(v);    // quad_perm [1, 0, 3, 2]
  v = dpp_add<0x4e, 0xf>(v);    // quad_perm [2, 3, 0, 1]: every lane holds its quad's sum
  v = dpp_add<0x114, 0xf>(v);   // row_shr:4
  v = dpp_add<0x118, 0xf>(v);   // row_shr:8: lanes 12-15 of a row hold the row's sum
  v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3: lane 63 holds all 64
  return v;
}

// Affine grids at 2 and 4 bits: sum_j code_j x_j of a unit with the codes spread to one per
// byte by a mask (one mask per 4 codes), so that the byte-to-float conversion does the
// extraction: two instructions per weight instead of three.
template <int BITS, int NBV>
__device__ __forceinline__ void unit_dot_bytes(const uint32_t (&w)[BITS], const float (&x)[NBV][UNIT],
                                               float (&dot)[NBV]) {
  static_assert(BITS == 2 || BITS == 4, "codes that do not straddle bytes");
  constexpr int PER_BYTE = 8 / BITS;                 // codes per byte
  constexpr int PER_WORD = 32 / BITS;
  constexpr uint32_t MASK = ((1u << BITS) - 1u) * 0x01010101u;
#pragma unroll
  for (int i = 0; i < BITS; ++i) {
#pragma unroll
    for (int s = 0; s < PER_BYTE; ++s) {
      uint32_t m = (w[i] >> (BITS * s)) & MASK;        // byte b holds code PER_BYTE * b + s of the word
      asm volatile("" : "+v"(m));                      // keep the mask: the compiler would go back to bit-field extracts
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const float v = (float)((m >> (8 * b)) & 0xffu);
#pragma unroll
        for (int n = 0; n < NBV; ++n) dot[n] = fmaf(v, x[n][PER_WORD * i + PER_BYTE * b + s], dot[n]);
      }
    }
  }
}

// RB rows per workgroup: 16 for layers with many rows (the input vector is re-read per
// workgroup), 8 where that leaves too few workgroups to fill the chip.  NBV input vectors
// share one pass over the codes.
template <int BITS, bool AFF, int U, int RB, int NBV>
__global__ __launch_bounds__(NT) void matvec_packed_kernel(MvArgs a) {
  constexpr int K = 1 << BITS;
  constexpr int UB = UNIT * BITS / 8;                  // bytes per unit
  __shared__ float sLut[RB][K];
  __shared__ float sPart[RB][NBV][NT / 64];
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
  // this lane's columns of the input vectors, and their sums (affine: the zero-point term)
  float x[U][NBV][UNIT];
  float xsum[U][NBV];
#pragma unroll
  for (int i = 0; i < U; ++i) {
#pragma unroll
    for (int n = 0; n < NBV; ++n) {
      xsum[i][n] = 0.0f;
#pragma unroll
      for (int q4 = 0; q4 < UNIT / 4; ++q4) {
        float4 v = *reinterpret_cast<const float4*>(a.x + (int64_t)n * a.c + (int64_t)uidx[i] * UNIT + 4 * q4);
        if (!uval[i]) v = make_float4(0.f, 0.f, 0.f, 0.f);
        x[i][n][4 * q4 + 0] = v.x; x[i][n][4 * q4 + 1] = v.y; x[i][n][4 * q4 + 2] = v.z; x[i][n][4 * q4 + 3] = v.w;
        xsum[i][n] += (v.x + v.y) + (v.z + v.w);
      }
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
      float acc[NBV];
#pragma unroll
      for (int n = 0; n < NBV; ++n) acc[n] = 0.0f;
#pragma unroll
      for (int i = 0; i < U; ++i) {
        if (AFF) {
          // Section 2.1: (w_int - Z) S, with the unit's group pair: S (sum code x - Z sum x)
          const float S = __half2float(__ushort_as_half((uint16_t)(sz[q][i] & 0xffffu)));
          const float Z = (float)(int16_t)(sz[q][i] >> 16);
          float dot[NBV];
#pragma unroll
          for (int n = 0; n < NBV; ++n) dot[n] = 0.0f;
          if constexpr (BITS == 3) unit_fma<BITS, true, NBV, 0>(w[q][i], x[i], nullptr, dot);
          else unit_dot_bytes<BITS, NBV>(w[q][i], x[i], dot);
#pragma unroll
          for (int n = 0; n < NBV; ++n) acc[n] = fmaf(S, dot[n] - Z * xsum[i][n], acc[n]);
        } else {
          unit_fma<BITS, false, NBV, 0>(w[q][i], x[i], sLut[rb], acc);
        }
      }
#pragma unroll
      for (int n = 0; n < NBV; ++n) {
        const float v = wave_sum_lane63(acc[n]);
        if (lane == 63) sPart[rb][n][wave] = v;
      }
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
  if (tid < RB * NBV) {
    const int rb = tid / NBV, n = tid % NBV;
    if (row0 + rb < a.r) {
      float s = 0.0f;
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) s += sPart[rb][n][w];
      a.y[(int64_t)n * a.r + row0 + rb] = s;
    }
  }
}

template <int BITS, bool AFF, int U, int NBV>
void launch_mv_n(const MvArgs& a, hipStream_t st) {
  dim3 block(NT);
  if (a.r < 16 * 1024)
    hipLaunchKernelGGL((matvec_packed_kernel<BITS, AFF, U, 8, NBV>), dim3((unsigned)lq::ceil_div(a.r, 8)), block, 0, st, a);
  else
    hipLaunchKernelGGL((matvec_packed_kernel<BITS, AFF, U, 16, NBV>), dim3((unsigned)lq::ceil_div(a.r, 16)), block, 0, st, a);
}

// nbv input vectors in one launch: 4, 2 or 1 (a lane holds 32 U nbv values of x in registers,
// which caps U nbv at 4)
template <int BITS, bool AFF>
void launch_mv(const MvArgs& a, int U, int nbv, hipStream_t st) {
  if (U <= 1) {
    if (nbv == 4) launch_mv_n<BITS, AFF, 1, 4>(a, st);
    else if (nbv == 2) launch_mv_n<BITS, AFF, 1, 2>(a, st);
    else launch_mv_n<BITS, AFF, 1, 1>(a, st);
  } else {
    if (nbv == 2) launch_mv_n<BITS, AFF, 2, 2>(a, st);
    else launch_mv_n<BITS, AFF, 2, 1>(a, st);
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
  for (int64_t n = 0; n < nb;) {           // one pass over the codes per 4, 2 or 1 input vectors
    const int64_t left = nb - n;
    const int nbv = (U <= 1 && left >= 4) ? 4 : (left >= 2 ? 2 : 1);
    MvArgs a;
    a.packed = packed; a.packed_ld = packed_ld; a.table = table;
    a.x = X + n * c; a.y = Y + n * r; a.r = r; a.c = (int)c;
    a.group = (int)g; a.ngroups = (int)(c / g);
    if (P->bits == 2) { if (aff) launch_mv<2, true>(a, U, nbv, st); else launch_mv<2, false>(a, U, nbv, st); }
    else if (P->bits == 3) { if (aff) launch_mv<3, true>(a, U, nbv, st); else launch_mv<3, false>(a, U, nbv, st); }
    else { if (aff) launch_mv<4, true>(a, U, nbv, st); else launch_mv<4, false>(a, U, nbv, st); }
    LQ_CHECK_LAUNCH("matvec_packed_kernel");
    n += nbv;
  }
  return LQ_OK;
}
