// Column kernel of lq_quantize_layer (Algorithm 1 lines 11-18) for one block of B columns.
//
// A wavefront owns 64 rows of W; its 64 x B piece of the block lives in LDS for the
// whole kernel.  The block is processed in sub-blocks of 32 columns:
//   * the sub-block's columns are pulled into registers with one lane per row, and the
//     32 columns are handled in order: quantize against the row's grid (line 13 / 15),
//     E = (w - q) / U_jj (line 16), subtract E * U[j, j+1:] inside the sub-block
//     (line 17) with U read from LDS at wave-uniform addresses, row j + 1 one column ahead;
//   * the rest of line 17, the update of the block's later columns by the sub-block's 32
//     error columns, is a 64 x 32 by 32 x (up to 96) product done on fp32 MFMA straight
//     on the LDS-resident piece (the A operand is built from the per-lane errors with a
//     cross-half lane exchange, the B operand comes from the packed U block).
// The code of one sub-block is a few thousand instructions and is reused by a run-time
// loop, so the kernel stays inside the instruction cache.  E is written transposed
// ([B x r]) for the trailing update across blocks.  The B x B diagonal blocks of U are
// packed, zero-padded, by a small kernel once per layer.
#pragma once

#include "lq_common.h"
#include "lq_mfma.h"

namespace lq {

constexpr int QT = 256;   // threads per workgroup = rows per workgroup (4 wavefronts x 64 rows)
constexpr int SB = 32;    // sub-block width

struct ColArgs {
  float* W; int64_t ldw;
  int64_t r, c;
  int64_t i0;           // first column of the block
  int nb;               // columns in this block (<= B)
  const float* grid;    // nu: [r x K]; aff: [r x ngroups x 2]
  int group; int ngroups;
  uint8_t* codes;
  float* Et; int64_t rpad;
  float* row_loss;      // may be null
  int first;            // 1 for the first block (row_loss starts from zero)
  int vecw;             // W rows are 16-byte aligned (ldw % 4 == 0)
  int vecc;             // rows of codes are 4-byte aligned (base pointer and c)
};

// Nearest point of an ascending grid; ties go to the lower point.  code = number of
// midpoints below w, found by bisection: each level compares with the middle candidate
// and keeps the half of the midpoints and grid points that is still possible.  The
// candidates travel as vector values (halved by .lo / .hi), which keeps them in registers
// and needs one comparison mask per level.
typedef float f2v __attribute__((ext_vector_type(2)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef float f8v __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

template <int K> struct GridVec;
template <> struct GridVec<4> { typedef f4v type; };
template <> struct GridVec<8> { typedef f8v type; };
template <> struct GridVec<16> { typedef f16v type; };

// g: the K grid points; m: the K - 1 midpoints in elements 0..K-2 (element K-1 unused).
// The code is built most significant bit first as code = 2 * code + bit in a vector
// register at each level; the empty asm at the end keeps the compiler from holding the
// comparison masks of a whole sub-block in scalar registers (and spilling them) until the
// codes are stored.
__device__ __forceinline__ void quant_nu_bits(float w, f2v g, f2v m, float& q, int& code) {
  const bool up = w > m.x;
  q = up ? g.y : g.x;
  code = 2 * code + (up ? 1 : 0);
}
__device__ __forceinline__ void quant_nu_bits(float w, f4v g, f4v m, float& q, int& code) {
  const bool up = w > m.y;
  code = 2 * code + (up ? 1 : 0);
  quant_nu_bits(w, up ? g.hi : g.lo, up ? m.hi : m.lo, q, code);
}
__device__ __forceinline__ void quant_nu_bits(float w, f8v g, f8v m, float& q, int& code) {
  const bool up = w > m.s3;
  code = 2 * code + (up ? 1 : 0);
  quant_nu_bits(w, up ? g.hi : g.lo, up ? m.hi : m.lo, q, code);
}
__device__ __forceinline__ void quant_nu_bits(float w, f16v g, f16v m, float& q, int& code) {
  const bool up = w > m.s7;
  code = 2 * code + (up ? 1 : 0);
  quant_nu_bits(w, up ? g.hi : g.lo, up ? m.hi : m.lo, q, code);
}
template <typename V>
__device__ __forceinline__ void quant_nu_vec(float w, V g, V m, float& q, int& code) {
  int c = 0;
  quant_nu_bits(w, g, m, q, c);
  asm volatile("" : "+v"(c));
  code = c;
}

template <int B, int BITS, bool AFF>
__global__ __launch_bounds__(QT) void column_block_kernel(ColArgs a, const float* __restrict__ ud,
                                                          const float* __restrict__ urinv) {
  // ud: this block's B x B piece of U (entries left of the diagonal and outside the
  // matrix are zero), urinv: 1 / U_jj (zero outside the matrix).
  constexpr int K = 1 << BITS;
  constexpr int NSB = B / SB;
  constexpr int LD = B + 1;                  // odd: row-per-lane and tile accesses are conflict-free
  extern __shared__ __align__(16) float smq[];
  float* sUd = smq;                          // [NSB][32][32] diagonal sub-blocks of the U block
  float* sRinv = sUd + NSB * SB * SB;        // [B]
  float* sWall = sRinv + B;                  // [4 wavefronts][64][LD]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ml = lane & 31, hl = lane >> 5;
  float* sW = sWall + wave * 64 * LD;
  const int64_t row0 = (int64_t)blockIdx.x * QT + wave * 64;   // first row of this wavefront
  const int64_t row = row0 + lane;
  const bool valid = row < a.r;
  const int nb = a.nb;

  for (int f = tid; f < NSB * SB * SB; f += QT) {
    int s = f / (SB * SB), j = (f / SB) % SB, jj = f % SB;
    sUd[f] = ud[(s * SB + j) * B + s * SB + jj];
  }
  for (int j = tid; j < B; j += QT) sRinv[j] = urinv[j];

  // the row's grid first (its loads overlap the block load below)
  typename GridVec<K>::type g, mid;
  float S = 1.0f, Z = 0.0f, invS = 1.0f;
  if (!AFF) {
    // rows past r read row 0's grid (their results are never stored)
    const float* grow = a.grid + (valid ? row : 0) * K;
    if constexpr (K >= 4) {
#pragma unroll
      for (int m4 = 0; m4 < K / 4; ++m4) {
        const float4 v = reinterpret_cast<const float4*>(grow)[m4];
        g[4 * m4 + 0] = v.x; g[4 * m4 + 1] = v.y; g[4 * m4 + 2] = v.z; g[4 * m4 + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int m = 0; m < K; ++m) g[m] = grow[m];
    }
  } else {
#pragma unroll
    for (int m = 0; m < K; ++m) g[m] = 0.0f;
  }

  // this wavefront's 64 x B piece of W -> LDS (rows past r and columns past c read as zero);
  // eight 16-byte loads are in flight before their values are written to LDS
  if (a.vecw && nb == B) {
    constexpr int PER_LANE = 64 * (B / 4) / 64;
    static_assert(PER_LANE % 8 == 0, "block load is unrolled by eight");
    for (int it = 0; it < PER_LANE; it += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int f = lane + (it + u) * 64;
        const int rr = f / (B / 4), c4 = f % (B / 4);
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row0 + rr < a.r) v[u] = *reinterpret_cast<const float4*>(a.W + (row0 + rr) * a.ldw + a.i0 + 4 * c4);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int f = lane + (it + u) * 64;
        const int rr = f / (B / 4), c4 = f % (B / 4);
        float* d = sW + rr * LD + 4 * c4;
        d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
      }
    }
  } else {
    for (int f = lane; f < 64 * B; f += 64) {
      int rr = f / B, cc = f % B;
      sW[rr * LD + cc] = (row0 + rr < a.r && cc < nb) ? a.W[(row0 + rr) * a.ldw + a.i0 + cc] : 0.0f;
    }
  }

#pragma unroll
  for (int m = 0; m < K; ++m) mid[m] = (m < K - 1) ? 0.5f * (g[m] + g[m < K - 1 ? m + 1 : m]) : 0.0f;
  __syncthreads();

  float loss = 0.0f;
  const float qmax = (float)(K - 1);

  for (int sb = 0; sb < NSB; ++sb) {
    const int cb = sb * SB;                       // first column of the sub-block within the block
    float ws[SB], e[SB];
#pragma unroll
    for (int k = 0; k < SB; ++k) ws[k] = sW[lane * LD + cb + k];
    const float* su = sUd + sb * SB * SB;
    uint32_t pk[SB / 4];
#pragma unroll
    for (int q4 = 0; q4 < SB / 4; ++q4) pk[q4] = 0u;
    // B operand of the first tile updated after this sub-block: loaded now, used after the
    // column phase (rows cb.. of the packed U block, columns of the next sub-block)
    float bpre[SB / 2];
#pragma unroll
    for (int kk = 0; kk < SB / 2; ++kk)
      bpre[kk] = (sb + 1 < NSB) ? ud[(cb + 2 * kk + hl) * B + (sb + 1) * SB + ml] : 0.0f;

    // Row j of the sub-block's U (the same values for every lane) is fetched from LDS one
    // column ahead: with one wavefront per SIMD nothing else hides the LDS round trip, so the
    // reads of row j + 1 are issued before column j is quantized and are waited for only
    // when column j + 1 needs them.
    float ucur[SB], unxt[SB];
    float rcur = sRinv[cb], rnxt = 0.0f;
#pragma unroll
    for (int jj = 1; jj < SB; ++jj) ucur[jj] = su[jj];

    // Columns past the end of a ragged last block hold zeros and have 1 / U_jj = 0, so
    // they produce E = 0 and change nothing; only the stores are guarded.
#pragma unroll
    for (int j = 0; j < SB; ++j) {
      if (j + 1 < SB) {
        rnxt = sRinv[cb + j + 1];
#pragma unroll
        for (int jj = j + 2; jj < SB; ++jj) unxt[jj] = su[(j + 1) * SB + jj];
        __builtin_amdgcn_sched_barrier(0);       // the reads stay here, ahead of the column's work
      }
      float q;
      int code;
      const float wj = ws[j];
      if (AFF) {
        const int64_t col = a.i0 + cb + j;
        if (j == 0 || (col % a.group) == 0) {
          const int64_t gi = (col < a.c ? col : a.c - 1) / a.group;
          const float* sz = a.grid + ((valid ? row : 0) * a.ngroups + gi) * 2;
          S = sz[0];
          Z = sz[1];
          invS = 1.0f / S;
        }
        // Section 2.1: w_int = clip(round(w / S) + Z, 0, 2^b - 1); quant = (w_int - Z) S
        float wi = fminf(fmaxf(rintf(wj * invS) + Z, 0.0f), qmax);
        code = (int)wi;
        q = (wi - Z) * S;
      } else {
        quant_nu_vec(wj, g, mid, q, code);
      }
      const float ej = (wj - q) * rcur;
      e[j] = ej;
      ws[j] = q;
      pk[j >> 2] |= (uint32_t)code << (8 * (j & 3));
      loss = fmaf(0.5f * ej, ej, loss);
      a.Et[(int64_t)(cb + j) * a.rpad + row] = ej;      // rpad covers every lane of the launch
#pragma unroll
      for (int jj = j + 1; jj < SB; ++jj) ws[jj] = fmaf(-ej, ucur[jj], ws[jj]);
      rcur = rnxt;
#pragma unroll
      for (int jj = j + 2; jj < SB; ++jj) ucur[jj] = unxt[jj];
    }

    // quantized values back to the LDS piece, codes to global memory
#pragma unroll
    for (int k = 0; k < SB; ++k) sW[lane * LD + cb + k] = ws[k];
    if (valid) {
      uint8_t* cout = a.codes + row * a.c + a.i0 + cb;
      if (cb + SB <= nb && a.vecc && (a.i0 % 4) == 0) {
#pragma unroll
        for (int q4 = 0; q4 < SB / 4; ++q4) reinterpret_cast<uint32_t*>(cout)[q4] = pk[q4];
      } else {
#pragma unroll
        for (int j = 0; j < SB; ++j)
          if (cb + j < nb) cout[j] = (uint8_t)((pk[j >> 2] >> (8 * (j & 3))) & 0xffu);
      }
    }

    if (sb + 1 < NSB) {
      // A operands of the 64 x 32 error block for the two 32-row halves: lanes 0..31 supply
      // k even, lanes 32..63 k odd, of rows (lane % 32) and (lane % 32) + 32.
      float a_lo[SB / 2], a_hi[SB / 2];
#pragma unroll
      for (int kk = 0; kk < SB / 2; ++kk) {
        const float x = -e[2 * kk], y = -e[2 * kk + 1];
        const float xs = __shfl_xor(x, 32, 64), ys = __shfl_xor(y, 32, 64);
        a_lo[kk] = hl ? ys : x;     // rows 0..31:  lane < 32 -> own x;  lane >= 32 -> y of lane - 32
        a_hi[kk] = hl ? y : xs;     // rows 32..63: lane < 32 -> x of lane + 32;  lane >= 32 -> own y
      }
      for (int t = sb + 1; t < NSB; ++t) {
        float b[SB / 2];
        if (t == sb + 1) {
#pragma unroll
          for (int kk = 0; kk < SB / 2; ++kk) b[kk] = bpre[kk];
        } else {
#pragma unroll
          for (int kk = 0; kk < SB / 2; ++kk) b[kk] = ud[(cb + 2 * kk + hl) * B + t * SB + ml];
        }
        floatx16 c_lo, c_hi;
        float* tl = sW + t * SB + ml;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = 8 * (v >> 2) + 4 * hl + (v & 3);
          c_lo[v] = tl[m * LD];
          c_hi[v] = tl[(m + 32) * LD];
        }
#pragma unroll
        for (int kk = 0; kk < SB / 2; ++kk) {
          c_lo = __builtin_amdgcn_mfma_f32_32x32x2f32(a_lo[kk], b[kk], c_lo, 0, 0, 0);
          c_hi = __builtin_amdgcn_mfma_f32_32x32x2f32(a_hi[kk], b[kk], c_hi, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = 8 * (v >> 2) + 4 * hl + (v & 3);
          tl[m * LD] = c_lo[v];
          tl[(m + 32) * LD] = c_hi[v];
        }
      }
    }
  }

  // W_hat of the block back to global memory, row by row (coalesced)
  if (a.vecw && nb == B) {
#pragma unroll 8
    for (int f = lane; f < 64 * (B / 4); f += 64) {
      int rr = f / (B / 4), c4 = f % (B / 4);
      if (row0 + rr < a.r) {
        const float* d = sW + rr * LD + 4 * c4;
        *reinterpret_cast<float4*>(a.W + (row0 + rr) * a.ldw + a.i0 + 4 * c4) = make_float4(d[0], d[1], d[2], d[3]);
      }
    }
  } else {
    for (int f = lane; f < 64 * B; f += 64) {
      int rr = f / B, cc = f % B;
      if (row0 + rr < a.r && cc < nb) a.W[(row0 + rr) * a.ldw + a.i0 + cc] = sW[rr * LD + cc];
    }
  }
  if (valid && a.row_loss) a.row_loss[row] = (a.first ? 0.0f : a.row_loss[row]) + loss;
}

template <int B>
constexpr size_t column_lds_bytes() {
  return (size_t)((B / SB) * SB * SB + B + 4 * 64 * (B + 1)) * sizeof(float);
}

template <int B>
lq_status launch_column(const ColArgs& a, const float* ud, const float* urinv, const lq_params* P,
                        hipStream_t st) {
  const size_t lds = column_lds_bytes<B>();
  dim3 grid((unsigned)lq::ceil_div(a.r, QT)), block(QT);
#define LQ_COL(BITS, AFF)                                                                          \
  do {                                                                                             \
    static lq::DeviceOnce attr_once;                                                               \
    if (lq::DeviceOnceGuard once(attr_once); once.first()) {                                       \
      LQ_CHECK_HIP(hipFuncSetAttribute((const void*)column_block_kernel<B, BITS, AFF>,             \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));     \
      once.done();                                                                                 \
    }                                                                                              \
    hipLaunchKernelGGL((column_block_kernel<B, BITS, AFF>), grid, block, lds, st, a, ud, urinv);   \
  } while (0)
  const bool aff = P->mode == LQ_GRID_AFFINE;
  if (P->bits == 2) { if (aff) LQ_COL(2, true); else LQ_COL(2, false); }
  else if (P->bits == 3) { if (aff) LQ_COL(3, true); else LQ_COL(3, false); }
  else { if (aff) LQ_COL(4, true); else LQ_COL(4, false); }
#undef LQ_COL
  LQ_CHECK_LAUNCH("column_block_kernel");
  return LQ_OK;
}

lq_status launch_column_128(const ColArgs& a, const float* ud, const float* urinv,
                            const lq_params* P, hipStream_t st);
lq_status launch_column_64(const ColArgs& a, const float* ud, const float* urinv,
                            const lq_params* P, hipStream_t st);
lq_status launch_column_32(const ColArgs& a, const float* ud, const float* urinv,
                            const lq_params* P, hipStream_t st);

}  // namespace lq
