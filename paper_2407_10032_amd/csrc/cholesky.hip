// lq_cholesky_inv: U = upper Cholesky factor of (H + lambda I)^-1 and its diagonal
// (Algorithm 1 line 4; dampening and Cholesky as described in Section 2.2).
//
// Route: with J the index reversal, factor J H_d J = L L^T (ordinary lower Cholesky),
// so H_d = R R^T with R = J L J upper triangular; then H_d^-1 = R^-T R^-1 and, by
// uniqueness of the Cholesky factor, U = R^-1 = J L^-1 J.  One blocked factorization
// and one blocked triangular inverse (2/3 c^3 flop) instead of invert-then-factor.
// diag(H_d^-1)_i = sum_k U_ki^2 falls out as the column norms of L^-1.
//
// All block operations work on a zero/identity padded copy whose order is a multiple
// of 128, so no tile needs edge handling.  Panel and trailing updates are 128-deep
// fp32 MFMA tile products; the 128 x 128 diagonal blocks are factored and inverted
// by one workgroup in LDS.
#include "lq_common.h"
#include "lq_mfma.h"

namespace {

using lq::TILE;
using lq::WG_THREADS;
constexpr int NB = 128;
constexpr int DLD = 129;  // LDS leading dimension of the diagonal block

// ---------------------------------------------------------------- small kernels
__global__ __launch_bounds__(1024) void diag_mean_kernel(const float* __restrict__ H, int64_t ldh,
                                                         int64_t c, float damp,
                                                         float* __restrict__ scal,
                                                         int32_t* __restrict__ info) {
  __shared__ double red[1024];
  double s = 0.0;
  for (int64_t i = threadIdx.x; i < c; i += 1024) s += (double)H[i * ldh + i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    scal[0] = (float)((double)damp * red[0] / (double)c);
    *info = 0;
  }
}

// A[i][j] = H_d[c-1-i][c-1-j] for i, j < c; identity on the padding.
__global__ __launch_bounds__(256) void flip_damp_kernel(const float* __restrict__ H, int64_t ldh,
                                                        int64_t c, int64_t cp,
                                                        const float* __restrict__ scal,
                                                        float* __restrict__ A) {
  int64_t i = blockIdx.y;
  int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= cp) return;
  float v;
  if (i < c && j < c) {
    v = H[(c - 1 - i) * ldh + (c - 1 - j)];
    if (i == j) v += scal[0];
  } else {
    v = (i == j) ? 1.0f : 0.0f;
  }
  A[i * cp + j] = v;
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ p, int64_t n, float v) {
  int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 3 < n) {
    *reinterpret_cast<float4*>(p + i) = make_float4(v, v, v, v);
  } else {
    for (; i < n; ++i) p[i] = v;
  }
}

// ---------------------------------------------------------------- diagonal block
// 32 x 32 tile product on one wavefront, operands in LDS:
//   acc += sign * A * B,  A[m][k] = pa[m*lda + k],
//   B[k][n] = B_TRANS ? pb[n*ldb + k] : pb[k*ldb + n],  k < 32.
// Leading dimensions of row-read operands are odd (129, 33), so the reads are conflict-free.
template <bool B_TRANS, bool NEGATE>
__device__ __forceinline__ void tile32_mma(lq::floatx16& acc, const float* pa, int lda,
                                           const float* pb, int ldb, int lane) {
  const int ml = lane & 31, kl = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < 16; ++kk) {
    const int k = 2 * kk + kl;
    float a = pa[ml * lda + k];
    float b = B_TRANS ? pb[ml * ldb + k] : pb[k * ldb + ml];
    if (NEGATE) a = -a;
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
  }
}

__device__ __forceinline__ void tile32_store(const lq::floatx16& acc, float* dst, int ld, int lane,
                                             float scale) {
#pragma unroll
  for (int v = 0; v < 16; ++v)
    dst[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * ld + (lane & 31)] = scale * acc[v];
}

__device__ __forceinline__ void tile32_load(lq::floatx16& acc, const float* src, int ld, int lane) {
#pragma unroll
  for (int v = 0; v < 16; ++v)
    acc[v] = src[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * ld + (lane & 31)];
}

__device__ __forceinline__ float lane_bcast(float v, int src_lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

constexpr int XLD = 33;                 // leading dimension of a 32 x 32 block of the inverse
constexpr int XBLK = 32 * XLD;
__device__ __forceinline__ int xblk(int i, int k) { return (i * (i + 1) / 2 + k) * XBLK; }

// One right-looking substitution step on a lane's 32 values, shared by the row solve
// (x L^T = a) and the inverse of a sub-block's factor: the column `step` of the factor
// arrives in `cur` (broadcast float4 pieces), column step + 1 is fetched into `nxt`
// meanwhile.  SOLVE: x[step] *= rd, x[k] -= x[step] L[k][step].  Otherwise (inverse,
// lane = column ri): x[step] = (delta - x[step]) * rd, x[k] += L[k][step] x[step].
// The empty asm pins the updates to this step; otherwise they are sunk to their last use
// and every prefetched column stays live.
template <int STEP, bool SOLVE>
__device__ __forceinline__ void subst_step(float (&x)[32], const float4 (&cur)[8], float4 (&nxt)[8],
                                           const float* lt, const float* rd, float& rdn, int ri) {
  const float rdi = rdn;
  if (STEP + 1 < 32) {
    rdn = rd[STEP + 1];
#pragma unroll
    for (int k4 = (STEP + 2) / 4; k4 < 8; ++k4)
      nxt[k4] = *reinterpret_cast<const float4*>(lt + (STEP + 1) * 32 + 4 * k4);
  }
  __builtin_amdgcn_sched_barrier(0);
  if (SOLVE) x[STEP] *= rdi;
  else x[STEP] = ((ri == STEP) ? 1.0f : -x[STEP]) * rdi;
  const float xs = SOLVE ? -x[STEP] : x[STEP];
#pragma unroll
  for (int k4 = (STEP + 1) / 4; k4 < 8; ++k4) {
    const float4 lv = cur[k4];
    if (4 * k4 + 0 > STEP) x[4 * k4 + 0] = fmaf(xs, lv.x, x[4 * k4 + 0]);
    if (4 * k4 + 1 > STEP) x[4 * k4 + 1] = fmaf(xs, lv.y, x[4 * k4 + 1]);
    if (4 * k4 + 2 > STEP) x[4 * k4 + 2] = fmaf(xs, lv.z, x[4 * k4 + 2]);
    if (4 * k4 + 3 > STEP) x[4 * k4 + 3] = fmaf(xs, lv.w, x[4 * k4 + 3]);
  }
#pragma unroll
  for (int k = STEP + 1; k < 32; ++k) asm volatile("" : "+v"(x[k]));
  __builtin_amdgcn_sched_barrier(0);
}

template <int STEP, bool SOLVE>
__device__ __forceinline__ void subst_steps(float (&x)[32], float4 (&ca)[8], float4 (&cb)[8],
                                            const float* lt, const float* rd, float& rdn, int ri) {
  if constexpr (STEP < 32) {
    subst_step<STEP, SOLVE>(x, ca, cb, lt, rd, rdn, ri);
    subst_step<STEP + 1, SOLVE>(x, cb, ca, lt, rd, rdn, ri);
    subst_steps<STEP + 2, SOLVE>(x, ca, cb, lt, rd, rdn, ri);
  }
}

// x: the lane's 32 values (SOLVE: a row of the sub-panel; otherwise zeros on entry, a
// column of the inverse on exit); lt: the factor column-major, [32][32]; rd: 1 / diagonal.
template <bool SOLVE>
__device__ __forceinline__ void substitute32(float (&x)[32], const float* lt, const float* rd, int ri) {
  float4 ca[8], cb[8];
  float rdn = rd[0];
#pragma unroll
  for (int k4 = 0; k4 < 8; ++k4) {
    ca[k4] = *reinterpret_cast<const float4*>(lt + 4 * k4);
    cb[k4] = ca[k4];
  }
  subst_steps<0, SOLVE>(x, ca, cb, lt, rd, rdn, ri);
}

// Factor the 128 x 128 diagonal block kb and invert its factor, all in LDS, one
// workgroup.  The block is processed as 4 sub-panels of 32 columns: wavefront 0
// factors the 32 x 32 diagonal sub-block in registers (lane = row; entries of other
// lanes come through v_readlane), the rows below it are solved against the sub-block by
// forward substitution (one row per lane, the factor read as broadcast values), and the
// rest of the block is updated with 32 x 32 MFMA tiles.  The inverse of a sub-block's
// factor (lane = column) is not needed by these steps; wavefront 3 computes it while
// wavefront 0 factors the next sub-block.  The inverse of the whole factor is then
// assembled block by block: X_ik = -X_ii * sum_{k<=m<i} L_im X_mk.
// Writes L_kk back (upper part zeroed) and its inverse to Dinv[kb] (128 x 128, ld 128).
__global__ __launch_bounds__(256, 1) void potrf_diag_kernel(float* __restrict__ A, int64_t cp, int kb,
                                                         float* __restrict__ Dinv,
                                                         int32_t* __restrict__ info, int64_t c) {
  extern __shared__ __align__(16) float sm[];
  float* sL = sm;                       // [128][129]
  float* sX = sm + NB * DLD;            // 10 lower blocks of the inverse, [32][33] each
  float* sT = sX + 10 * XBLK;           // 3 temporaries, [32][33] each
  float* sLt = sT + 3 * XBLK;           // [4][32][32] column-major copies of the sub-blocks' factors
  float* sCol = sLt + 4 * 32 * 32;      // [2][32] the two latest columns of the factor
  float* sRd = sCol + 64;               // [4][32] reciprocals of the factors' diagonals
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* tile = A + ((int64_t)kb * NB) * cp + (int64_t)kb * NB;
  {
    // all sixteen 16-byte loads of a thread are in flight before the first LDS store
    float4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int f = tid + u * 256;
      v[u] = *reinterpret_cast<const float4*>(tile + (int64_t)(f >> 5) * cp + 4 * (f & 31));
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int f = tid + u * 256;
      float* d = sL + (f >> 5) * DLD + 4 * (f & 31);
      d[0] = v[u].x; d[1] = v[u].y; d[2] = v[u].z; d[3] = v[u].w;
    }
  }
  __syncthreads();

  // inverse of sub-block q's factor, column ri in each of 32 lanes (right-looking
  // substitution on the unit vector e_ri)
  auto invert_subblock = [&](int q) {
    const int ri = lane & 31;
    float x[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] = 0.0f;
    substitute32<false>(x, sLt + q * 1024, sRd + q * 32, ri);
    if (lane < 32) {
#pragma unroll
      for (int k = 0; k < 32; ++k) sX[xblk(q, q) + k * XLD + ri] = (k >= ri) ? x[k] : 0.0f;
    }
  };

  for (int kk = 0; kk < 4; ++kk) {
    const int c0 = kk * 32;
    if (wave == 0) {
      const int ri = lane & 31;
      float a[32];
#pragma unroll
      for (int k = 0; k < 32; ++k) a[k] = sL[(c0 + ri) * DLD + c0 + k];
      // Right-looking Cholesky of the 32 x 32 sub-block, row ri in this lane.  The update of
      // the very next column takes the one value it needs through v_readlane (short
      // dependency chain from pivot to pivot); all other columns get column j's update one
      // step later from a copy of the column in LDS, read back as wave-uniform float4s,
      // by which time the copy has long arrived.
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        float pj = lane_bcast(a[j], j);
        if (!(pj > 0.0f)) {
          int64_t q = (int64_t)kb * NB + c0 + j;
          if (lane == 0 && q < c && *info == 0) *info = (int32_t)(c - 1 - q) + 1;
          pj = 1.0f;
        }
        float rj = __builtin_amdgcn_rsqf(pj);
        rj = rj * fmaf(-0.5f * pj * rj, rj, 1.5f);      // one Newton step: full fp32 accuracy
        const float dj = pj * rj;
        a[j] = (ri == j) ? dj : a[j] * rj;
        if (lane == 0) sRd[kk * 32 + j] = rj;
        if (j < 31) {
          sCol[(j & 1) * 32 + ri] = a[j];
          a[j + 1] = fmaf(-a[j], lane_bcast(a[j], j + 1), a[j + 1]);
        }
        if (j >= 1 && j < 31) {
          // deferred update from column j - 1 to columns j + 1 .. 31
          const float* cb = sCol + ((j - 1) & 1) * 32;
#pragma unroll
          for (int k4 = (j + 1) / 4; k4 < 8; ++k4) {
            const float4 cv = *reinterpret_cast<const float4*>(cb + 4 * k4);
            if (4 * k4 + 0 > j) a[4 * k4 + 0] = fmaf(-a[j - 1], cv.x, a[4 * k4 + 0]);
            if (4 * k4 + 1 > j) a[4 * k4 + 1] = fmaf(-a[j - 1], cv.y, a[4 * k4 + 1]);
            if (4 * k4 + 2 > j) a[4 * k4 + 2] = fmaf(-a[j - 1], cv.z, a[4 * k4 + 2]);
            if (4 * k4 + 3 > j) a[4 * k4 + 3] = fmaf(-a[j - 1], cv.w, a[4 * k4 + 3]);
          }
        }
      }
      // factor rows to LDS: the block itself and an aligned column-major copy for the solves
      if (lane < 32) {
        float* lt = sLt + kk * 1024;
#pragma unroll
        for (int k = 0; k < 32; ++k) {
          if (k <= ri) sL[(c0 + ri) * DLD + c0 + k] = a[k];
          lt[k * 32 + ri] = (k <= ri) ? a[k] : 0.0f;
        }
      }
    } else if (wave == 3 && kk > 0) {
      // the previous sub-block's inverse is only needed for the assembly at the end: it is
      // computed here, next to the factorization, instead of between factorization and solve
      invert_subblock(kk - 1);
    }
    __syncthreads();
    // sub-panel: rows below the sub-block, one row per lane (wavefronts 0 and 1):
    // x L_kk^T = a by substitution, right-looking: x[j] /= L[j][j], then
    // x[k] -= x[j] L[k][j] for k > j with column j of the factor as broadcast float4s
    {
      const int rrow = c0 + 32 + wave * 64 + lane;
      if (wave < 2 && rrow < NB) {
        float* arow = sL + rrow * DLD + c0;
        float x[32];
#pragma unroll
        for (int k = 0; k < 32; ++k) x[k] = arow[k];
        substitute32<true>(x, sLt + kk * 1024, sRd + kk * 32, 0);
#pragma unroll
        for (int k = 0; k < 32; ++k) arow[k] = x[k];
      }
    }
    __syncthreads();
    // rest of the block: A[ib, jb] -= P_ib P_jb^T for kk < jb <= ib
    {
      const int m = 3 - kk;
      const int ntile = m * (m + 1) / 2;
      for (int t = wave; t < ntile; t += 4) {
        int ii = (t >= 3) ? 2 : (t >= 1) ? 1 : 0;
        int jj = t - ii * (ii + 1) / 2;
        const int ib = kk + 1 + ii, jb = kk + 1 + jj;
        float* ct = sL + (ib * 32) * DLD + jb * 32;
        lq::floatx16 acc;
        tile32_load(acc, ct, DLD, lane);
        tile32_mma<true, true>(acc, sL + (ib * 32) * DLD + c0, DLD, sL + (jb * 32) * DLD + c0, DLD, lane);
        tile32_store(acc, ct, DLD, lane, 1.0f);
      }
    }
    __syncthreads();
  }
  if (wave == 3) invert_subblock(3);
  __syncthreads();

  // inverse of the 128 x 128 factor from the inverted diagonal sub-blocks
  for (int dist = 1; dist < 4; ++dist) {
    const int k = wave, i = wave + dist;
    const bool active = i < 4;
    if (active) {
      lq::floatx16 acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
      for (int m = k; m < i; ++m)
        tile32_mma<false, false>(acc, sL + (i * 32) * DLD + m * 32, DLD, sX + xblk(m, k), XLD, lane);
      tile32_store(acc, sT + wave * XBLK, XLD, lane, 1.0f);
    }
    __syncthreads();
    if (active) {
      lq::floatx16 acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
      tile32_mma<false, false>(acc, sX + xblk(i, i), XLD, sT + wave * XBLK, XLD, lane);
      tile32_store(acc, sX + xblk(i, k), XLD, lane, -1.0f);
    }
    __syncthreads();
  }

  float* dinv = Dinv + (int64_t)kb * NB * NB;
  for (int f = tid; f < NB * NB / 4; f += 256) {
    const int row = f >> 5, col = 4 * (f & 31);
    const int ib = row >> 5, jb = col >> 5;
    float l[4], xv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      l[e] = (col + e <= row) ? sL[row * DLD + col + e] : 0.0f;
      xv[e] = (jb <= ib) ? sX[xblk(ib, jb) + (row & 31) * XLD + ((col + e) & 31)] : 0.0f;
    }
    *reinterpret_cast<float4*>(tile + (int64_t)row * cp + col) = make_float4(l[0], l[1], l[2], l[3]);
    *reinterpret_cast<float4*>(dinv + row * NB + col) = make_float4(xv[0], xv[1], xv[2], xv[3]);
  }
}

// ---------------------------------------------------------------- 128-deep tile products
enum ChMode { CH_PANEL = 0, CH_SYRK = 1, CH_TRI_ROW = 2, CH_TRI_UPD = 3 };

struct ChArgs {
  float* A;      // factor workspace (cp x cp), lower triangle = L
  float* Xb;     // inverse workspace (cp x cp)
  float* Dinv;   // inverted diagonal blocks
  int64_t cp;
  int step;      // kb (PANEL, SYRK) or i (TRI_ROW, TRI_UPD)
};

template <int MODE>
__global__ __launch_bounds__(WG_THREADS, 2) void chol_gemm_kernel(ChArgs a) {
  __shared__ float sA[TILE * lq::RM_LD];
  __shared__ float sB[TILE * lq::RM_LD];
  static_assert(TILE * lq::RM_LD >= lq::RM_KT * TILE, "k-major chunk must fit");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int b = blockIdx.x;
  const int64_t cp = a.cp;

  const float* Aop; int64_t lda;
  const float* Bop; int64_t ldb;
  float* Out; int64_t ldo;
  constexpr bool B_KMAJOR = (MODE == CH_TRI_ROW || MODE == CH_TRI_UPD);
  constexpr bool SUBTRACT = (MODE == CH_SYRK || MODE == CH_TRI_UPD);

  if (MODE == CH_PANEL) {
    int64_t i = a.step + 1 + b;
    Aop = a.A + (i * NB) * cp + (int64_t)a.step * NB; lda = cp;
    Bop = a.Dinv + (int64_t)a.step * NB * NB; ldb = NB;
    Out = a.A + (i * NB) * cp + (int64_t)a.step * NB; ldo = cp;
  } else if (MODE == CH_SYRK) {
    int ii = (int)((sqrtf(8.0f * (float)b + 1.0f) - 1.0f) * 0.5f);
    while (ii * (ii + 1) / 2 > b) --ii;
    while ((ii + 1) * (ii + 2) / 2 <= b) ++ii;
    int jj = b - ii * (ii + 1) / 2;
    int64_t i = a.step + 1 + ii, j = a.step + 1 + jj;
    Aop = a.A + (i * NB) * cp + (int64_t)a.step * NB; lda = cp;
    Bop = a.A + (j * NB) * cp + (int64_t)a.step * NB; ldb = cp;
    Out = a.A + (i * NB) * cp + j * NB; ldo = cp;
  } else if (MODE == CH_TRI_ROW) {
    int64_t i = a.step, k = b;
    Out = a.Xb + (i * NB) * cp + k * NB; ldo = cp;
    if (k == i) {
      const float* src = a.Dinv + i * NB * NB;
      for (int f = tid; f < NB * NB / 4; f += WG_THREADS) {
        int row = f >> 5, c4 = f & 31;
        *reinterpret_cast<float4*>(Out + (int64_t)row * ldo + 4 * c4) =
            *reinterpret_cast<const float4*>(src + row * NB + 4 * c4);
      }
      return;
    }
    Aop = a.Dinv + i * NB * NB; lda = NB;
    Bop = Out; ldb = cp;
  } else {
    int64_t i = a.step;
    int jj = b / (int)(i + 1), k = b - jj * (int)(i + 1);
    int64_t j = i + 1 + jj;
    Aop = a.A + (j * NB) * cp + i * NB; lda = cp;
    Bop = a.Xb + (i * NB) * cp + (int64_t)k * NB; ldb = cp;
    Out = a.Xb + (j * NB) * cp + (int64_t)k * NB; ldo = cp;
  }

  lq::Acc2x2 acc;
  acc.clear();
  for (int k0 = 0; k0 < NB; k0 += lq::RM_KT) {
    lq::fill_rowmajor(sA, Aop + k0, lda, tid);
    if (B_KMAJOR) lq::fill_kmajor32(sB, Bop + (int64_t)k0 * ldb, ldb, tid);
    else lq::fill_rowmajor(sB, Bop + k0, ldb, tid);
    __syncthreads();
    lq::mma_chunk_rowmajor_a<B_KMAJOR>(sA, sB, wm, wn, lane, acc);
    __syncthreads();
  }

  // all loads of the old values are issued before the first store (a load after a store to
  // a possibly aliasing address would wait for it)
  if (SUBTRACT) {
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
      for (int tn = 0; tn < 2; ++tn) {
        float old[16];
#pragma unroll
        for (int v = 0; v < 16; ++v)
          old[v] = Out[(int64_t)lq::acc_row(wm, tm, v, lane) * ldo + lq::acc_col(wn, tn, lane)];
#pragma unroll
        for (int v = 0; v < 16; ++v) acc.t[tm][tn][v] = old[v] - acc.t[tm][tn][v];
      }
  }
#pragma unroll
  for (int tm = 0; tm < 2; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        Out[(int64_t)lq::acc_row(wm, tm, v, lane) * ldo + lq::acc_col(wn, tn, lane)] = acc.t[tm][tn][v];
}

// The same four products cut into smaller output tiles, for steps that have too few
// 128 x 128 tiles to occupy the chip (every step at c <= 8192 or so): one workgroup
// computes a TM x TN piece with all 128 k-values of both operands loaded into LDS at once
// (one barrier, no stage loop), so a step's latency is one short workgroup instead of one
// long one.  In-place modes are only cut along the dimension they do not read across:
// the panel by rows (64 x 128), the inverse's row update by columns (128 x 64); the two
// trailing updates, which write tiles they do not read, into 64 x 64 quarters.
constexpr int SLD = 129;   // LDS leading dimension of a row-major 128-deep operand

template <int ROWS>
__device__ __forceinline__ void fill_rows_k128(float* __restrict__ s, const float* __restrict__ src,
                                               int64_t ld, int tid) {
  // ROWS x 128 values, src[row*ld + k] -> s[row*SLD + k]; coalesced 16-byte global loads
#pragma unroll
  for (int p = 0; p < ROWS / 8; ++p) {
    const int f = tid + p * WG_THREADS;
    const int row = f >> 5, k4 = f & 31;
    const float4 v = *reinterpret_cast<const float4*>(src + (int64_t)row * ld + 4 * k4);
    float* d = s + row * SLD + 4 * k4;
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
  }
}

template <int COLS>
__device__ __forceinline__ void fill_kmajor_k128(float* __restrict__ s, const float* __restrict__ src,
                                                 int64_t ld, int tid) {
  // 128 k-rows x COLS values, src[k*ld + n] -> s[k*COLS + n]
  constexpr int F4_PER_ROW = COLS / 4;
#pragma unroll
  for (int p = 0; p < 128 * F4_PER_ROW / WG_THREADS; ++p) {
    const int f = tid + p * WG_THREADS;
    const int k = f / F4_PER_ROW, c4 = f % F4_PER_ROW;
    *reinterpret_cast<float4*>(s + k * COLS + 4 * c4) =
        *reinterpret_cast<const float4*>(src + (int64_t)k * ld + 4 * c4);
  }
}

template <int MODE>
__global__ __launch_bounds__(WG_THREADS) void chol_small_kernel(ChArgs a) {
  constexpr bool B_KMAJOR = (MODE == CH_TRI_ROW || MODE == CH_TRI_UPD);
  constexpr bool SUBTRACT = (MODE == CH_SYRK || MODE == CH_TRI_UPD);
  constexpr int TM = (MODE == CH_TRI_ROW) ? 128 : 64;
  constexpr int TN = (MODE == CH_PANEL) ? 128 : 64;
  constexpr int NA = TM / 64, NBN = TN / 64;    // 32 x 32 accumulators per wave: NA x NBN
  extern __shared__ __align__(16) float ssm[];
  float* sA = ssm;                               // [TM][SLD]
  float* sB = ssm + TM * SLD;                    // [TN][SLD] or [128][TN]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int ml = lane & 31, kl = lane >> 5;
  const int b = blockIdx.x;
  const int64_t cp = a.cp;

  const float* Aop; int64_t lda;
  const float* Bop; int64_t ldb;
  float* Out; int64_t ldo;
  if (MODE == CH_PANEL) {
    const int64_t i = a.step + 1 + (b >> 1);
    const int sr = b & 1;
    Aop = a.A + (i * NB + sr * 64) * cp + (int64_t)a.step * NB; lda = cp;
    Bop = a.Dinv + (int64_t)a.step * NB * NB; ldb = NB;
    Out = a.A + (i * NB + sr * 64) * cp + (int64_t)a.step * NB; ldo = cp;
  } else if (MODE == CH_SYRK) {
    const int big = b >> 2, sr = (b >> 1) & 1, sc = b & 1;
    int ii = (int)((sqrtf(8.0f * (float)big + 1.0f) - 1.0f) * 0.5f);
    while (ii * (ii + 1) / 2 > big) --ii;
    while ((ii + 1) * (ii + 2) / 2 <= big) ++ii;
    const int jj = big - ii * (ii + 1) / 2;
    const int64_t i = a.step + 1 + ii, j = a.step + 1 + jj;
    Aop = a.A + (i * NB + sr * 64) * cp + (int64_t)a.step * NB; lda = cp;
    Bop = a.A + (j * NB + sc * 64) * cp + (int64_t)a.step * NB; ldb = cp;
    Out = a.A + (i * NB + sr * 64) * cp + j * NB + sc * 64; ldo = cp;
  } else if (MODE == CH_TRI_ROW) {
    const int64_t i = a.step, k = b >> 1;
    const int sc = b & 1;
    Out = a.Xb + (i * NB) * cp + k * NB + sc * 64; ldo = cp;
    if (k == i) {
      const float* src = a.Dinv + i * NB * NB + sc * 64;
      for (int f = tid; f < NB * 16; f += WG_THREADS) {
        const int row = f >> 4, c4 = f & 15;
        *reinterpret_cast<float4*>(Out + (int64_t)row * ldo + 4 * c4) =
            *reinterpret_cast<const float4*>(src + row * NB + 4 * c4);
      }
      return;
    }
    Aop = a.Dinv + i * NB * NB; lda = NB;
    Bop = Out; ldb = cp;
  } else {
    const int64_t i = a.step;
    const int big = b >> 2, sr = (b >> 1) & 1, sc = b & 1;
    const int jj = big / (int)(i + 1), k = big - jj * (int)(i + 1);
    const int64_t j = i + 1 + jj;
    Aop = a.A + (j * NB + sr * 64) * cp + i * NB; lda = cp;
    Bop = a.Xb + (i * NB) * cp + (int64_t)k * NB + sc * 64; ldb = cp;
    Out = a.Xb + (j * NB + sr * 64) * cp + (int64_t)k * NB + sc * 64; ldo = cp;
  }

  fill_rows_k128<TM>(sA, Aop, lda, tid);
  if (B_KMAJOR) fill_kmajor_k128<TN>(sB, Bop, ldb, tid);
  else fill_rows_k128<TN>(sB, Bop, ldb, tid);
  __syncthreads();

  lq::floatx16 acc[NA][NBN];
#pragma unroll
  for (int x = 0; x < NA; ++x)
#pragma unroll
    for (int y = 0; y < NBN; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.0f;

  const float* pa = sA + (wm * (TM / 2) + ml) * SLD + kl;
  const float* pb = B_KMAJOR ? sB + kl * TN + wn * (TN / 2) + ml : sB + (wn * (TN / 2) + ml) * SLD + kl;
#pragma unroll 8
  for (int k = 0; k < 128; k += 2) {
    float av[NA], bv[NBN];
#pragma unroll
    for (int x = 0; x < NA; ++x) av[x] = pa[x * 32 * SLD + k];
#pragma unroll
    for (int y = 0; y < NBN; ++y) bv[y] = B_KMAJOR ? pb[k * TN + y * 32] : pb[y * 32 * SLD + k];
#pragma unroll
    for (int x = 0; x < NA; ++x)
#pragma unroll
      for (int y = 0; y < NBN; ++y)
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[x], bv[y], acc[x][y], 0, 0, 0);
  }

  // old values first, all loads in flight together, then the stores
  if (SUBTRACT) {
#pragma unroll
    for (int x = 0; x < NA; ++x)
#pragma unroll
      for (int y = 0; y < NBN; ++y) {
        float old[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = wm * (TM / 2) + x * 32 + 8 * (v >> 2) + 4 * kl + (v & 3);
          const int col = wn * (TN / 2) + y * 32 + ml;
          old[v] = Out[(int64_t)row * ldo + col];
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[x][y][v] = old[v] - acc[x][y][v];
      }
  }
#pragma unroll
  for (int x = 0; x < NA; ++x)
#pragma unroll
    for (int y = 0; y < NBN; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = wm * (TM / 2) + x * 32 + 8 * (v >> 2) + 4 * kl + (v & 3);
        const int col = wn * (TN / 2) + y * 32 + ml;
        Out[(int64_t)row * ldo + col] = acc[x][y][v];
      }
}

template <int MODE>
constexpr size_t chol_small_lds() {
  constexpr int TM = (MODE == CH_TRI_ROW) ? 128 : 64;
  constexpr int TN = (MODE == CH_PANEL) ? 128 : 64;
  constexpr bool BK = (MODE == CH_TRI_ROW || MODE == CH_TRI_UPD);
  return (size_t)(TM * SLD + (BK ? 128 * TN : TN * SLD)) * sizeof(float);
}

// d[c-1-q] = sum_{p=q}^{c-1} Xb[p][q]^2 : column norms of L^-1 = diag(H_d^-1) reversed.
// Two kernels: sums over slices of 128 rows (thread = column, so a row of the slice is one
// coalesced read; slices entirely above the diagonal are skipped), then the slices of a
// column are added in order.  part: [cp / 128][cp].
__global__ __launch_bounds__(256) void colnorm_part_kernel(const float* __restrict__ Xb, int64_t cp,
                                                           float* __restrict__ part) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t p0 = (int64_t)blockIdx.y * NB;
  if (q >= cp) return;
  if (p0 + NB <= (int64_t)blockIdx.x * 256) return;     // every row of the slice is above every column
  float s = 0.0f;
#pragma unroll 8
  for (int64_t p = p0; p < p0 + NB; ++p) {
    const float x = (p >= q) ? Xb[p * cp + q] : 0.0f;
    s = fmaf(x, x, s);
  }
  part[(int64_t)blockIdx.y * cp + q] = s;
}

__global__ __launch_bounds__(256) void colnorm_sum_kernel(const float* __restrict__ part, int64_t cp,
                                                          int64_t c, float* __restrict__ d) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= c) return;
  float t = 0.0f;
  for (int64_t sl = q / NB; sl < cp / NB; ++sl) t += part[sl * cp + q];
  d[c - 1 - q] = t;
}

// U[a][b] = Xb[c-1-a][c-1-b] for b >= a, else 0.
__global__ __launch_bounds__(256) void flip_out_kernel(const float* __restrict__ Xb, int64_t cp,
                                                       int64_t c, float* __restrict__ U, int64_t ldu) {
  int64_t a = blockIdx.y;
  int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (b >= c) return;
  U[a * ldu + b] = (b >= a) ? Xb[(c - 1 - a) * cp + (c - 1 - b)] : 0.0f;
}

struct CholPlan {
  int64_t cp;
  int nb;
  size_t off_A, off_X, off_D, off_S, total;
};

CholPlan make_plan(int64_t c) {
  CholPlan p;
  p.nb = (int)lq::ceil_div(c, NB);
  p.cp = (int64_t)p.nb * NB;
  size_t mat = (size_t)p.cp * p.cp * sizeof(float);
  p.off_A = 0;
  p.off_X = lq::align_up(mat, 256);
  p.off_D = p.off_X + lq::align_up(mat, 256);
  p.off_S = p.off_D + (size_t)p.nb * NB * NB * sizeof(float);
  p.total = p.off_S + 256;
  return p;
}

}  // namespace

namespace lq {
size_t cholesky_workspace_bytes(int64_t c) { return make_plan(c).total; }
}  // namespace lq

extern "C" lq_status lq_cholesky_inv(const float* H, int64_t ldh, int64_t c, float damp, float* U,
                                     int64_t ldu, float* hinv_diag, int32_t* info, void* ws,
                                     size_t ws_bytes, void* stream) {
  if (!H || !U || !hinv_diag || !info) return lq::fail(LQ_ERR_INVALID_ARG, "lq_cholesky_inv: null pointer");
  if (c < 1 || ldh < c || ldu < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_cholesky_inv: c=%lld ldh=%lld ldu=%lld", (long long)c, (long long)ldh, (long long)ldu);
  if (!(damp >= 0.0f)) return lq::fail(LQ_ERR_INVALID_ARG, "lq_cholesky_inv: damp must be >= 0");
  if (c > 65535) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_cholesky_inv: c > 65535");
  CholPlan plan = make_plan(c);
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < plan.total)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_cholesky_inv: workspace needs %zu bytes, 256-byte aligned", plan.total);

  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)ws;
  float* A = (float*)(base + plan.off_A);
  float* Xb = (float*)(base + plan.off_X);
  float* Dinv = (float*)(base + plan.off_D);
  float* scal = (float*)(base + plan.off_S);
  const int64_t cp = plan.cp;
  const int nb = plan.nb;

  const size_t potrf_lds = (NB * DLD + 13 * 32 * 33 + 4 * 32 * 32 + 64 + 128) * sizeof(float);
  static lq::DeviceOnce attr_once;
  if (lq::DeviceOnceGuard once(attr_once); once.first()) {
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)potrf_diag_kernel,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)potrf_lds));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)chol_small_kernel<CH_PANEL>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)chol_small_lds<CH_PANEL>()));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)chol_small_kernel<CH_SYRK>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)chol_small_lds<CH_SYRK>()));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)chol_small_kernel<CH_TRI_ROW>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)chol_small_lds<CH_TRI_ROW>()));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)chol_small_kernel<CH_TRI_UPD>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)chol_small_lds<CH_TRI_UPD>()));
    once.done();
  }

  hipLaunchKernelGGL(diag_mean_kernel, dim3(1), dim3(1024), 0, st, H, ldh, c, damp, scal, info);
  LQ_CHECK_LAUNCH("diag_mean_kernel");
  dim3 g2((unsigned)lq::ceil_div(cp, 256), (unsigned)cp);
  hipLaunchKernelGGL(flip_damp_kernel, g2, dim3(256), 0, st, H, ldh, c, cp, (const float*)scal, A);
  LQ_CHECK_LAUNCH("flip_damp_kernel");

  // The inverse workspace starts from zero; cleared before the factorization so that the
  // inverse chain can start as soon as the first panel exists.
  int64_t n = cp * cp;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)lq::ceil_div(n, 1024)), dim3(256), 0, st, Xb, n, 0.0f);
  LQ_CHECK_LAUNCH("fill_kernel");

  // Two chains: the factorization (diagonal block, panel, trailing update per step) on
  // the caller's stream, and the triangular inverse on a side stream.  Step i of the
  // inverse needs only the panels up to i, so it follows the factorization one step behind
  // instead of waiting for all of it.
  lq::SideStream* side = lq::side_stream(0);
  hipStream_t sinv = side ? side->stream : st;

  ChArgs a;
  a.A = A; a.Xb = Xb; a.Dinv = Dinv; a.cp = cp;
  // A launch with few 128 x 128 tiles is cut into smaller pieces (see chol_small_kernel).
  constexpr int SMALL_LIMIT = 768;
  constexpr int PANEL_STREAM_NB = 48;
  auto launch = [&](int mode, int big_tiles, hipStream_t sx, const ChArgs& arg) -> lq_status {
    // The single-shot panel kernel holds 100 KB of LDS: next to the inverse chain's large
    // launches on the side stream (many blocks) it would wait for a compute unit with that
    // much free, on the critical path; the streaming kernel (36 KB) fits beside them.
    const bool small = big_tiles <= SMALL_LIMIT && !(mode == CH_PANEL && nb > PANEL_STREAM_NB);
    switch (mode) {
      case CH_PANEL:
        if (small) hipLaunchKernelGGL(chol_small_kernel<CH_PANEL>, dim3(2 * big_tiles), dim3(WG_THREADS), chol_small_lds<CH_PANEL>(), sx, arg);
        else hipLaunchKernelGGL(chol_gemm_kernel<CH_PANEL>, dim3(big_tiles), dim3(WG_THREADS), 0, sx, arg);
        break;
      case CH_SYRK:
        if (small) hipLaunchKernelGGL(chol_small_kernel<CH_SYRK>, dim3(4 * big_tiles), dim3(WG_THREADS), chol_small_lds<CH_SYRK>(), sx, arg);
        else hipLaunchKernelGGL(chol_gemm_kernel<CH_SYRK>, dim3(big_tiles), dim3(WG_THREADS), 0, sx, arg);
        break;
      case CH_TRI_ROW:
        if (small) hipLaunchKernelGGL(chol_small_kernel<CH_TRI_ROW>, dim3(2 * big_tiles), dim3(WG_THREADS), chol_small_lds<CH_TRI_ROW>(), sx, arg);
        else hipLaunchKernelGGL(chol_gemm_kernel<CH_TRI_ROW>, dim3(big_tiles), dim3(WG_THREADS), 0, sx, arg);
        break;
      default:
        if (small) hipLaunchKernelGGL(chol_small_kernel<CH_TRI_UPD>, dim3(4 * big_tiles), dim3(WG_THREADS), chol_small_lds<CH_TRI_UPD>(), sx, arg);
        else hipLaunchKernelGGL(chol_gemm_kernel<CH_TRI_UPD>, dim3(big_tiles), dim3(WG_THREADS), 0, sx, arg);
        break;
    }
    LQ_CHECK_LAUNCH("cholesky tile product");
    return LQ_OK;
  };
  auto inverse_step = [&](int i) -> lq_status {
    ChArgs b = a;
    b.step = i;
    lq_status s1 = launch(CH_TRI_ROW, i + 1, sinv, b);
    if (s1 != LQ_OK) return s1;
    if (i + 1 < nb) return launch(CH_TRI_UPD, (nb - i - 1) * (i + 1), sinv, b);
    return LQ_OK;
  };
  // (a lambda, so that a failing launch in the middle still joins the side stream below)
  auto factor_chain = [&]() -> lq_status {
  for (int kb = 0; kb < nb; ++kb) {
    hipLaunchKernelGGL(potrf_diag_kernel, dim3(1), dim3(256), potrf_lds, st, A, cp, kb, Dinv, info, c);
    LQ_CHECK_LAUNCH("potrf_diag_kernel");
    int m = nb - kb - 1;
    if (m > 0) {
      a.step = kb;
      lq_status sp = launch(CH_PANEL, m, st, a);
      if (sp != LQ_OK) return sp;
    }
    if (side) {
      hipEvent_t ev = side->fork[kb & 3];
      LQ_CHECK_HIP(hipEventRecord(ev, st));
      LQ_CHECK_HIP(hipStreamWaitEvent(side->stream, ev, 0));
      lq_status si = inverse_step(kb);
      if (si != LQ_OK) return si;
    }
    if (m > 0) {
      a.step = kb;
      lq_status ss = launch(CH_SYRK, m * (m + 1) / 2, st, a);
      if (ss != LQ_OK) return ss;
    }
  }
  return LQ_OK;
  };
  const lq_status chain_rc = factor_chain();
  if (side) {
    // joined also after an error: whatever reached the side stream stays ordered before the
    // caller's later work on `stream`
    const hipError_t e1 = hipEventRecord(side->join, side->stream);
    const hipError_t e2 = hipStreamWaitEvent(st, side->join, 0);
    if (chain_rc != LQ_OK) return chain_rc;
    LQ_CHECK_HIP(e1);
    LQ_CHECK_HIP(e2);
  } else {
    if (chain_rc != LQ_OK) return chain_rc;
    for (int i = 0; i < nb; ++i) {
      lq_status si = inverse_step(i);
      if (si != LQ_OK) return si;
    }
  }

  // the factor workspace A is free once the inverse is complete: it holds the partial sums
  hipLaunchKernelGGL(colnorm_part_kernel, dim3((unsigned)lq::ceil_div(cp, 256), (unsigned)nb), dim3(256), 0, st,
                     (const float*)Xb, cp, A);
  LQ_CHECK_LAUNCH("colnorm_part_kernel");
  hipLaunchKernelGGL(colnorm_sum_kernel, dim3((unsigned)lq::ceil_div(c, 256)), dim3(256), 0, st,
                     (const float*)A, cp, c, hinv_diag);
  LQ_CHECK_LAUNCH("colnorm_sum_kernel");
  dim3 g3((unsigned)lq::ceil_div(c, 256), (unsigned)c);
  hipLaunchKernelGGL(flip_out_kernel, g3, dim3(256), 0, st, (const float*)Xb, cp, c, U, ldu);
  LQ_CHECK_LAUNCH("flip_out_kernel");
  return LQ_OK;
}
