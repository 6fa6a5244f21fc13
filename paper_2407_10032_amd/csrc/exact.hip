// lq_quantize_exact: LeanQuant-Exact, Algorithm 2 of the appendix ("for million-parameter
// networks").  Per row: in each of c steps the not yet quantized weight with the smallest
// loss error (quant(w_i) - w_i)^2 / (2 Hinv_ii) (Eq. 3) is quantized, the other weights
// move by -Hinv[:, i] / Hinv_ii (w_i - w_hat_i), and row and column i leave the inverse
// Hessian (Eq. 9).  O(c^3) per row, so every row needs its own copy of the inverse.
//
// One workgroup per row, all arithmetic in fp64 (the greedy order is decided by comparing
// loss errors, so the decision is taken in the precision of the inverse handed in).  The
// row's c x c copy lives in the workspace and is streamed once per step (rows of weights
// already quantized are skipped); the weights, the running diagonal and the current row of
// the inverse sit in LDS.  Memory bound: c^3 / 2 x 16 bytes per row.
#include "lq_common.h"

namespace {

constexpr int NT = 256;
constexpr int MAX_C = 2048;
constexpr int MAX_SLOTS = 512;

struct ExactArgs {
  float* W; int64_t ldw;
  int64_t r; int c;
  const double* Hinv; int64_t ldh;
  const float* grid;
  uint8_t* codes;
  int32_t* order;
  float* row_loss;
  double* slots;        // [gridDim.x][c][c]
  int bits; int aff;
};

// Nearest point of the ascending grid, ties to the lower point (non-uniform), or Section
// 2.1's clip(round(w / S) + Z, 0, 2^b - 1) (affine).
__device__ __forceinline__ void quant1(double w, const double* g, int K, int aff, double S, double Z,
                                       double qmax, double& q, int& code) {
  if (aff) {
    const double wi = fmin(fmax(rint(w / S) + Z, 0.0), qmax);
    q = (wi - Z) * S;
    code = (int)wi;
  } else {
    double best = fabs(w - g[0]);
    int bi = 0;
    for (int m = 1; m < K; ++m) {
      const double dm = fabs(w - g[m]);
      if (dm < best) { best = dm; bi = m; }
    }
    q = g[bi];
    code = bi;
  }
}

__global__ __launch_bounds__(NT) void exact_rows_kernel(ExactArgs a) {
  extern __shared__ __align__(16) unsigned char smraw[];
  const int c = a.c;
  double* sw = reinterpret_cast<double*>(smraw);     // [c] working weights
  double* shd = sw + c;                              // [c] running diagonal of the inverse
  double* srow = shd + c;                            // [c] row i of the inverse at this step
  uint8_t* sdone = reinterpret_cast<uint8_t*>(srow + c);   // [c]
  __shared__ double sG[16];
  __shared__ double sRedS[NT];
  __shared__ int sRedI[NT];
  __shared__ double sPick[4];                        // q_i, score_i, h_ii, e
  __shared__ int sPickI[2];                          // i, code

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int K = 1 << a.bits;
  const double qmax = (double)(K - 1);
  double* M = a.slots + (int64_t)blockIdx.x * c * c;

  for (int64_t row = blockIdx.x; row < a.r; row += gridDim.x) {
    for (int64_t f = tid; f < (int64_t)c * c; f += NT) {
      const int i = (int)(f / c), j = (int)(f - (int64_t)i * c);
      M[f] = a.Hinv[(int64_t)i * a.ldh + j];
    }
    for (int k = tid; k < c; k += NT) {
      sw[k] = (double)a.W[row * a.ldw + k];
      shd[k] = a.Hinv[(int64_t)k * a.ldh + k];
      sdone[k] = 0;
    }
    double S = 1.0, Z = 0.0;
    if (a.aff) {
      S = (double)a.grid[row * 2];
      Z = (double)a.grid[row * 2 + 1];
    } else if (tid < K) {
      sG[tid] = (double)a.grid[row * K + tid];
    }
    double loss = 0.0;
    __syncthreads();

    for (int step = 0; step < c; ++step) {
      // (a) smallest loss error among the weights this thread looks at
      // (bi starts at the first weight still to do that this thread sees, so that the pick is a
      // valid index even when every score is NaN or infinite: non-finite input then gives a
      // meaningless but complete order instead of an access outside the row)
      double bs = INFINITY;
      int bi = 0x7fffffff;
      for (int k = tid; k < c; k += NT) {
        if (!sdone[k]) {
          if (bi == 0x7fffffff) bi = k;
          double q; int code;
          quant1(sw[k], sG, K, a.aff, S, Z, qmax, q, code);
          const double dq = q - sw[k];
          const double s = dq * dq / (2.0 * shd[k]);
          if (s < bs) { bs = s; bi = k; }
        }
      }
      sRedS[tid] = bs; sRedI[tid] = bi;
      __syncthreads();
      for (int h = NT / 2; h > 0; h >>= 1) {
        if (tid < h) {
          const double so = sRedS[tid + h]; const int io = sRedI[tid + h];
          if (so < sRedS[tid] || (so == sRedS[tid] && io < sRedI[tid])) { sRedS[tid] = so; sRedI[tid] = io; }
        }
        __syncthreads();
      }
      // one weight is still to do in every step, so the reduction holds a valid index; the
      // clamp only keeps every access below inside the row whatever the input
      const int i = min(sRedI[0], c - 1);
      if (tid == 0) {
        double q; int code;
        quant1(sw[i], sG, K, a.aff, S, Z, qmax, q, code);
        const double hii = shd[i];
        sPick[0] = q; sPick[1] = sRedS[0]; sPick[2] = hii; sPick[3] = (sw[i] - q) / hii;
        sPickI[0] = i; sPickI[1] = code;
      }
      // (b) row i of the inverse (= column i, the matrix is symmetric)
      for (int k = tid; k < c; k += NT) srow[k] = M[(int64_t)i * c + k];
      __syncthreads();
      const double qi = sPick[0], hii = sPick[2], e = sPick[3];
      // (c) the other weights move; weight i takes its grid value
      for (int k = tid; k < c; k += NT) {
        if (k == i) {
          sw[k] = qi;
        } else if (!sdone[k]) {
          sw[k] -= srow[k] * e;
          shd[k] -= (srow[k] / hii) * srow[k];
        }
      }
      if (tid == 0) {
        loss += sPick[1];
        a.codes[row * c + i] = (uint8_t)sPickI[1];
        if (a.order) a.order[row * c + step] = i;
      }
      // (d) Eq. 9 on the rows of weights still to come; row and column i become zero
      for (int ar = wave; ar < c; ar += NT / 64) {
        if (ar == i) {
          for (int b = lane; b < c; b += 64) M[(int64_t)ar * c + b] = 0.0;
        } else if (!sdone[ar]) {
          const double fa = srow[ar] / hii;
          double* mr = M + (int64_t)ar * c;
          for (int b = lane; b < c; b += 64) mr[b] = (b == i) ? 0.0 : mr[b] - fa * srow[b];
        }
      }
      __syncthreads();
      if (tid == 0) sdone[i] = 1;
      __syncthreads();
    }
    for (int k = tid; k < c; k += NT) a.W[row * a.ldw + k] = (float)sw[k];
    if (tid == 0 && a.row_loss) a.row_loss[row] = (float)loss;
    __syncthreads();
  }
}

// Hinv[i][j] = sum_k U[k][i] U[k][j] in fp64 (U upper triangular: k <= min(i, j)).
__global__ __launch_bounds__(256) void hinv_from_factor_kernel(const float* __restrict__ U, int64_t ldu,
                                                               int c, double* __restrict__ Hinv,
                                                               int64_t ldh) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int i = blockIdx.y;
  if (j >= c) return;
  const int kmax = i < j ? i : j;
  double s = 0.0;
  for (int k = 0; k <= kmax; ++k) s = fma((double)U[(int64_t)k * ldu + i], (double)U[(int64_t)k * ldu + j], s);
  Hinv[(int64_t)i * ldh + j] = s;
}

int exact_slots(int64_t r) { return (int)(r < MAX_SLOTS ? (r > 0 ? r : 1) : MAX_SLOTS); }

}  // namespace

namespace lq {
size_t exact_workspace_bytes(int64_t r, int64_t c) {
  return align_up((size_t)exact_slots(r) * (size_t)c * (size_t)c * sizeof(double), 256);
}
}  // namespace lq

extern "C" lq_status lq_hinv_from_factor(const float* U, int64_t ldu, int64_t c, double* Hinv,
                                         int64_t ldh, void* stream) {
  if (!U || !Hinv) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hinv_from_factor: null pointer");
  if (c < 1 || ldu < c || ldh < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hinv_from_factor: c=%lld ldu=%lld ldh=%lld", (long long)c, (long long)ldu, (long long)ldh);
  if (c > 65535) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_hinv_from_factor: c > 65535");
  dim3 grid((unsigned)lq::ceil_div(c, 256), (unsigned)c);
  hipLaunchKernelGGL(hinv_from_factor_kernel, grid, dim3(256), 0, (hipStream_t)stream, U, ldu, (int)c, Hinv, ldh);
  LQ_CHECK_LAUNCH("hinv_from_factor_kernel");
  return LQ_OK;
}

extern "C" lq_status lq_quantize_exact(float* W, int64_t r, int64_t c, int64_t ldw, const double* Hinv,
                                       int64_t ldh, const float* grid, const lq_params* P,
                                       uint8_t* codes, int32_t* order, float* row_loss, void* ws,
                                       size_t ws_bytes, void* stream) {
  if (r == 0 && c >= 1) return LQ_OK;
  if (!W || !Hinv || !grid || !codes) return lq::fail(LQ_ERR_INVALID_ARG, "lq_quantize_exact: null pointer");
  if (r < 0 || c < 1 || ldw < c || ldh < c)
    return lq::fail(LQ_ERR_INVALID_ARG, "lq_quantize_exact: r=%lld c=%lld ldw=%lld ldh=%lld", (long long)r, (long long)c, (long long)ldw, (long long)ldh);
  lq_status stt = lq::check_params(P, c);
  if (stt != LQ_OK) return stt;
  if (P->mode == LQ_GRID_AFFINE && P->group_size != 0 && P->group_size != c)
    return lq::fail(LQ_ERR_INVALID_ARG, "lq_quantize_exact: Algorithm 2 has one (S, Z) per row: group_size must be 0");
  if (c > MAX_C) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_quantize_exact: c=%lld (limit %d)", (long long)c, MAX_C);
  const size_t need = lq::exact_workspace_bytes(r, c);
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < need)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_quantize_exact: workspace needs %zu bytes, 256-byte aligned", need);

  ExactArgs a;
  a.W = W; a.ldw = ldw; a.r = r; a.c = (int)c;
  a.Hinv = Hinv; a.ldh = ldh;
  a.grid = grid; a.codes = codes; a.order = order; a.row_loss = row_loss;
  a.slots = (double*)ws;
  a.bits = P->bits; a.aff = (P->mode == LQ_GRID_AFFINE);
  const size_t lds = (size_t)c * (3 * sizeof(double) + 1) + 16;
  static lq::DeviceOnce attr_once;
  if (lq::DeviceOnceGuard once(attr_once); once.first()) {
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)exact_rows_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)(MAX_C * 25 + 16)));
    once.done();
  }
  hipLaunchKernelGGL(exact_rows_kernel, dim3((unsigned)exact_slots(r)), dim3(NT), lds, (hipStream_t)stream, a);
  LQ_CHECK_LAUNCH("exact_rows_kernel");
  return LQ_OK;
}
