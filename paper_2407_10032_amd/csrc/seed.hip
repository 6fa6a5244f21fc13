// lq_kmeanspp_seed: weighted k-means++ seeding of the non-uniform grids, the initialisation
// the paper's appendix table on grid point initialisation compares Eq. 6 against (D^2
// sampling with the importance weights of Eq. 5 as point masses).  The uniform numbers are an
// input, so the result is a function of the arguments.
//
// One workgroup per row, everything in fp64 (a draw is decided by comparing a cumulative mass
// with u * total).  Thread t owns the contiguous columns [t E, (t + 1) E): its cumulative
// masses are a running sum in column order on top of the exclusive scan of the threads'
// totals.  The row sits in LDS, each point's squared distance to its nearest centre so far
// in registers.
#include "lq_common.h"

namespace lq {
size_t fit_grid_workspace_bytes(int64_t c);
}

namespace {

constexpr int NT = 256;

// omega_i = (d_i / min d)^-p in fp64, as the grid fit uses it
__global__ __launch_bounds__(1024) void seed_importance_kernel(const float* __restrict__ d, int64_t c, float p,
                                                               double* __restrict__ om64) {
  __shared__ float red[1024];
  float m = INFINITY;
  for (int64_t i = threadIdx.x; i < c; i += 1024) m = fminf(m, d[i]);
  red[threadIdx.x] = m;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = fminf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  const double dmin = (double)red[0];
  for (int64_t i = threadIdx.x; i < c; i += 1024) om64[i] = pow((double)d[i] / dmin, -(double)p);
}

// smallest value over the workgroup (every thread gets it); `slot` is NT / 64 ints of LDS
__device__ __forceinline__ int block_min(int v, int* slot) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  __syncthreads();                       // the previous use of slot is over
  if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  int m = slot[0];
#pragma unroll
  for (int w = 1; w < NT / 64; ++w) m = min(m, slot[w]);
  return m;
}

template <int EMAX>
__global__ __launch_bounds__(NT) void kmeanspp_rows_kernel(const float* __restrict__ W, int64_t r, int64_t c,
                                                           int64_t ldw, const double* __restrict__ om64,
                                                           const double* __restrict__ u, int K,
                                                           float* __restrict__ G) {
  extern __shared__ float sw[];          // the row, c floats
  __shared__ double sScan[NT];
  __shared__ int sSlot[NT / 64];
  __shared__ float sCentre[16];
  const int tid = threadIdx.x;
  const int E = (int)((c + NT - 1) / NT);
  const int64_t j0 = (int64_t)tid * E;

  for (int64_t row = blockIdx.x; row < r; row += gridDim.x) {
    __syncthreads();                     // the previous row's LDS is no longer read
    for (int64_t j = tid; j < c; j += NT) sw[j] = W[row * ldw + j];
    __syncthreads();
    double dist2[EMAX];
#pragma unroll
    for (int e = 0; e < EMAX; ++e) dist2[e] = INFINITY;

    for (int m = 0; m < K; ++m) {
      // mass of point j: omega_j for the first centre, omega_j * dist2_j afterwards
      double local = 0.0;
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        const int64_t j = j0 + e;
        if (e < E && j < c) local += (m == 0) ? om64[j] : om64[j] * dist2[e];
      }
      // inclusive scan of the threads' totals
      __syncthreads();
      sScan[tid] = local;
      __syncthreads();
      for (int o = 1; o < NT; o <<= 1) {
        const double add = tid >= o ? sScan[tid - o] : 0.0;
        __syncthreads();
        sScan[tid] += add;
        __syncthreads();
      }
      const double total = sScan[NT - 1];
      const double excl = tid > 0 ? sScan[tid - 1] : 0.0;
      int pick = 0;
      if (total > 0.0) {
        const double target = u[row * K + m] * total;
        // first index whose cumulative mass reaches the target
        int first = 0x7fffffff;
        double run = excl;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
          const int64_t j = j0 + e;
          if (e < E && j < c) {
            run += (m == 0) ? om64[j] : om64[j] * dist2[e];
            if (run >= target && first == 0x7fffffff) first = (int)j;
          }
        }
        first = block_min(first, sSlot);
        if (first == 0x7fffffff) first = (int)c - 1;
        // a point without mass cannot be drawn: move on to the next one that has some
        int next = 0x7fffffff;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
          const int64_t j = j0 + e;
          if (e < E && j < c && j >= first && next == 0x7fffffff) {
            const double mass = (m == 0) ? om64[j] : om64[j] * dist2[e];
            if (mass != 0.0) next = (int)j;
          }
        }
        next = block_min(next, sSlot);
        pick = next == 0x7fffffff ? (int)c - 1 : next;
      }
      const float g = sw[pick];
      if (tid == 0) sCentre[m] = g;
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        const int64_t j = j0 + e;
        if (e < E && j < c) {
          const double diff = (double)sw[j] - (double)g;
          dist2[e] = fmin(dist2[e], diff * diff);
        }
      }
    }
    __syncthreads();
    if (tid == 0) {                      // ascending order, as the Lloyd iteration expects
      float v[16];
      for (int m = 0; m < K; ++m) v[m] = sCentre[m];
      for (int a = 1; a < K; ++a) {
        const float x = v[a];
        int b = a - 1;
        while (b >= 0 && v[b] > x) { v[b + 1] = v[b]; --b; }
        v[b + 1] = x;
      }
      for (int m = 0; m < K; ++m) G[row * K + m] = v[m];
    }
  }
}

}  // namespace

extern "C" lq_status lq_kmeanspp_seed(const float* W, int64_t r, int64_t c, int64_t ldw,
                                      const float* hinv_diag, const lq_params* P, const double* u,
                                      float* grid_init, void* ws, size_t ws_bytes, void* stream) {
  if (r == 0 && c >= 1) return LQ_OK;
  if (!W || !hinv_diag || !u || !grid_init) return lq::fail(LQ_ERR_INVALID_ARG, "lq_kmeanspp_seed: null pointer");
  if (r < 0 || c < 1 || ldw < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_kmeanspp_seed: r=%lld c=%lld ldw=%lld", (long long)r, (long long)c, (long long)ldw);
  lq_status stt = lq::check_params(P, c);
  if (stt != LQ_OK) return stt;
  if (P->mode != LQ_GRID_NONUNIFORM) return lq::fail(LQ_ERR_INVALID_ARG, "lq_kmeanspp_seed: seeding applies to non-uniform grids only");
  if (c > 64 * NT) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_kmeanspp_seed: supports c <= %d", 64 * NT);
  const size_t need = lq::fit_grid_workspace_bytes(c);
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < need)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_kmeanspp_seed: workspace needs %zu bytes, 256-byte aligned", need);

  hipStream_t st = (hipStream_t)stream;
  double* om64 = (double*)ws;
  hipLaunchKernelGGL(seed_importance_kernel, dim3(1), dim3(1024), 0, st, hinv_diag, c, P->p, om64);
  LQ_CHECK_LAUNCH("seed_importance_kernel");
  const int K = 1 << P->bits;
  const size_t lds = (size_t)c * sizeof(float);
  const dim3 grid((unsigned)(r < 8192 ? r : 8192)), block(NT);
  static lq::DeviceOnce attr_once;
  if (lq::DeviceOnceGuard once(attr_once); once.first()) {
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)kmeanspp_rows_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * NT * 4));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)kmeanspp_rows_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * NT * 4));
    once.done();
  }
  if (c <= 16 * NT)
    hipLaunchKernelGGL(kmeanspp_rows_kernel<16>, grid, block, lds, st, W, r, c, ldw, (const double*)om64, u, K, grid_init);
  else
    hipLaunchKernelGGL(kmeanspp_rows_kernel<64>, grid, block, lds, st, W, r, c, ldw, (const double*)om64, u, K, grid_init);
  LQ_CHECK_LAUNCH("kmeanspp_rows_kernel");
  return LQ_OK;
}
