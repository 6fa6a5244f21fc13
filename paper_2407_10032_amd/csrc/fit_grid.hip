// lq_fit_grid: loss-error-aware grids (Algorithm 1 lines 5-9).
//
// Non-uniform (Eq. 5, init Eq. 6): one workgroup walks rows of W; a row's weights
// and the importance weights live in registers (one HBM read of W), every Lloyd
// iteration is compare-and-accumulate in registers/LDS, and the 2*2^b cluster sums
// are reduced in a fixed order (double precision across threads).
//
// Affine (Eq. 7, t from Eq. 8): the candidate set {(t_min, t_max)} collapses to far
// fewer distinct grids.  S depends only on s = t_min + t_max, and for a fixed s the
// zero-point Z = -round(lo / S) is monotone in t_min.  A grid is fully described by
// (S, Z), so each distinct (s, Z) is scored once, in double precision, and the
// smallest objective wins -- the same minimizer as the full enumeration, at a few
// thousand instead of (t + 1)^2 evaluations per group.  When lo / S moves by less
// than one per step of t_min (T - 2t > 2^b - 1, as for T = 2048) the zero-points of a
// given s are all integers between the two ends of the t_min range; for a coarser
// partition the t_min range is walked and a grid scored whenever Z changes.
#include <math.h>

#include <type_traits>

#include "lq_common.h"

namespace {

constexpr int NT = 256;  // threads per workgroup

// ------------------------------------------------------------ importance weights
// omega_i = (d_i / min d)^-p in fp32 and fp64 (the common factor changes no argmin and
// keeps the values inside fp32 range).
__global__ __launch_bounds__(1024) void importance_kernel(const float* __restrict__ d, int64_t c,
                                                          float p, float* __restrict__ om32,
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
  for (int64_t i = threadIdx.x; i < c; i += 1024) {
    double o = pow((double)d[i] / dmin, -(double)p);
    om64[i] = o;
    om32[i] = (float)o;
  }
}

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ------------------------------------------------------------ non-uniform: weighted Lloyd
template <int K, int EPT>
__global__ __launch_bounds__(NT) void kmeans_rows_kernel(const float* __restrict__ W, int64_t r,
                                                         int64_t c, int64_t ldw,
                                                         const float* __restrict__ om32,
                                                         const float* __restrict__ init,
                                                         int max_iter, float* __restrict__ G) {
  constexpr int ACC_LD = 2 * K + 1;
  constexpr int PARTS = NT / (2 * K);   // threads that share one column of the reduction
  constexpr int RPP = NT / PARTS;       // accumulator rows per part (= 2K)
  __shared__ float sAcc[NT * ACC_LD];
  __shared__ double sSum[2 * K];
  __shared__ float sG[K];
  __shared__ float sRed[8];
  __shared__ int sChanged[2];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  float om[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    int64_t col = (int64_t)e * NT + tid;
    om[e] = (col < c) ? om32[col] : 0.0f;
  }

  for (int64_t row = blockIdx.x; row < r; row += gridDim.x) {
    float w[EPT];
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      int64_t col = (int64_t)e * NT + tid;
      if (col < c) {
        w[e] = W[row * ldw + col];
        lo = fminf(lo, w[e]);
        hi = fmaxf(hi, w[e]);
      } else {
        w[e] = 0.0f;
      }
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    if (lane == 0) { sRed[wave] = lo; sRed[4 + wave] = hi; }
    if (tid == 0) { sChanged[0] = 0; sChanged[1] = 0; }
    __syncthreads();
    lo = fminf(fminf(sRed[0], sRed[1]), fminf(sRed[2], sRed[3]));
    hi = fmaxf(fmaxf(sRed[4], sRed[5]), fmaxf(sRed[6], sRed[7]));
    // Eq. 6: evenly spaced initial grid from min to max, unless the caller supplies one
    if (tid < K) sG[tid] = init ? init[row * K + tid] : lo + (hi - lo) / (float)(K - 1) * (float)tid;
    __syncthreads();

    for (int it = 0; it < max_iter; ++it) {
      float mid[K - 1];
#pragma unroll
      for (int m = 0; m < K - 1; ++m) mid[m] = 0.5f * (sG[m] + sG[m + 1]);
      float* mine = sAcc + tid * ACC_LD;
#pragma unroll
      for (int m = 0; m < 2 * K; ++m) mine[m] = 0.0f;
      // Columns past c hold w = 0 with omega = 0 and add nothing.  The cluster of a weight is
      // the number of midpoints below it, counted from the sign bits of mid - w (w > mid
      // exactly when the difference is negative): no comparison masks, no selects, no
      // branches, so the loop is one block and the LDS updates of one weight overlap the
      // counting of the next.  (Measured alternatives: a bisection over the midpoints, same
      // speed; the read-add-writes of four weights batched, 8 % slower; LDS float atomics on
      // the thread's own slots, five times slower.)
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        uint32_t cnt = 0;
#pragma unroll
        for (int m = 0; m < K - 1; ++m) cnt += __float_as_uint(mid[m] - w[e]) >> 31;
        mine[cnt] += om[e] * w[e];
        mine[K + cnt] += om[e];
      }
      __syncthreads();
      {
        // column sums of the NT x 2K accumulator array, fixed order, in double
        const int colm = tid / PARTS, part = tid % PARTS;
        double s = 0.0;
        for (int q = 0; q < RPP; ++q) s += (double)sAcc[(part * RPP + q) * ACC_LD + colm];
#pragma unroll
        for (int o = PARTS / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (part == 0) sSum[colm] = s;
      }
      __syncthreads();
      if (tid < K) {
        double den = sSum[K + tid];
        float old = sG[tid];
        float gn = (den > 0.0) ? (float)(sSum[tid] / den) : old;
        if (gn != old) sChanged[it & 1] = 1;
        sG[tid] = gn;
      }
      __syncthreads();
      const int changed = sChanged[it & 1];
      if (tid == 0) sChanged[(it + 1) & 1] = 0;
      if (!changed) break;
    }
    if (tid < K) G[row * K + tid] = sG[tid];
    __syncthreads();
  }
}

// ------------------------------------------------------------ affine: search of Eq. 7
struct AffBest {
  double loss;
  int key;   // position of the class's first member in (t_min, t_max) lexicographic order
  double S, Z;
};

__device__ __forceinline__ bool aff_better(double l, int k, const AffBest& b) {
  return (l < b.loss) || (l == b.loss && k < b.key);
}

// NTA threads per group: the 2t + 1 values of s are dealt out NTA at a time, so the host
// picks the NTA (64, 128 or 256) that leaves the fewest idle lanes in the last round.
template <int NTA>
__global__ __launch_bounds__(NTA) void affine_search_kernel(const float* __restrict__ W, int64_t c,
                                                            int64_t ldw, int g, int ngroups,
                                                            const double* __restrict__ om64, int bits,
                                                            int T, int t, float* __restrict__ SZ) {
  constexpr int NW = NTA / 64;
  extern __shared__ __align__(16) unsigned char smraw[];
  double* sOm = reinterpret_cast<double*>(smraw);          // [g]
  double* sW = sOm + g;                                    // [g]
  __shared__ float sRed[2 * NW];
  __shared__ double sBestLoss[NTA];
  __shared__ int sBestKey[NTA];
  __shared__ double sBestS[NTA], sBestZ[NTA];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x / ngroups;
  const int gi = blockIdx.x % ngroups;
  const float* wsrc = W + row * ldw + (int64_t)gi * g;

  float lo = INFINITY, hi = -INFINITY;
  for (int i = tid; i < g; i += NTA) {
    float x = wsrc[i];
    sW[i] = (double)x;
    sOm[i] = om64[(int64_t)gi * g + i];
    lo = fminf(lo, x);
    hi = fmaxf(hi, x);
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  if (lane == 0) { sRed[wave] = lo; sRed[NW + wave] = hi; }
  __syncthreads();
  float lof = sRed[0], hif = sRed[NW];
#pragma unroll
  for (int w = 1; w < NW; ++w) { lof = fminf(lof, sRed[w]); hif = fmaxf(hif, sRed[NW + w]); }
  const double lo0 = (double)lof;
  const double hi0 = (double)hif;
  const double R = hi0 - lo0;
  float* out = SZ + (row * ngroups + gi) * 2;
  if (R == 0.0) {  // constant group
    if (tid == 0) { out[0] = 1.0f; out[1] = 0.0f; }
    return;
  }
  const double qmax = (double)((1 << bits) - 1);
  const double dT = (double)T;

  AffBest best;
  best.loss = INFINITY; best.key = 0x7fffffff; best.S = 1.0; best.Z = 0.0;
  // Objective of Eq. 7 for one grid (S, Z); key orders equal losses like the plain enumeration.
  auto score = [&](double S, double Z, int key) {
    const double invS = 1.0 / S;
    const double cl = -Z, ch = qmax - Z;
    double loss = 0.0;
    for (int i = 0; i < g; ++i) {
      double w = sW[i];
      double u = fmin(fmax(rint(w * invS), cl), ch);
      double dlt = fma(u, S, -w);
      loss = fma(sOm[i] * dlt, dlt, loss);
    }
    if (aff_better(loss, key, best)) { best.loss = loss; best.key = key; best.S = S; best.Z = Z; }
  };
  // The same objective for ZC consecutive zero-points Z0, Z0 - 1, .. of one scale in a single
  // pass over the weights: round(w / S) does not depend on Z, only the clipping does.  With
  // CLIP32 the clipping is one fp32 median-of-three instead of an fp64 max and min (both
  // half rate); round(w / S) and the bounds are integers below 2^23 in that case (checked per
  // group), so the clipped value is the same number and every loss is bit-identical to score().
  auto score_many = [&](auto zc_tag, auto clip_tag, double S, double Z0, double* loss) {
    constexpr int ZC = decltype(zc_tag)::value;
    constexpr bool CLIP32 = decltype(clip_tag)::value;
    const double invS = 1.0 / S;
    double l[ZC];
    float clf[ZC], chf[ZC];
#pragma unroll
    for (int k = 0; k < ZC; ++k) {
      l[k] = 0.0;
      clf[k] = (float)(-(Z0 - (double)k));
      chf[k] = (float)(qmax - (Z0 - (double)k));
    }
    for (int i = 0; i < g; ++i) {
      const double w = sW[i], om = sOm[i];
      const double u0 = rint(w * invS);
      const float u0f = (float)u0;
#pragma unroll
      for (int k = 0; k < ZC; ++k) {
        double u;
        if (CLIP32) {
          u = (double)__builtin_amdgcn_fmed3f(u0f, clf[k], chf[k]);
        } else {
          const double Z = Z0 - (double)k;
          u = fmin(fmax(u0, -Z), qmax - Z);
        }
        const double dlt = fma(u, S, -w);
        l[k] = fma(om * dlt, dlt, l[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < ZC; ++k) loss[k] = l[k];
  };
  // |round(w / S)| and |Z| stay below 2^23 for every candidate of this group if
  // max|w| / S_min does, with S_min = R (T - 2t) / (T (2^b - 1)) the smallest scale searched
  const double smin = R * (double)(T - 2 * t) / (dT * qmax);
  const bool clip32 = smin > 0.0 && fmax(fabs(lo0), fabs(hi0)) / smin < 4.0e6;
  // lo / S moves by (2^b - 1) / (T - s) per step of t_min.  When that is below one for every
  // s (T - 2t > 2^b - 1, true for the paper's T = 2048) the zero-points reached for a given s
  // are exactly the integers between the values at the two ends of the t_min range.
  const bool dense = (double)(T - 2 * t) > qmax;
  const int rounds = (2 * t + NTA) / NTA;                 // every lane runs every round: the
  for (int rd = 0; rd < rounds; ++rd) {                   // pass width is chosen per wavefront
    const int s = tid + rd * NTA;
    const bool live = s <= 2 * t;
    const int ta = (s > t) ? (s - t) : 0;      // smallest t_min with t_max = s - t_min <= t
    const int tb = (s < t) ? s : t;            // largest t_min
    if (dense) {
      const double lo_a = lo0 + (double)ta * R / dT;
      const double hi_a = hi0 - (double)(s - ta) * R / dT;
      const double S = (hi_a - lo_a) / qmax;
      const bool ok = live && (S > 0.0);
      const double Sx = ok ? S : 1.0;
      const double lo_b = lo0 + (double)tb * R / dT;
      const double zf = -rint(lo_a / Sx);
      const double zl = -rint(lo_b / Sx);
      double span = zf - zl;
      if (!(span >= 0.0)) span = 0.0;
      const int nz = ok ? (int)fmin(span, 63.0) + 1 : 0;
      // widest class count in this wavefront decides how many zero-points share a pass
      int nzw = nz;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) nzw = max(nzw, __shfl_xor(nzw, o, 64));
      for (int z0 = 0; z0 < nzw; ) {
        double loss[4];
        int cnt;
        const double Z0 = zf - (double)z0;
        cnt = nzw - z0 >= 4 ? 4 : nzw - z0;
        if (clip32) {
          if (cnt == 4) score_many(std::integral_constant<int, 4>{}, std::true_type{}, Sx, Z0, loss);
          else if (cnt == 3) score_many(std::integral_constant<int, 3>{}, std::true_type{}, Sx, Z0, loss);
          else if (cnt == 2) score_many(std::integral_constant<int, 2>{}, std::true_type{}, Sx, Z0, loss);
          else score_many(std::integral_constant<int, 1>{}, std::true_type{}, Sx, Z0, loss);
        } else {
          if (cnt >= 2) { score_many(std::integral_constant<int, 2>{}, std::false_type{}, Sx, Z0, loss); cnt = 2; }
          else score_many(std::integral_constant<int, 1>{}, std::false_type{}, Sx, Z0, loss);
        }
        for (int k = 0; k < cnt; ++k) {
          const int zi = z0 + k;
          if (zi < nz) {
            const double Z = zf - (double)zi;
            // first t_min of this class: smallest t_min >= ta with round(lo / S) == -Z
            int tf = ta;
            if (zi > 0) {
              tf = (int)ceil(((-Z - 0.5) * S - lo0) * dT / R);
              tf = tf < ta ? ta : (tf > tb ? tb : tf);
            }
            const int key = tf * (t + 1) + (s - tf);
            if (aff_better(loss[k], key, best)) { best.loss = loss[k]; best.key = key; best.S = S; best.Z = Z; }
          }
        }
        z0 += cnt;
      }
    } else if (live) {
      double zprev = 0.0;
      for (int tm = ta; tm <= tb; ++tm) {
        const double lo_c = lo0 + (double)tm * R / dT;
        const double hi_c = hi0 - (double)(s - tm) * R / dT;
        const double S = (hi_c - lo_c) / qmax;
        if (!(S > 0.0)) continue;
        const double Z = -rint(lo_c / S);
        if (tm == ta || Z != zprev) score(S, Z, tm * (t + 1) + (s - tm));
        zprev = Z;
      }
    }
  }
  sBestLoss[tid] = best.loss; sBestKey[tid] = best.key; sBestS[tid] = best.S; sBestZ[tid] = best.Z;
  __syncthreads();
  for (int w2 = NTA / 2; w2 > 0; w2 >>= 1) {
    if (tid < w2) {
      AffBest o;
      o.loss = sBestLoss[tid]; o.key = sBestKey[tid];
      if (aff_better(sBestLoss[tid + w2], sBestKey[tid + w2], o)) {
        sBestLoss[tid] = sBestLoss[tid + w2]; sBestKey[tid] = sBestKey[tid + w2];
        sBestS[tid] = sBestS[tid + w2]; sBestZ[tid] = sBestZ[tid + w2];
      }
    }
    __syncthreads();
  }
  if (tid == 0) { out[0] = (float)sBestS[0]; out[1] = (float)sBestZ[0]; }
}

template <int K>
lq_status launch_kmeans(const float* W, int64_t r, int64_t c, int64_t ldw, const float* om32,
                        const float* init, int max_iter, float* G, hipStream_t st) {
  int64_t ept = lq::ceil_div(c, NT);
  unsigned grid = (unsigned)(r < 2048 ? r : 2048);
#define LQ_KM(E)                                                                              \
  hipLaunchKernelGGL((kmeans_rows_kernel<K, E>), dim3(grid), dim3(NT), 0, st, W, r, c, ldw, \
                     om32, init, max_iter, G)
  if (ept <= 2) LQ_KM(2);
  else if (ept <= 4) LQ_KM(4);
  else if (ept <= 8) LQ_KM(8);
  else if (ept <= 16) LQ_KM(16);
  else if (ept <= 32) LQ_KM(32);
  else if (ept <= 44) LQ_KM(44);
  else LQ_KM(64);
#undef LQ_KM
  LQ_CHECK_LAUNCH("kmeans_rows_kernel");
  return LQ_OK;
}

}  // namespace

namespace lq {
size_t fit_grid_workspace_bytes(int64_t c) {
  return align_up((size_t)c * sizeof(double), 256) + align_up((size_t)c * sizeof(float), 256);
}
}  // namespace lq

namespace {
lq_status fit_grid_impl(const float* W, int64_t r, int64_t c, int64_t ldw, const float* hinv_diag,
                        const lq_params* P, const float* init_grid, float* grid, void* ws,
                        size_t ws_bytes, void* stream);

// ---- scratch of lq_fit_grid_static: the importance weights of up to STATIC_MAX_C columns in
// fp64 and fp32, held in the library's own device image (one copy per GPU, for the life of the
// process).  Host code never uses the array's name as an address: its device address is asked
// for once per device and kept.
constexpr int64_t STATIC_MAX_C = 16384;
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)STATIC_MAX_C * (sizeof(double) + sizeof(float));
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

lq_status static_scratch(void** out) {
  static std::mutex mu;
  static void* ptr[lq::MAX_DEVICES] = {};
  int dev = -1;
  LQ_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= lq::MAX_DEVICES)
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid_static: device index %d (limit %d)", dev, lq::MAX_DEVICES);
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    LQ_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return lq::fail(LQ_ERR_HIP, "lq_fit_grid_static: the scratch array has no device address");
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return LQ_OK;
}
}


extern "C" lq_status lq_fit_grid(const float* W, int64_t r, int64_t c, int64_t ldw,
                                 const float* hinv_diag, const lq_params* P, float* grid, void* ws,
                                 size_t ws_bytes, void* stream) {
  return fit_grid_impl(W, r, c, ldw, hinv_diag, P, nullptr, grid, ws, ws_bytes, stream);
}

extern "C" lq_status lq_fit_grid_static(const float* W, int64_t r, int64_t c, int64_t ldw,
                                        const float* hinv_diag, const lq_params* P, float* grid,
                                        void* stream) {
  if (c > STATIC_MAX_C)
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid_static: c=%lld exceeds the built-in scratch (c <= %lld); "
                    "use lq_fit_grid with a workspace", (long long)c, (long long)STATIC_MAX_C);
  if (c >= 1 && lq::fit_grid_workspace_bytes(c) > STATIC_SCRATCH_BYTES)
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid_static: c=%lld needs more than the built-in scratch", (long long)c);
  void* ws = nullptr;
  lq_status st = static_scratch(&ws);
  if (st != LQ_OK) return st;
  // the kernels write every scratch entry they later read (importance weights of the c
  // columns), so nothing needs clearing between calls
  return fit_grid_impl(W, r, c, ldw, hinv_diag, P, nullptr, grid, ws, STATIC_SCRATCH_BYTES, stream);
}

extern "C" lq_status lq_fit_grid_from(const float* W, int64_t r, int64_t c, int64_t ldw,
                                      const float* hinv_diag, const lq_params* P,
                                      const float* init_grid, float* grid, void* ws, size_t ws_bytes,
                                      void* stream) {
  if (P && P->mode != LQ_GRID_NONUNIFORM && init_grid)
    return lq::fail(LQ_ERR_INVALID_ARG, "lq_fit_grid_from: an initial grid applies to non-uniform grids only");
  return fit_grid_impl(W, r, c, ldw, hinv_diag, P, init_grid, grid, ws, ws_bytes, stream);
}

namespace {
lq_status fit_grid_impl(const float* W, int64_t r, int64_t c, int64_t ldw, const float* hinv_diag,
                        const lq_params* P, const float* init_grid, float* grid, void* ws,
                        size_t ws_bytes, void* stream) {
  if (r == 0 && c >= 1) return LQ_OK;   // nothing to do; empty buffers may be null
  if (!W || !hinv_diag || !grid) return lq::fail(LQ_ERR_INVALID_ARG, "lq_fit_grid: null pointer");
  if (r < 0 || c < 1 || ldw < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_fit_grid: r=%lld c=%lld ldw=%lld", (long long)r, (long long)c, (long long)ldw);
  lq_status stt = lq::check_params(P, c);
  if (stt != LQ_OK) return stt;
  size_t need = lq::fit_grid_workspace_bytes(c);
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < need)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_fit_grid: workspace needs %zu bytes, 256-byte aligned", need);
  if (r == 0) return LQ_OK;

  hipStream_t st = (hipStream_t)stream;
  double* om64 = (double*)ws;
  float* om32 = (float*)((char*)ws + lq::align_up((size_t)c * sizeof(double), 256));

  if (P->mode == LQ_GRID_NONUNIFORM) {
    if (c > 64 * NT) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid: non-uniform fit supports c <= %d", 64 * NT);
    hipLaunchKernelGGL(importance_kernel, dim3(1), dim3(1024), 0, st, hinv_diag, c, P->p, om32, om64);
    LQ_CHECK_LAUNCH("importance_kernel");
    switch (P->bits) {
      case 2: return launch_kmeans<4>(W, r, c, ldw, om32, init_grid, P->kmeans_max_iter, grid, st);
      case 3: return launch_kmeans<8>(W, r, c, ldw, om32, init_grid, P->kmeans_max_iter, grid, st);
      default: return launch_kmeans<16>(W, r, c, ldw, om32, init_grid, P->kmeans_max_iter, grid, st);
    }
  }

  const int64_t g = P->group_size > 0 ? P->group_size : c;
  if (g > 8192) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid: affine group of %lld columns (limit 8192)", (long long)g);
  const int64_t ngroups = c / g;
  if (r * ngroups > 0x7fffffffLL) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid: more than 2^31 groups");
  hipLaunchKernelGGL(importance_kernel, dim3(1), dim3(1024), 0, st, hinv_diag, c, P->p, om32, om64);
  LQ_CHECK_LAUNCH("importance_kernel");
  const size_t lds = (size_t)g * 2 * sizeof(double);
  const int t = lq::resolve_t(P);
  const int ns = 2 * t + 1;
  // threads per group: fewest idle lanes in the last round of s values; ties go to the larger
  int nta = 256;
  {
    int best = (ns + 255) / 256 * 256;
    for (int cand : {128, 64}) {
      const int padded = (ns + cand - 1) / cand * cand;
      if (padded < best) { best = padded; nta = cand; }
    }
  }
  static lq::DeviceOnce attr_once;
  if (lq::DeviceOnceGuard once(attr_once); once.first()) {
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)affine_search_kernel<64>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)(8192 * 16)));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)affine_search_kernel<128>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)(8192 * 16)));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)affine_search_kernel<256>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)(8192 * 16)));
    once.done();
  }
  const dim3 ggrid((unsigned)(r * ngroups));
#define LQ_AFF(N) hipLaunchKernelGGL(affine_search_kernel<N>, ggrid, dim3(N), lds, st, W, c, ldw, (int)g, \
                                     (int)ngroups, (const double*)om64, P->bits, P->T, t, grid)
  if (nta == 64) LQ_AFF(64);
  else if (nta == 128) LQ_AFF(128);
  else LQ_AFF(256);
#undef LQ_AFF
  LQ_CHECK_LAUNCH("affine_search_kernel");
  return LQ_OK;
}
}  // namespace

