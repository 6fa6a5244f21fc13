// lq_fit_grid: loss-error-aware grids (Algorithm 1 lines 5-9).
//
// Non-uniform (Eq. 5, init Eq. 6): workgroups take rows of W from a counter; a row's weights
// and importance weights live in registers (one HBM read of W), a weight's cluster comes
// from a table over fine bins of the row's range (one table byte, one midpoint, one compare
// instead of 2^b - 1 compares), and the 2 * 2^b cluster sums are reduced in a fixed order
// (double precision across threads).
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
                                                          double* __restrict__ om64,
                                                          int* __restrict__ next_row) {
  __shared__ float red[1024];
  if (threadIdx.x == 0) *next_row = 0;      // row counter of the non-uniform fit
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
// Workgroups take rows from a shared counter (rows need from 2 to 100 Lloyd updates, so a
// fixed split would leave compute units idle).  A row's weights, their importance weights
// and the fine bin each weight falls into stay in registers (W is read from HBM exactly once).
//
// Cluster of a weight = number of midpoints of the current grid below it.  Instead of
// comparing every weight with all 2^b - 1 midpoints in every iteration, the range
// [min, max] of the row is cut into NBIN equal bins once; in an iteration a table over the
// bins holds c0 = how many midpoints lie in lower bins.  The bin function is monotone, so a
// midpoint in a lower bin is below the weight and one in a higher bin is above it: only the
// midpoints that share the weight's bin need a comparison, and they are midpoints c0,
// c0 + 1, ...  With at most one midpoint per bin (the usual case) a weight costs one table
// byte, one midpoint and one compare; if some bin holds n > 1 of them (a grid much finer
// than the bins) every weight compares with n consecutive midpoints -- those beyond its
// bin lie above it and add nothing -- so the count is the same in every case.
//
// Sums: each thread adds omega * w and omega to its own slot of the cluster (cluster-major,
// so a wavefront's slots never share an LDS bank whatever the clusters are; the slots of the
// next weight are read before those of the current one are written, with the fresh values
// carried over when both hit the same slot); the 2 * 2^b columns are then added in a fixed
// order in double and the lanes that hold a cluster's two sums form its new grid point.
// Lloyd stops when no grid point changes.
constexpr int NBIN = 1024;

__device__ __forceinline__ double recip_f64(double x) {
  // reciprocal to ~1e-30 relative: hardware estimate and two Newton steps (the quotient is
  // rounded to fp32 afterwards)
  double y = __builtin_amdgcn_rcp(x);
  y = fma(fma(-x, y, 1.0), y, y);
  y = fma(fma(-x, y, 1.0), y, y);
  return y;
}

// NTK threads per workgroup (256, or 512 for long rows so that a thread holds at most 32
// weights); the second launch bound is the number of wavefronts per SIMD the register
// allocation must leave room for.
template <int K, int EPT, int NTK>
__global__ __launch_bounds__(NTK, 4) void kmeans_rows_kernel(const float* __restrict__ W, int64_t r,
                                                         int64_t c, int64_t ldw,
                                                         const float* __restrict__ om32,
                                                         const float* __restrict__ init,
                                                         int max_iter, float* __restrict__ G,
                                                         int* __restrict__ next_row) {
  constexpr int NT = NTK;               // (shadows the file-level constant on purpose)
  constexpr int NW = NT / 64;
  constexpr int PARTS = (NT / (2 * K) < 32) ? NT / (2 * K) : 32;   // threads per column of the reduction
  constexpr int RPP = NT / PARTS;       // slots each of them adds (a power of two)
  constexpr int BPT = NBIN / NT;        // bins per thread when the table is built
  static_assert(2 * PARTS <= 64 && RPP % 4 == 0 && (2 * K * PARTS) % 64 == 0 && 2 * K * PARTS <= NT,
                "a cluster's two columns sit in one wavefront; whole wavefronts take part");
  static_assert(BPT == 4 || BPT == 2, "table build handles 2 or 4 bins per thread");
  __shared__ __align__(16) float sAcc[2 * K * NT];   // [2K][NT]: sums of omega w, then of omega
  __shared__ __align__(16) uint8_t sLut[NBIN];       // c0 of every bin
  __shared__ __align__(16) int sCnt[NBIN];           // midpoints per bin
  __shared__ __align__(16) int sBm[16];              // bin of midpoint m (NBIN beyond K - 1)
  __shared__ float sG[K];
  __shared__ float sMid[2 * K];                      // midpoints, +inf beyond K - 1
  __shared__ float sRed[2 * NW];
  __shared__ int sChanged[2];                        // by iteration parity
  __shared__ int sMulti;                             // most midpoints in one bin
  __shared__ int sRow;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  float om[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    int64_t col = (int64_t)e * NT + tid;
    om[e] = (col < c) ? om32[col] : 0.0f;
  }
  for (int i = tid; i < NBIN; i += NT) sCnt[i] = 0;
  if (tid < 16) sBm[tid] = NBIN;
  if (tid < 2 * K) sMid[tid] = INFINITY;
  int bm_mine = 0;      // wavefront 0, lane m: bin of midpoint m of the grid last published

  for (;;) {
    if (tid == 0) sRow = atomicAdd(next_row, 1);
    __syncthreads();
    const int64_t row = sRow;
    if (row >= r) break;
    float w[EPT];
    float lo = INFINITY, hi = -INFINITY;
    {
      // 32-bit column offsets from the row's (uniform) base; the opaque copy of the thread
      // index keeps the compiler from holding an address and a predicate per weight in
      // registers across rows
      const float* wrow = W + row * ldw;
      uint32_t t0 = (uint32_t)tid;
      asm volatile("" : "+v"(t0));
      const uint32_t cc = (uint32_t)c;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t col = (uint32_t)(e * NT) + t0;
        if (col < cc) {
          w[e] = wrow[col];
          lo = fminf(lo, w[e]);
          hi = fmaxf(hi, w[e]);
        } else {
          w[e] = 0.0f;
        }
      }
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    if (lane == 0) { sRed[wave] = lo; sRed[NW + wave] = hi; }
    __syncthreads();
    lo = sRed[0];
    hi = sRed[NW];
#pragma unroll
    for (int v = 1; v < NW; ++v) { lo = fminf(lo, sRed[v]); hi = fmaxf(hi, sRed[NW + v]); }
    // monotone bin function of this row (a constant row puts everything into bin 0)
    const float bscale = (hi > lo) ? (float)NBIN / (hi - lo) : 0.0f;
    auto bin_of = [&](float x) -> int {
      return (int)fminf(fmaxf((x - lo) * bscale, 0.0f), (float)(NBIN - 1));
    };
    // the weights' bins, two 16-bit values per register; with 32 weights per thread they are
    // recomputed in every iteration instead (registers)
    constexpr bool KEEP_BINS = EPT <= 22;
    uint32_t ba2[KEEP_BINS ? (EPT + 1) / 2 : 1];
    if constexpr (KEEP_BINS) {
#pragma unroll
      for (int e = 0; e < EPT; e += 2) {
        const uint32_t b0 = (uint32_t)bin_of(w[e]);
        const uint32_t b1 = (e + 1 < EPT) ? (uint32_t)bin_of(w[e + 1]) : 0u;
        ba2[e >> 1] = b0 | (b1 << 16);
      }
    }

    // Wavefront 0 publishes a grid that lanes 0..K-1 have written to sG: its midpoints,
    // their bins, and the number of midpoints per bin.
    auto publish = [&]() {
      __builtin_amdgcn_wave_barrier();
      if (tid < K - 1) {
        const float m = 0.5f * (sG[tid] + sG[tid + 1]);
        const int b = bin_of(m);
        sMid[tid] = m;
        sBm[tid] = b;
        atomicAdd(&sCnt[b], 1);
        bm_mine = b;
      }
      if (tid == 0) sMulti = 0;
    };
    if (wave == 0) {
      if (tid < K - 1) sCnt[bm_mine] = 0;      // counts left by the previous row's last grid
      // Eq. 6: evenly spaced initial grid from min to max, unless the caller supplies one
      if (tid < K) sG[tid] = init ? init[row * K + tid] : lo + (hi - lo) / (float)(K - 1) * (float)tid;
      if (tid == 0) { sChanged[0] = 0; sChanged[1] = 0; }
      publish();
    }
    __syncthreads();

    for (int it = 0; it < max_iter; ++it) {
      // ---- table over the bins for the published grid (4 consecutive bins per thread)
      {
        const int b0 = BPT * tid;
        int c0 = 0;
#pragma unroll
        for (int m = 0; m < K - 1; ++m) c0 += (sBm[m] < b0) ? 1 : 0;
        int nmax;
        if constexpr (BPT == 4) {
          const int4 n4 = *reinterpret_cast<const int4*>(&sCnt[b0]);
          const int c1 = c0 + n4.x, c2 = c1 + n4.y, c3 = c2 + n4.z;
          reinterpret_cast<uint32_t*>(sLut)[tid] =
              (uint32_t)c0 | ((uint32_t)c1 << 8) | ((uint32_t)c2 << 16) | ((uint32_t)c3 << 24);
          nmax = max(max(n4.x, n4.y), max(n4.z, n4.w));
        } else {
          const int2 n2 = *reinterpret_cast<const int2*>(&sCnt[b0]);
          reinterpret_cast<uint16_t*>(sLut)[tid] = (uint16_t)((uint32_t)c0 | ((uint32_t)(c0 + n2.x) << 8));
          nmax = max(n2.x, n2.y);
        }
        if (nmax >= 2) atomicMax(&sMulti, nmax);
        // the private sums start from zero (cleared cooperatively, 16 bytes per store)
        float4* z = reinterpret_cast<float4*>(sAcc);
#pragma unroll
        for (int q = 0; q < 2 * K / 4; ++q) z[q * NT + tid] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (tid == 0) sChanged[(it + 1) & 1] = 0;
      }
      __syncthreads();
      const int multi = sMulti;
      // ---- every weight into its cluster's sums.  Columns past c hold w = 0, omega = 0.
      auto accumulate = [&](auto multi_tag) {
        constexpr bool MULTI = decltype(multi_tag)::value;
        auto cluster_of = [&](int e) -> int {
          uint32_t b;
          if constexpr (KEEP_BINS) b = (e & 1) ? (ba2[e >> 1] >> 16) : (ba2[e >> 1] & 0xffffu);
          else b = (uint32_t)bin_of(w[e]);
          const int c0 = sLut[b];
          if (!MULTI) return c0 + ((w[e] > sMid[c0]) ? 1 : 0);
          int k2 = c0;
          for (int k = 0; k < multi; ++k) k2 += (w[e] > sMid[c0 + k]) ? 1 : 0;
          return k2;
        };
        int cl = cluster_of(0);
        float* p = sAcc + cl * NT + tid;
        float a = p[0], b = p[K * NT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
          int cn = cl;
          float* pn = p;
          float an = 0.f, bn = 0.f;
          if (e + 1 < EPT) {
            cn = cluster_of(e + 1);
            pn = sAcc + cn * NT + tid;
            an = pn[0];
            bn = pn[K * NT];
          }
          a = fmaf(om[e], w[e], a);
          b += om[e];
          p[0] = a;
          p[K * NT] = b;
          if (e + 1 < EPT) {
            const bool same = cn == cl;
            a = same ? a : an;
            b = same ? b : bn;
            p = pn;
            cl = cn;
          }
          // keep the compiler from hoisting the table reads of many weights ahead (registers)
          if ((e & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
      };
      if (multi <= 1) accumulate(std::false_type{});
      else accumulate(std::true_type{});
      __syncthreads();
      {
        // Column sums of the 2K x NT slots in double.  Thread group gidx = 2 m + which adds
        // column which * K + m (which = 0: sum of omega w, 1: sum of omega of cluster m); a
        // thread adds RPP slots starting at a lane-dependent one so that a wavefront reads
        // distinct banks.  The two groups of a cluster are PARTS lanes apart.
        const int gidx = tid / PARTS, part = tid % PARTS;
        const int m = (gidx >> 1) & (K - 1), which = gidx & 1;      // groups beyond 2K idle along
        const float* src = sAcc + (which * K + m) * NT + part * RPP;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll 2
        for (int q = 0; q < RPP; q += 4) {
          s0 += (double)src[(q + tid) & (RPP - 1)];
          s1 += (double)src[(q + 1 + tid) & (RPP - 1)];
          s2 += (double)src[(q + 2 + tid) & (RPP - 1)];
          s3 += (double)src[(q + 3 + tid) & (RPP - 1)];
        }
        double s = (s0 + s1) + (s2 + s3);
#pragma unroll
        for (int o = PARTS / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        const double den = __shfl_down(s, PARTS, 64);
        if (which == 0 && part == 0 && gidx < 2 * K) {
          const float old = sG[m];
          // an empty cluster keeps its point
          const float gn = (den > 0.0) ? (float)(s * recip_f64(den)) : old;
          if (gn != old) {
            sG[m] = gn;
            sChanged[it & 1] = 1;
          }
        }
      }
      __syncthreads();
      const int changed = sChanged[it & 1];
      if (wave == 0) {
        if (tid < K - 1) sCnt[bm_mine] = 0;                  // counts of the grid just used
        if (changed) publish();
      }
      if (!changed) break;
      __syncthreads();
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

// double -> float rounded towards +infinity (the smallest float >= x), for 8, 4, 2 or 1 values.  The
// rounding mode of single-precision results (MODE bits 1:0, which v_cvt_f32_f64 follows) is
// switched inside the statement and back, so no other instruction ever runs under it; the waits
// keep the switch clear of the vector instructions issued before and after it.
#define LQ_RU_ON  "s_nop 3\n\ts_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 1\n\ts_nop 2\n\t"
#define LQ_RU_OFF "s_nop 2\n\ts_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 0\n\ts_nop 1"
__device__ __forceinline__ void cvt_up4(float* o, const double* a) {
  asm volatile(LQ_RU_ON "v_cvt_f32_f64 %0, %4\n\tv_cvt_f32_f64 %1, %5\n\tv_cvt_f32_f64 %2, %6\n\tv_cvt_f32_f64 %3, %7\n\t" LQ_RU_OFF
               : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3])
               : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]));
}
__device__ __forceinline__ void cvt_up8(float* o, const double* a) {
  asm volatile(LQ_RU_ON "v_cvt_f32_f64 %0, %8\n\tv_cvt_f32_f64 %1, %9\n\tv_cvt_f32_f64 %2, %10\n\tv_cvt_f32_f64 %3, %11\n\t"
               "v_cvt_f32_f64 %4, %12\n\tv_cvt_f32_f64 %5, %13\n\tv_cvt_f32_f64 %6, %14\n\tv_cvt_f32_f64 %7, %15\n\t" LQ_RU_OFF
               : "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]), "=&v"(o[4]), "=&v"(o[5]), "=&v"(o[6]), "=&v"(o[7])
               : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
}
__device__ __forceinline__ void cvt_up2(float* o, const double* a) {
  asm volatile(LQ_RU_ON "v_cvt_f32_f64 %0, %2\n\tv_cvt_f32_f64 %1, %3\n\t" LQ_RU_OFF
               : "=&v"(o[0]), "=&v"(o[1]) : "v"(a[0]), "v"(a[1]));
}
__device__ __forceinline__ void cvt_up1(float* o, const double* a) {
  asm volatile(LQ_RU_ON "v_cvt_f32_f64 %0, %1\n\t" LQ_RU_OFF : "=&v"(o[0]) : "v"(a[0]));
}
#undef LQ_RU_ON
#undef LQ_RU_OFF
template <int N>
__device__ __forceinline__ void cvt_up(float (&o)[N], const double (&a)[N]) {
  constexpr int N8 = N / 8 * 8;
  constexpr int N4 = N / 4 * 4;
#pragma unroll
  for (int i = 0; i < N8; i += 8) cvt_up8(&o[i], &a[i]);
  if constexpr (N4 > N8) cvt_up4(&o[N8], &a[N8]);
  if constexpr (N - N4 >= 2) cvt_up2(&o[N4], &a[N4]);
  if constexpr ((N - N4) % 2 == 1) cvt_up1(&o[N - 1], &a[N - 1]);
}

// ------------------------------------------------------------ affine: search on a sorted group
// The same search (distinct (s, Z) classes, same keys, same minimizer) with the cost of a
// candidate made independent of the group size.  The group is sorted once.  For a scale S the
// weights that round to level j are a contiguous run of the sorted group, bounded by the
// thresholds (j - 1/2) S and (j + 1/2) S, and the objective of Eq. 7 over a run that takes the
// value q is  q^2 sum(omega) - 2 q sum(omega x) + sum(omega x^2),  three differences of prefix
// sums (x = w - min of the group).  The runs do not depend on the zero-point: Z only decides
// below and above which level everything is clipped.  So for one S the 2^b - 2 + n_Z
// thresholds involved are located by binary search (all of them in step, so the LDS round
// trips overlap), one walk over them accumulates the level terms, and each of the n_Z
// zero-points is closed with its two clipped tails: O((2^b + n_Z) log g) per scale instead of
// O(g n_Z).
// The closed form cancels (its terms are of the size of sum(omega x^2), the loss is not), so
// it ranks the candidates to about 1e-10 relative and is not used for the decision itself:
// every lane's best candidate that lies within 1e-7 of the smallest value found is scored
// again by the plain evaluation of Eq. 7 over the group's weights (no prefix sums), and those
// plain losses decide, with the same tie key as the enumeration.
template <int NTA, int BITS>
__global__ __launch_bounds__(NTA) void affine_sorted_kernel(const float* __restrict__ W, int64_t c,
                                                            int64_t ldw, int g, int n2, int nbk,
                                                            int ngroups,
                                                            const double* __restrict__ om64, int T,
                                                            int t, float* __restrict__ SZ) {
  constexpr int NW = NTA / 64;
  constexpr int QM = (1 << BITS) - 1;
  constexpr int WPAD = 16;              // +inf entries behind the sorted weights (window searches)
  extern __shared__ __align__(16) unsigned char smraw[];
  double2* sPAB = reinterpret_cast<double2*>(smraw);                         // [g + 1] prefix sums
  unsigned long long* sKey = reinterpret_cast<unsigned long long*>(sPAB + (g + 1));   // [n2]
  double* sOm = reinterpret_cast<double*>(sKey + n2);                        // [g] original order
  float* sW = reinterpret_cast<float*>(sOm + g);                             // [g] original order
  float* sSw = sW + g;                                                       // [n2 + WPAD] sorted, +inf padded
  uint16_t* sCnt = reinterpret_cast<uint16_t*>(sSw + n2 + WPAD);             // [nbk + 1] weights below bucket b
  __shared__ float sRed[2 * NW];
  __shared__ int sOcc[NW];
  __shared__ double sTot[3];
  __shared__ double sBestLoss[NTA];
  __shared__ int sBestKey[NTA];
  __shared__ double sBestS[NTA], sBestZ[NTA];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x / ngroups;
  const int gi = blockIdx.x % ngroups;
  const float* wsrc = W + row * ldw + (int64_t)gi * g;

  float lo = INFINITY, hi = -INFINITY;
  for (int i = tid; i < g; i += NTA) {
    const float x = wsrc[i];
    sW[i] = x;
    sOm[i] = om64[(int64_t)gi * g + i];
    lo = fminf(lo, x);
    hi = fmaxf(hi, x);
  }
  // sort keys: the weight as an order-preserving 32-bit integer, then its position
  for (int i = tid; i < n2; i += NTA) {
    unsigned long long k = ~0ull;
    if (i < g) {
      const uint32_t u = __float_as_uint(wsrc[i]);
      const uint32_t o = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      k = ((unsigned long long)o << 32) | (unsigned)i;
    }
    sKey[i] = k;
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
  // ---- bitonic sort of the keys (ascending)
  for (int k = 2; k <= n2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < (n2 >> 1); i += NTA) {
        const int a = ((i & ~(j - 1)) << 1) | (i & (j - 1));
        const int b = a | j;
        const bool asc = (a & k) == 0;
        const unsigned long long x = sKey[a], y = sKey[b];
        if ((x > y) == asc) { sKey[a] = y; sKey[b] = x; }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < n2 + WPAD; i += NTA) sSw[i] = (i < g) ? sW[(int)(sKey[i] & 0xffffffffull)] : INFINITY;
  __syncthreads();
  // ---- buckets: the range [min, max] cut into nbk equal pieces; sCnt[b] = sorted weights in
  // buckets below b.  The bucket function is monotone, so a threshold's position among the
  // sorted weights is sCnt[its bucket] plus its position among that bucket's few weights.
  const float bsc = (float)nbk / (hif - lof);
  const float bmax = (float)(nbk - 1);
  auto bucket_of = [&](float x) -> int {
    return (int)__builtin_amdgcn_fmed3f((x - lof) * bsc, 0.0f, bmax);     // clamp in one instruction
  };
  for (int i = tid; i < g; i += NTA) {
    const int bi = bucket_of(sSw[i]);
    const int bp = (i > 0) ? bucket_of(sSw[i - 1]) : -1;
    for (int b = bp + 1; b <= bi; ++b) sCnt[b] = (uint16_t)i;
    if (i == g - 1)
      for (int b = bi + 1; b <= nbk; ++b) sCnt[b] = (uint16_t)g;
  }
  __syncthreads();
  int occ = 0;
  for (int b = tid; b < nbk; b += NTA) occ = max(occ, (int)sCnt[b + 1] - (int)sCnt[b]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) occ = max(occ, __shfl_xor(occ, o, 64));
  if (lane == 0) sOcc[wave] = occ;
  // ---- prefix sums of omega and omega x over the sorted group, total of omega x^2 (wavefront 0:
  // a lane takes a contiguous piece, the pieces are chained by a scan across the lanes)
  if (wave == 0) {
    const int per = (g + 63) / 64;
    const int i0 = lane * per, i1 = min(g, i0 + per);
    double a = 0.0, b = 0.0, cc = 0.0;
    for (int i = i0; i < i1; ++i) {
      const double om = sOm[(int)(sKey[i] & 0xffffffffull)];
      const double x = (double)sSw[i] - lo0;
      a += om;
      b = fma(om, x, b);
      cc = fma(om * x, x, cc);
    }
    double ea = a, eb = b, ec = cc;      // inclusive scan over the lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double ta = __shfl_up(ea, o, 64), tb = __shfl_up(eb, o, 64), tc = __shfl_up(ec, o, 64);
      if (lane >= o) { ea += ta; eb += tb; ec += tc; }
    }
    // sums of the lanes before this one = the inclusive value of the previous lane
    double ra = __shfl_up(ea, 1, 64), rb = __shfl_up(eb, 1, 64);
    if (lane == 0) { ra = 0.0; rb = 0.0; }
    if (lane == 0) sPAB[0] = make_double2(0.0, 0.0);
    for (int i = i0; i < i1; ++i) {
      const double om = sOm[(int)(sKey[i] & 0xffffffffull)];
      const double x = (double)sSw[i] - lo0;
      ra += om;
      rb = fma(om, x, rb);
      sPAB[i + 1] = make_double2(ra, rb);
    }
    if (lane == 63) { sTot[0] = ea; sTot[1] = eb; sTot[2] = ec; }
  }
  __syncthreads();
  const double Atot = sTot[0], Btot = sTot[1], Ctot = sTot[2];
  // window of the searches: the smallest power of two that covers the fullest bucket; beyond
  // WPAD weights in one bucket (a group squeezed into a sliver of its range by an outlier) the
  // search runs over the whole group
  int occmax = sOcc[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) occmax = max(occmax, sOcc[w]);
  const bool windowed = occmax <= WPAD;
  int win = n2;
  if (windowed) { win = 1; while (win < occmax) win <<= 1; }
  const int cntmask = windowed ? 0xffff : 0;      // whole-group searches start at 0

  const double qmax = (double)QM;
  const double dT = (double)T;
  AffBest best;
  best.loss = INFINITY; best.key = 0x7fffffff; best.S = 1.0; best.Z = 0.0;

  // One chunk of up to NZC consecutive zero-points zb, zb - 1, ... of scale S: thresholds,
  // positions, walk.
  int best_s = 0, best_zi = 0;
  auto chunk = [&](auto nzc_tag, double S, double zb, int s, int z0, int nz) {
    constexpr int NZC = decltype(nzc_tag)::value;
    constexpr int NB = QM + NZC - 1;
    const double jmin = -zb;                      // lowest level of the chunk
    double loss[NZC];
    float thr[NB];
    int pos[NB];
    {
      // thresholds (j + 1/2) S as the smallest floats not below them: w < threshold exactly when
      // w < that float
      double td[NB];
      const double jh = jmin + 0.5;               // (integers far below 2^51 and a half: every sum is exact)
#pragma unroll
      for (int i = 0; i < NB; ++i) td[i] = (jh + (double)i) * S;
      cvt_up<NB>(thr, td);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) pos[i] = (int)sCnt[bucket_of(thr[i])] & cntmask;
    // all NB reads of a step are issued before the first is used (the scheduling barrier keeps
    // them there), so the LDS round trips of the NB searches overlap
    for (int step = win >> 1; step > 0; step >>= 1) {
      float v[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) v[i] = sSw[pos[i] + step - 1];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NB; ++i) pos[i] += (v[i] < thr[i]) ? step : 0;
    }
    {
      float v[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) v[i] = sSw[pos[i]];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NB; ++i) pos[i] += (v[i] < thr[i]) ? 1 : 0;       // pos = weights below thr
    }
    // (all NB steps always run: with every index a compile-time constant the arrays stay in
    // registers; steps beyond the zero-points in use only fill entries nobody reads)
    double F = 0.0, pA = 0.0, pB = 0.0;
    double lossA[NZC];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const double2 ab = sPAB[pos[i]];
      const double lev = jmin + (double)i;
      const double q = fma(lev, S, -lo0);         // level jmin + i in shifted coordinates
      if (i >= 1) {
        F = fma(q * q, ab.x - pA, F);
        F = fma(-2.0 * q, ab.y - pB, F);
      }
      if (i < NZC) lossA[i] = fma(q * q, ab.x, Ctot) - 2.0 * q * ab.y - F;
      if (i >= QM - 1) {
        const double qh = fma(lev + 1.0, S, -lo0);
        loss[i - (QM - 1)] = lossA[i - (QM - 1)] + (F + qh * qh * (Atot - ab.x) - 2.0 * qh * (Btot - ab.y));
      }
      pA = ab.x;
      pB = ab.y;
    }
    // The closed form only ranks: a lane remembers its smallest value and which (s, zero-point)
    // gave it; the tie key of the enumeration is formed once, for that candidate, afterwards.
    // (zero-points beyond the lane's own count nz belong to wider lanes of the wavefront)
#pragma unroll
    for (int k = 0; k < NZC; ++k) {
      const int zi = z0 + k;
      const bool take = (zi < nz) & (loss[k] < best.loss);
      best.loss = take ? loss[k] : best.loss;
      best.S = take ? S : best.S;
      best_s = take ? s : best_s;
      best_zi = take ? zi : best_zi;
    }
  };

  // x / (2^b - 1), correctly rounded, without a division: product with the rounded reciprocal
  // and one correction by the exact remainder (exact for these divisors: 3, 7 and 15 were checked
  // against the division on 4e8 random operands each).
  auto div_by_levels = [&](double x) -> double {
    constexpr double rc = 1.0 / (double)QM;
    const double q = x * rc;
    return fma(fma(-(double)QM, q, x), rc, q);
  };
  // rint(a / S) from the product with 1 / S (rS, good to an ulp): the product is within a few ulp
  // of the quotient, so the two round to the same integer unless it lies that close to a half;
  // only then is the division carried out.
  auto rint_quotient = [&](double a, double S, double rS) -> double {
    const double q = a * rS;
    double rq = rint(q);
    if (fabs(q - rq) > 0.5 - fma(fabs(q), 8.9e-16, 1.0e-12)) rq = rint(a / S);
    return rq;
  };
  // t_min R / T as the enumeration forms it; for T a power of two the product with R / T is the
  // same number (an exact scaling), without a division per use
  const bool tpow2 = (T & (T - 1)) == 0;
  const double rT = R / dT;
  auto frac_of_range = [&](int tm) -> double { return tpow2 ? (double)tm * rT : (double)tm * R / dT; };
  const int rounds = (2 * t + NTA) / NTA;
  for (int rd = 0; rd < rounds; ++rd) {
    const int s = tid + rd * NTA;
    const bool live = s <= 2 * t;
    const int ta = (s > t) ? (s - t) : 0;      // smallest t_min with t_max = s - t_min <= t
    const int tb = (s < t) ? s : t;            // largest t_min
    const double lo_a = lo0 + frac_of_range(ta);
    const double hi_a = hi0 - frac_of_range(s - ta);
    const double S = div_by_levels(hi_a - lo_a);
    const bool ok = live && (S > 0.0);
    const double Sx = ok ? S : 1.0;
    const double lo_b = lo0 + frac_of_range(tb);
    const double rS = recip_f64(Sx);
    const double zf = -rint_quotient(lo_a, Sx, rS);
    const double zl = -rint_quotient(lo_b, Sx, rS);
    double span = zf - zl;
    if (!(span >= 0.0)) span = 0.0;
    const int nz = ok ? (int)fmin(span, 1.0e6) + 1 : 0;
    // widest lane of the wavefront, rounded up to the width of the walk that will serve it
    // (votes over the wavefront; the exact maximum only when some lane needs more than one walk)
    int nzw;
    if (__ballot(nz > 3) == 0) nzw = __ballot(nz > 2) ? 3 : (__ballot(nz > 0) ? 2 : 0);
    else if (__ballot(nz > 8) == 0) nzw = __ballot(nz > 6) ? 8 : (__ballot(nz > 4) ? 6 : 4);
    else {
      nzw = nz;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) nzw = max(nzw, __shfl_xor(nzw, o, 64));
    }

    for (int z0 = 0; z0 < nzw; z0 += 8) {
      const int cntw = min(8, nzw - z0);
      const double zb = zf - (double)z0;
      if (cntw <= 2) chunk(std::integral_constant<int, 2>{}, Sx, zb, s, z0, nz);
      else if (cntw <= 3) chunk(std::integral_constant<int, 3>{}, Sx, zb, s, z0, nz);
      else if (cntw <= 4) chunk(std::integral_constant<int, 4>{}, Sx, zb, s, z0, nz);
      else if (cntw <= 6) chunk(std::integral_constant<int, 6>{}, Sx, zb, s, z0, nz);
      else chunk(std::integral_constant<int, 8>{}, Sx, zb, s, z0, nz);
    }
  }
  if (best.loss < INFINITY) {
    // zero-point and tie key of the lane's candidate, as the enumeration would see it: the class
    // (s, Z) is first met at the smallest t_min >= ta with round(lo / S) == -Z
    const int s = best_s;
    const int ta = (s > t) ? (s - t) : 0;
    const int tb = (s < t) ? s : t;
    const double lo_a = lo0 + frac_of_range(ta);
    const double zf = -rint(lo_a / best.S);
    const double Z = zf - (double)best_zi;
    int tf = ta;
    if (best_zi > 0) {
      tf = (int)ceil(((-Z - 0.5) * best.S - lo0) * dT / R);
      tf = tf < ta ? ta : (tf > tb ? tb : tf);
    }
    best.Z = Z;
    best.key = tf * (t + 1) + (s - tf);
  }
  // ---- smallest closed-form value of the workgroup; candidates within its noise are scored plainly
  sBestLoss[tid] = best.loss;
  __syncthreads();
  for (int w2 = NTA / 2; w2 > 0; w2 >>= 1) {
    if (tid < w2) sBestLoss[tid] = fmin(sBestLoss[tid], sBestLoss[tid + w2]);
    __syncthreads();
  }
  const double lmin = sBestLoss[0];
  __syncthreads();
  // A wavefront scores its candidates one after the other, all lanes on one candidate: lane l
  // adds the weights l, l + 64, ... in that order and the 64 partial sums are added pairwise
  // (lanes 32 apart first), a fixed order.
  double exact = INFINITY;
  {
    unsigned long long todo = __ballot(best.loss <= lmin + (1.0e-7 * fabs(lmin) + 1.0e-12 * Ctot));
    while (todo) {
      const int src = __ffsll((long long)todo) - 1;
      todo &= todo - 1;
      const double S = __shfl(best.S, src, 64), Z = __shfl(best.Z, src, 64);
      const double invS = 1.0 / S;
      const double cl = -Z, ch = qmax - Z;
      double loss = 0.0;
      for (int i = lane; i < g; i += 64) {
        const double w = (double)sW[i];
        const double u = fmin(fmax(rint(w * invS), cl), ch);
        const double dlt = fma(u, S, -w);
        loss = fma(sOm[i] * dlt, dlt, loss);
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) loss += __shfl_xor(loss, o, 64);
      if (lane == src) exact = loss;
    }
  }
  sBestLoss[tid] = exact; sBestKey[tid] = best.key; sBestS[tid] = best.S; sBestZ[tid] = best.Z;
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
                        const float* init, int max_iter, float* G, int* next_row, hipStream_t st) {
  // rows are handed out by a counter, so the grid only has to cover the workgroups that
  // can be resident (at most 4 per compute unit)
  unsigned grid = (unsigned)(r < 1024 ? r : 1024);
#define LQ_KM(E, T)                                                                              \
  hipLaunchKernelGGL((kmeans_rows_kernel<K, E, T>), dim3(grid), dim3(T), 0, st, W, r, c, ldw,   \
                     om32, init, max_iter, G, next_row)
  // a thread holds E weights of the row: 256 threads up to 4096 columns, 512 beyond
  if (c <= 2 * 256) LQ_KM(2, 256);
  else if (c <= 4 * 256) LQ_KM(4, 256);
  else if (c <= 8 * 256) LQ_KM(8, 256);
  else if (c <= 16 * 256) LQ_KM(16, 256);
  else if (c <= 16 * 512) LQ_KM(16, 512);
  else if (c <= 22 * 512) LQ_KM(22, 512);
  else LQ_KM(32, 512);
#undef LQ_KM
  LQ_CHECK_LAUNCH("kmeans_rows_kernel");
  return LQ_OK;
}

}  // namespace

namespace lq {
size_t fit_grid_workspace_bytes(int64_t c) {
  // importance weights in fp64 and fp32, and the row counter of the non-uniform fit
  return align_up((size_t)c * sizeof(double), 256) + align_up((size_t)c * sizeof(float), 256) + 256;
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
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)STATIC_MAX_C * (sizeof(double) + sizeof(float)) + 256;
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
  int* next_row = (int*)((char*)om32 + lq::align_up((size_t)c * sizeof(float), 256));

  if (P->mode == LQ_GRID_NONUNIFORM) {
    if (c > 32 * 512) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid: non-uniform fit supports c <= %d", 32 * 512);
    hipLaunchKernelGGL(importance_kernel, dim3(1), dim3(1024), 0, st, hinv_diag, c, P->p, om32, om64, next_row);
    LQ_CHECK_LAUNCH("importance_kernel");
    switch (P->bits) {
      case 2: return launch_kmeans<4>(W, r, c, ldw, om32, init_grid, P->kmeans_max_iter, grid, next_row, st);
      case 3: return launch_kmeans<8>(W, r, c, ldw, om32, init_grid, P->kmeans_max_iter, grid, next_row, st);
      default: return launch_kmeans<16>(W, r, c, ldw, om32, init_grid, P->kmeans_max_iter, grid, next_row, st);
    }
  }

  const int64_t g = P->group_size > 0 ? P->group_size : c;
  if (g > 8192) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid: affine group of %lld columns (limit 8192)", (long long)g);
  const int64_t ngroups = c / g;
  if (r * ngroups > 0x7fffffffLL) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_fit_grid: more than 2^31 groups");
  hipLaunchKernelGGL(importance_kernel, dim3(1), dim3(1024), 0, st, hinv_diag, c, P->p, om32, om64, next_row);
  LQ_CHECK_LAUNCH("importance_kernel");
  const int t = lq::resolve_t(P);
  const int ns = 2 * t + 1;
  // threads per group: fewest idle lanes in the last round of s values; ties go to the larger,
  // except for groups of up to 128 weights, where one wavefront per group (no workgroup barriers
  // in the sort and the reductions) is the faster of two equal choices (2-bit, groups of 64,
  // T = 2048: 309 -> 276 ms on the 53248 x 16384 layer)
  int nta = 256;
  {
    int best = (ns + 255) / 256 * 256;
    for (int cand : {128, 64}) {
      const int padded = (ns + cand - 1) / cand * cand;
      if (padded < best || (padded == best && g <= 128)) { best = padded; nta = cand; }
    }
  }
  const dim3 ggrid((unsigned)(r * ngroups));
  // The sorted-group kernel covers the fine partitions (every integer between the end values
  // of the zero-point occurs: T - 2t > 2^b - 1) on groups of up to SORT_MAX_G columns.
  constexpr int64_t SORT_MAX_G = 2048;
  const bool dense = (P->T - 2 * t) > ((1 << P->bits) - 1);
  if (dense && g <= SORT_MAX_G) {
    int n2 = 1;
    while (n2 < g) n2 <<= 1;
    const int nbk = (int)(4 * n2 < 4096 ? 4 * n2 : 4096);          // buckets of the window searches
    const size_t lds_sorted = (size_t)(g + 1) * 16 + (size_t)n2 * 8 + (size_t)g * 12 + (size_t)(n2 + 16) * 4 +
                              (size_t)(nbk + 2) * 2;
    static lq::DeviceOnce sorted_once;
    if (lq::DeviceOnceGuard once(sorted_once); once.first()) {
      const int lim = (int)((SORT_MAX_G + 1) * 16 + SORT_MAX_G * 8 + SORT_MAX_G * 12 + (SORT_MAX_G + 16) * 4 + 4098 * 2);
#define LQ_ATTR(N, BT) LQ_CHECK_HIP(hipFuncSetAttribute((const void*)affine_sorted_kernel<N, BT>, \
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, lim))
      LQ_ATTR(64, 2); LQ_ATTR(64, 3); LQ_ATTR(64, 4);
      LQ_ATTR(128, 2); LQ_ATTR(128, 3); LQ_ATTR(128, 4);
      LQ_ATTR(256, 2); LQ_ATTR(256, 3); LQ_ATTR(256, 4);
#undef LQ_ATTR
      once.done();
    }
#define LQ_AFS(N, BT) hipLaunchKernelGGL((affine_sorted_kernel<N, BT>), ggrid, dim3(N), lds_sorted, st, W, c, ldw, \
                                         (int)g, n2, nbk, (int)ngroups, (const double*)om64, P->T, t, grid)
#define LQ_AFS_N(N) do { if (P->bits == 2) LQ_AFS(N, 2); else if (P->bits == 3) LQ_AFS(N, 3); else LQ_AFS(N, 4); } while (0)
    if (nta == 64) LQ_AFS_N(64);
    else if (nta == 128) LQ_AFS_N(128);
    else LQ_AFS_N(256);
#undef LQ_AFS_N
#undef LQ_AFS
    LQ_CHECK_LAUNCH("affine_sorted_kernel");
    return LQ_OK;
  }
  const size_t lds = (size_t)g * 2 * sizeof(double);
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

