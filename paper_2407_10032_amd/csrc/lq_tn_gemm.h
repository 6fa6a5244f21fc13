// C (+)= alpha * P^T Q on fp32 MFMA, with P [K x M] and Q [K x N] both k-major
// (row index = contraction index), the shape shared by the two dense
// contractions of Algorithm 1:
//   line 3   H += 2 X^T X            P = Q = X (tokens x channels), symmetric
//   line 19  W[:, i+B:] -= E U[...]  P = E^T stored as [B x r], Q = rows i..i+B of U
//
// A workgroup computes one 128 x 128 tile of C over a slice of the contraction
// range.  Global loads of the next k-chunk are issued into registers before
// the MFMAs of the current one and written to the other LDS buffer afterwards
// (one barrier per chunk).  In symmetric mode only tiles on or above the
// diagonal are computed; with a token split each slice writes a partial tile
// that a second kernel sums in a fixed order and mirrors.
#pragma once

#include "lq_mfma.h"

namespace lq {

struct TnGemmArgs {
  const float* P; int64_t ldp;
  const float* Q; int64_t ldq;
  float* C; int64_t ldc;
  int64_t M, N, K;
  float alpha;
  int tiles_m, tiles_n;
  int ntiles;           // tiles per split (upper-triangle count in symmetric mode)
  int splits;
  int64_t k_per_split;  // multiple of the k-chunk
  float* partial;       // [splits][ntiles][128*128] when PARTIAL
};

// Upper-triangle tile enumeration, row by row: index -> (bi, bj), bj >= bi.
__device__ __forceinline__ void decode_upper(int idx, int T, int& bi, int& bj) {
  float tf = 2.0f * T + 1.0f;
  int r = (int)((tf - sqrtf(tf * tf - 8.0f * (float)idx)) * 0.5f);
  if (r < 0) r = 0;
  if (r > T - 1) r = T - 1;
  // start(r) = r*T - r*(r-1)/2
  while (r > 0 && r * T - (r * (r - 1)) / 2 > idx) --r;
  while (r + 1 < T && (r + 1) * T - ((r + 1) * r) / 2 <= idx) ++r;
  bi = r;
  bj = r + (idx - (r * T - (r * (r - 1)) / 2));
}

// Tiles are handed out patch by patch (PATCH x PATCH tiles) so that workgroups that run at
// the same time on one XCD read few distinct operand panels and find them in that XCD's L2.
constexpr int PATCH = 8;
constexpr int XCDS = 8;          // workgroup ids go round-robin over the 8 XCDs
constexpr int XCD_CHUNK = 64;    // consecutive work items given to one XCD

// blockIdx -> work item: each XCD gets runs of XCD_CHUNK consecutive work items.
__device__ __forceinline__ int xcd_swizzle(int b, int total) {
  const int group = XCDS * XCD_CHUNK;
  const int full = (total / group) * group;
  if (b >= full) return b;
  const int xcd = b % XCDS, slot = b / XCDS;
  return (slot / XCD_CHUNK) * group + xcd * XCD_CHUNK + (slot % XCD_CHUNK);
}

// Patch-major enumeration of a tiles_m x tiles_n grid (general) or of the tiles strictly above
// the diagonal of a square grid (SYM, tiles_m == tiles_n): index -> (bi, bj).  Walks the
// patches in row-major order.
template <bool SYM>
__device__ __forceinline__ void decode_patch_major(int idx, int tiles_m, int tiles_n, int& bi, int& bj) {
  const int pm = (tiles_m + PATCH - 1) / PATCH, pn = (tiles_n + PATCH - 1) / PATCH;
  for (int pi = 0; pi < pm; ++pi) {
    const int h = min(PATCH, tiles_m - pi * PATCH);
    for (int pj = SYM ? pi : 0; pj < pn; ++pj) {
      const int w = min(PATCH, tiles_n - pj * PATCH);
      const int cnt = (SYM && pi == pj) ? h * (h - 1) / 2 : h * w;
      if (idx < cnt) {
        int li, lj;
        if (SYM && pi == pj) {
          decode_upper(idx, h - 1, li, lj);   // strictly upper of h x h = upper with diagonal of (h - 1) x (h - 1), shifted
          lj += 1;
        } else {
          li = idx / w;
          lj = idx - li * w;
        }
        bi = pi * PATCH + li;
        bj = pj * PATCH + lj;
        return;
      }
      idx -= cnt;
    }
  }
  bi = 0; bj = 0;  // not reached for idx < number of tiles
}

// Tile ids of a symmetric product with T x T tiles: the T (T - 1) / 2 tiles above the diagonal
// in patch-major order, then the T diagonal tiles.
__device__ __forceinline__ void decode_sym_tile(int tile, int T, int& bi, int& bj) {
  const int above = T * (T - 1) / 2;
  if (tile >= above) { bi = bj = tile - above; return; }
  decode_patch_major<true>(tile, T, T, bi, bj);
}

// One k-chunk (KT rows x 128 columns) of an operand in registers: KT / 8 float4 per thread,
// held as named members so that they stay in registers.
template <int KT> struct ChunkRegs;
template <> struct ChunkRegs<16> { float4 r0, r1; };
template <> struct ChunkRegs<32> { float4 r0, r1, r2, r3; };

// Element-wise guarded load of one float4 (rows past kend / columns past ncols read zero).
template <bool VEC>
__device__ __forceinline__ float4 tn_load_guarded(const float* __restrict__ base, int64_t ld,
                                                  int64_t k, int64_t kend, int64_t col,
                                                  int64_t ncols) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (k < kend) {
    const float* src = base + k * ld + col;
    if (VEC && col + 3 < ncols) {
      v = *reinterpret_cast<const float4*>(src);
    } else {
      if (col + 0 < ncols) v.x = src[0];
      if (col + 1 < ncols) v.y = src[1];
      if (col + 2 < ncols) v.z = src[2];
      if (col + 3 < ncols) v.w = src[3];
    }
  }
  return v;
}

// One guarded k-chunk of an operand: rows past kend and columns past ncols read as zero.
template <int KT, bool VEC>
__device__ __forceinline__ ChunkRegs<KT> tn_load_chunk(const float* __restrict__ base, int64_t ld,
                                                       int64_t k0, int64_t kend, int64_t col0,
                                                       int64_t ncols, int tid) {
  ChunkRegs<KT> c;
  const int64_t k = k0 + (tid >> 5);
  const int64_t col = col0 + 4 * (tid & 31);
  c.r0 = tn_load_guarded<VEC>(base, ld, k, kend, col, ncols);
  c.r1 = tn_load_guarded<VEC>(base, ld, k + 8, kend, col, ncols);
  if constexpr (KT == 32) {
    c.r2 = tn_load_guarded<VEC>(base, ld, k + 16, kend, col, ncols);
    c.r3 = tn_load_guarded<VEC>(base, ld, k + 24, kend, col, ncols);
  }
  return c;
}

template <int KT>
__device__ __forceinline__ void tn_store_chunk(float* __restrict__ s, const ChunkRegs<KT>& c, int tid) {
  float* d = s + (tid >> 5) * TILE + 4 * (tid & 31);
  *reinterpret_cast<float4*>(d) = c.r0;
  *reinterpret_cast<float4*>(d + 8 * TILE) = c.r1;
  if constexpr (KT == 32) {
    *reinterpret_cast<float4*>(d + 16 * TILE) = c.r2;
    *reinterpret_cast<float4*>(d + 24 * TILE) = c.r3;
  }
}

// The k loop of one tile, guarded variant (edge tiles, unaligned operands, ragged slices):
// global loads of stage s+1 are issued before the MFMAs of stage s and stored to the other
// LDS buffer after them.
template <int KT, bool VEC>
__device__ __forceinline__ void tn_mainloop_safe(const TnGemmArgs& a, float* smem, int64_t kbeg,
                                                 int64_t kend, int64_t m0, int64_t n0, bool diag,
                                                 int wm, int wn, int lane, int tid, Acc2x2& acc) {
  constexpr int STAGE = KT * TILE;
  ChunkRegs<KT> rp = tn_load_chunk<KT, VEC>(a.P, a.ldp, kbeg, kend, m0, a.M, tid);
  ChunkRegs<KT> rq = rp;
  if (!diag) rq = tn_load_chunk<KT, VEC>(a.Q, a.ldq, kbeg, kend, n0, a.N, tid);
  tn_store_chunk<KT>(smem, rp, tid);
  if (!diag) tn_store_chunk<KT>(smem + 2 * STAGE, rq, tid);
  __syncthreads();
  int buf = 0;
  for (int64_t k0 = kbeg; k0 < kend; k0 += KT) {
    const bool more = (k0 + KT) < kend;
    if (more) {
      rp = tn_load_chunk<KT, VEC>(a.P, a.ldp, k0 + KT, kend, m0, a.M, tid);
      if (!diag) rq = tn_load_chunk<KT, VEC>(a.Q, a.ldq, k0 + KT, kend, n0, a.N, tid);
    }
    const float* cp = smem + buf * STAGE;
    mma_chunk_kmajor<KT>(cp, diag ? cp : cp + 2 * STAGE, wm, wn, lane, acc);
    if (more) {
      float* np = smem + (buf ^ 1) * STAGE;
      tn_store_chunk<KT>(np, rp, tid);
      if (!diag) tn_store_chunk<KT>(np + 2 * STAGE, rq, tid);
    }
    __syncthreads();
    buf ^= 1;
  }
}

struct TnOperands { float a0[2], a1[2], b0[2], b1[2]; };

// Addresses one thread uses in one LDS buffer of the fast loop: where its wave reads the
// A and B operands of k-step 0 and where the thread stores its part of a stage (P operand;
// the Q operand sits 2 * KT * TILE floats further).
struct TnLdsAddr { const float* p; const float* q; float* st; };

// Global source of one operand for the fast loop: a wave-uniform row base (kept in scalar
// registers) plus this thread's byte offsets of its KT / 8 rows, so that a stage's loads
// need no vector-ALU address arithmetic.
template <int KT> struct TnFastSrc {
  typedef const __attribute__((address_space(1))) char* GlobalBytes;   // global_load, not flat_load
  typedef float Vec4 __attribute__((ext_vector_type(4)));
  typedef const __attribute__((address_space(1))) Vec4* GlobalVec4;
  GlobalBytes base;
  unsigned off[KT / 8];
  int64_t step;                                  // bytes per stage
  __device__ __forceinline__ void init(const float* src, int64_t ld, int64_t k0, int64_t col0, int tid) {
    const uint64_t v = reinterpret_cast<uint64_t>(src + k0 * ld + col0);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    base = (GlobalBytes)(((uint64_t)hi << 32) | lo);
#pragma unroll
    for (int i = 0; i < KT / 8; ++i)
      off[i] = (unsigned)(((tid >> 5) + 8 * i) * (int)ld + 4 * (tid & 31)) * 4u;
    step = (int64_t)KT * ld * 4;
  }
  // The empty asm keeps the 32-bit offset opaque at the point of use, so that its zero
  // extension is not hoisted out of the loop and instruction selection sees
  // "scalar base + 32-bit vector offset" (global_load with an SGPR base, no 64-bit add).
  __device__ __forceinline__ Vec4 load_one(int i) const {
    unsigned o = off[i];
    asm volatile("" : "+v"(o));
    return *(GlobalVec4)(base + o);
  }
  __device__ __forceinline__ ChunkRegs<KT> load() const {
    ChunkRegs<KT> c;
    const Vec4 v0 = load_one(0);
    const Vec4 v1 = load_one(1);
    c.r0 = make_float4(v0.x, v0.y, v0.z, v0.w);
    c.r1 = make_float4(v1.x, v1.y, v1.z, v1.w);
    if constexpr (KT == 32) {
      const Vec4 v2 = load_one(2);
      const Vec4 v3 = load_one(3);
      c.r2 = make_float4(v2.x, v2.y, v2.z, v2.w);
      c.r3 = make_float4(v3.x, v3.y, v3.z, v3.w);
    }
    return c;
  }
  __device__ __forceinline__ void next() { base += step; }
};

template <int KT>
__device__ __forceinline__ void tn_store_chunk_at(float* __restrict__ d, const ChunkRegs<KT>& c) {
  *reinterpret_cast<float4*>(d) = c.r0;
  *reinterpret_cast<float4*>(d + 8 * TILE) = c.r1;
  if constexpr (KT == 32) {
    *reinterpret_cast<float4*>(d + 16 * TILE) = c.r2;
    *reinterpret_cast<float4*>(d + 24 * TILE) = c.r3;
  }
}

// One k stage of tn_mainloop_fast over buffer `cur`.  On entry o.*[0] holds the operands
// of k-step 0 of this stage; if MORE, on exit it holds those of k-step 0 of the next
// stage, whose data (rp, rq) this stage stores to buffer `nxt`.  MASK: which of the wave's four
// sub-tiles are computed (bit 2 tm + tn); operands that no computed sub-tile uses are not read.
template <int KT, bool MORE, bool DIAG, int MASK>
__device__ __forceinline__ void tn_fast_stage(const TnLdsAddr& cur, const TnLdsAddr& nxt,
                                              const ChunkRegs<KT>& rp, const ChunkRegs<KT>& rq,
                                              TnOperands& o, Acc2x2& acc) {
  constexpr int STAGE = KT * TILE;
  constexpr int STEPS = KT / 2;
  constexpr int STORE_AT = STEPS - 4;     // k-step before whose MFMAs the next stage is stored
  static_assert(STEPS % 2 == 0 && STORE_AT >= 0, "operand slots alternate per k-step");
  const float* p = cur.p;
  const float* q = cur.q;
#pragma unroll
  for (int kk = 0; kk < STEPS; ++kk) {
    const int c = kk & 1, n = c ^ 1;
    if (kk + 1 < STEPS) {
      o.a0[n] = p[2 * (kk + 1) * TILE];
      o.a1[n] = p[2 * (kk + 1) * TILE + 64];
      o.b0[n] = q[2 * (kk + 1) * TILE];
      o.b1[n] = q[2 * (kk + 1) * TILE + 64];
    }
    if (MORE && kk == STORE_AT) {
      tn_store_chunk_at<KT>(nxt.st, rp);
      if (!DIAG) tn_store_chunk_at<KT>(nxt.st + 2 * STAGE, rq);
    }
    if (MORE && kk == STEPS - 1) {
      __syncthreads();                       // stores landed, every read of this buffer issued
      o.a0[n] = nxt.p[0]; o.a1[n] = nxt.p[64];
      o.b0[n] = nxt.q[0]; o.b1[n] = nxt.q[64];
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MASK & 1) acc.t[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a0[c], o.b0[c], acc.t[0][0], 0, 0, 0);
    if constexpr (MASK & 2) acc.t[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a0[c], o.b1[c], acc.t[0][1], 0, 0, 0);
    if constexpr (MASK & 4) acc.t[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a1[c], o.b0[c], acc.t[1][0], 0, 0, 0);
    if constexpr (MASK & 8) acc.t[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.a1[c], o.b1[c], acc.t[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// The k loop of an interior tile (no predicates), written so that the MFMA pipe is the
// only vector unit the steady state uses:
//   * global loads of stage s+1 are issued at the top of stage s from a scalar base plus
//     fixed per-thread offsets;
//   * their LDS stores (into the buffer not being read) are issued a few k-steps before
//     the end of stage s, between MFMA groups;
//   * the barrier sits before the LAST MFMA group of the stage, whose operands are
//     already in registers; the first operands of stage s+1 are read right after it;
//   * all LDS addresses of both buffers are computed once, and the loop is unrolled over
//     the two buffers, so that a stage has no vector-ALU instruction at all: a VALU
//     instruction between MFMAs was measured to idle the MFMA pipe for about 16 cycles.
// Scheduling barriers pin the order.  nst = number of stages (>= 1), wave-uniform.
template <int KT, bool DIAG, int MASK>
__device__ __forceinline__ void tn_fast_loop(TnFastSrc<KT>& sp, TnFastSrc<KT>& sq, int nst,
                                             const TnLdsAddr& b0, const TnLdsAddr& b1,
                                             ChunkRegs<KT>& rp, ChunkRegs<KT>& rq, TnOperands& o,
                                             Acc2x2& acc) {
  int left = nst - 1;                            // stages that are followed by another
  while (left >= 2) {
    sp.next(); rp = sp.load();
    if (!DIAG) { sq.next(); rq = sq.load(); }
    tn_fast_stage<KT, true, DIAG, MASK>(b0, b1, rp, rq, o, acc);
    sp.next(); rp = sp.load();
    if (!DIAG) { sq.next(); rq = sq.load(); }
    tn_fast_stage<KT, true, DIAG, MASK>(b1, b0, rp, rq, o, acc);
    left -= 2;
  }
  if (left) {
    sp.next(); rp = sp.load();
    if (!DIAG) { sq.next(); rq = sq.load(); }
    tn_fast_stage<KT, true, DIAG, MASK>(b0, b1, rp, rq, o, acc);
    tn_fast_stage<KT, false, DIAG, MASK>(b1, b1, rp, rq, o, acc);
  } else {
    tn_fast_stage<KT, false, DIAG, MASK>(b0, b0, rp, rq, o, acc);
  }
}

// HALF: -1 = the whole 128 x 128 tile; 0 / 1 = only its upper / lower 64 rows (the sub-tiles
// tm = HALF of every wavefront), for launches that split a tile between two workgroups.
template <int KT, bool VEC, int HALF = -1>
__device__ __forceinline__ void tn_mainloop_fast(const TnGemmArgs& a, float* smem, int64_t kbeg,
                                                 int64_t kend, int64_t m0, int64_t n0, bool diag,
                                                 int wm, int wn, int lane, int tid, Acc2x2& acc) {
  constexpr int STAGE = KT * TILE;
  const int kl = lane >> 5, ml = lane & 31;
  const int offp = kl * TILE + wm * 32 + ml;
  const int offq = (diag ? 0 : 2 * STAGE) + kl * TILE + wn * 32 + ml;
  const int offs = (tid >> 5) * TILE + 4 * (tid & 31);
  TnLdsAddr b0, b1;
  b0.p = smem + offp;         b0.q = smem + offq;         b0.st = smem + offs;
  b1.p = smem + STAGE + offp; b1.q = smem + STAGE + offq; b1.st = smem + STAGE + offs;
  const int nst = __builtin_amdgcn_readfirstlane((int)((kend - kbeg) / KT));

  TnFastSrc<KT> sp, sq;
  sp.init(a.P, a.ldp, kbeg, m0, tid);
  sq.init(a.Q, a.ldq, kbeg, n0, tid);
  ChunkRegs<KT> rp = sp.load();
  ChunkRegs<KT> rq = rp;
  if (!diag) rq = sq.load();
  tn_store_chunk_at<KT>(b0.st, rp);
  if (!diag) tn_store_chunk_at<KT>(b0.st + 2 * STAGE, rq);
  __syncthreads();

  TnOperands o;
  o.a0[0] = b0.p[0]; o.a1[0] = b0.p[64];
  o.b0[0] = b0.q[0]; o.b1[0] = b0.q[64];
  // A diagonal tile of a symmetric product is needed on and above its own diagonal only: of
  // the 4 x 4 sub-tiles (wm + 2 tm, wn + 2 tn) the six with a row index above the column index
  // are left at zero (the reduce kernel mirrors their transposes): wavefront (1, 0) keeps
  // sub-tile (1, 2) alone, the other three drop (wm + 2, wn).
  if constexpr (HALF == 0) {
    tn_fast_loop<KT, false, 3>(sp, sq, nst, b0, b1, rp, rq, o, acc);
  } else if constexpr (HALF == 1) {
    tn_fast_loop<KT, false, 12>(sp, sq, nst, b0, b1, rp, rq, o, acc);
  } else if (diag) {
    if (wm * 2 + wn == 2) tn_fast_loop<KT, true, 2>(sp, sq, nst, b0, b1, rp, rq, o, acc);
    else tn_fast_loop<KT, true, 11>(sp, sq, nst, b0, b1, rp, rq, o, acc);
  } else {
    tn_fast_loop<KT, false, 15>(sp, sq, nst, b0, b1, rp, rq, o, acc);
  }
}

// SPLIT_TILE (general product, direct update only): the grid has two workgroups per tile and
// each computes and updates 64 of the tile's 128 rows.  Both load the whole operand stages (the
// panels come from L2), so this is for launches whose tiles would otherwise leave compute units
// idle or unevenly loaded: 2 n half-workgroups spread better over the chip than n whole ones.
template <int KT, bool SYM, bool PARTIAL, bool VEC, int MINW = 2, bool SPLIT_TILE = false>
__global__ __launch_bounds__(WG_THREADS, MINW) void tn_gemm_kernel(TnGemmArgs a) {
  static_assert(!SPLIT_TILE || (!SYM && !PARTIAL), "tiles are split for the direct general update only");
  extern __shared__ __align__(16) float smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: lives in a scalar register
  const int wm = wave >> 1, wn = wave & 1;

  int work = xcd_swizzle(blockIdx.x, a.splits * a.ntiles * (SPLIT_TILE ? 2 : 1));
  int half = 0;
  if (SPLIT_TILE) { half = work & 1; work >>= 1; }
  int split, tile, bi, bj;
  if (SYM) {
    // Diagonal tiles do less work (see tn_mainloop_fast) and finish earlier.  Workgroups that
    // share operand panels in an XCD's L2 stay together only while they take the same time,
    // so all (slice, diagonal tile) items come after all items of the tiles above the diagonal.
    const int above = a.ntiles - a.tiles_m;
    if (work < a.splits * above) {
      split = work / above;
      tile = work - split * above;
    } else {
      const int w = work - a.splits * above;
      split = w / a.tiles_m;
      tile = above + (w - split * a.tiles_m);
    }
    decode_sym_tile(tile, a.tiles_m, bi, bj);
  } else {
    split = work / a.ntiles;
    tile = work - split * a.ntiles;
    decode_patch_major<false>(tile, a.tiles_m, a.tiles_n, bi, bj);
  }
  const bool diag = SYM && (bi == bj);
  const int64_t m0 = (int64_t)bi * TILE, n0 = (int64_t)bj * TILE;
  const int64_t kbeg = (int64_t)split * a.k_per_split;
  int64_t kend = kbeg + a.k_per_split;
  if (kend > a.K) kend = a.K;

  Acc2x2 acc;
  acc.clear();

  if (kbeg < kend) {
    // interior tiles of an aligned operand whose slice is a whole number of stages take the
    // predicate-free loads; the two loops are separate so that each has one load variant
    const bool fast = VEC && (m0 + TILE <= a.M) && (n0 + TILE <= a.N) && ((kend - kbeg) % KT == 0) &&
                      a.ldp < (1 << 24) && a.ldq < (1 << 24);   // 32-bit byte offsets inside a stage
    if constexpr (SPLIT_TILE) {
      // (the guarded loop computes the whole tile; the half that is not this workgroup's is dropped)
      if (!fast) tn_mainloop_safe<KT, VEC>(a, smem, kbeg, kend, m0, n0, diag, wm, wn, lane, tid, acc);
      else if (half == 0) tn_mainloop_fast<KT, VEC, 0>(a, smem, kbeg, kend, m0, n0, diag, wm, wn, lane, tid, acc);
      else tn_mainloop_fast<KT, VEC, 1>(a, smem, kbeg, kend, m0, n0, diag, wm, wn, lane, tid, acc);
    } else {
      if (fast) tn_mainloop_fast<KT, VEC>(a, smem, kbeg, kend, m0, n0, diag, wm, wn, lane, tid, acc);
      else tn_mainloop_safe<KT, VEC>(a, smem, kbeg, kend, m0, n0, diag, wm, wn, lane, tid, acc);
    }
  }

  if constexpr (SPLIT_TILE) {
    // rows 64 * half .. 64 * half + 63 of the tile: the sub-tiles tm = half of every wavefront
    const bool direct = VEC && (m0 + TILE <= a.M) && (n0 + TILE <= a.N) && (a.ldc % 4 == 0) &&
                        ((reinterpret_cast<uintptr_t>(a.C) & 15) == 0) && (n0 % 4 == 0);
    if (direct) {
      float* cbase = a.C + (m0 + 64 * half) * a.ldc + n0;
      float4 cv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int f = tid + u * WG_THREADS;
        cv[u] = *reinterpret_cast<const float4*>(cbase + (int64_t)(f >> 5) * a.ldc + 4 * (f & 31));
      }
      __syncthreads();                             // the operand buffers are no longer read
#pragma unroll
      for (int tm = 0; tm < 2; ++tm) {
        if (tm != half) continue;
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            smem[(acc_row(wm, tm, v, lane) - 64 * tm) * TILE + acc_col(wn, tn, lane)] = a.alpha * acc.t[tm][tn][v];
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int f = tid + u * WG_THREADS;
        const float4 d = *reinterpret_cast<const float4*>(smem + (f >> 5) * TILE + 4 * (f & 31));
        cv[u].x += d.x; cv[u].y += d.y; cv[u].z += d.z; cv[u].w += d.w;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int f = tid + u * WG_THREADS;
        *reinterpret_cast<float4*>(cbase + (int64_t)(f >> 5) * a.ldc + 4 * (f & 31)) = cv[u];
      }
    } else {
#pragma unroll
      for (int tm = 0; tm < 2; ++tm) {
        if (tm != half) continue;
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int64_t row = m0 + acc_row(wm, tm, v, lane);
            const int64_t col = n0 + acc_col(wn, tn, lane);
            if (row < a.M && col < a.N) a.C[row * a.ldc + col] += a.alpha * acc.t[tm][tn][v];
          }
      }
    }
    return;
  }

  if (PARTIAL) {
    float* out = a.partial + ((int64_t)split * a.ntiles + tile) * (TILE * TILE);
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
      for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          out[acc_row(wm, tm, v, lane) * TILE + acc_col(wn, tn, lane)] = acc.t[tm][tn][v];
  } else if (!SYM && VEC && (m0 + TILE <= a.M) && (n0 + TILE <= a.N) && (a.ldc % 4 == 0) &&
             ((reinterpret_cast<uintptr_t>(a.C) & 15) == 0) && (n0 % 4 == 0)) {
    // Interior tile of a 16-byte aligned C: the accumulators go through LDS so that every
    // thread reads, updates and writes whole 16-byte pieces of C rows, with all of its
    // sixteen loads in flight before the first add (element-wise read-modify-write from
    // the accumulator layout is serialized by the possible aliasing of its own stores).
    // The staging area is the operand buffers: a whole tile at once where they hold 64 KB
    // (32-row stages), otherwise the two 64-row halves one after the other (the rows of
    // half h are the sub-tiles tm = h of every wavefront).
    float* cbase = a.C + m0 * a.ldc + n0;
    float4 cv[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int f = tid + u * WG_THREADS;            // u < 8: rows 0..63, u >= 8: rows 64..127
      cv[u] = *reinterpret_cast<const float4*>(cbase + (int64_t)(f >> 5) * a.ldc + 4 * (f & 31));
    }
    constexpr int HALVES = (4 * KT * TILE >= TILE * TILE) ? 1 : 2;
    static_assert(4 * KT * TILE * HALVES >= TILE * TILE, "staging area");
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
      __syncthreads();                             // the buffers (or the previous half) are no longer read
#pragma unroll
      for (int tm = 0; tm < 2; ++tm) {
        if (HALVES == 2 && tm != h) continue;
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = acc_row(wm, tm, v, lane) - (HALVES == 2 ? 64 * h : 0);
            smem[row * TILE + acc_col(wn, tn, lane)] = a.alpha * acc.t[tm][tn][v];
          }
      }
      __syncthreads();
      constexpr int PER = 16 / HALVES;
#pragma unroll
      for (int u2 = 0; u2 < PER; ++u2) {
        const int u = h * PER + u2;
        const int f = tid + u2 * WG_THREADS;         // position inside the staged rows
        const float4 d = *reinterpret_cast<const float4*>(smem + (f >> 5) * TILE + 4 * (f & 31));
        cv[u].x += d.x; cv[u].y += d.y; cv[u].z += d.z; cv[u].w += d.w;
      }
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int f = tid + u * WG_THREADS;
      *reinterpret_cast<float4*>(cbase + (int64_t)(f >> 5) * a.ldc + 4 * (f & 31)) = cv[u];
    }
  } else {
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
      for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int64_t row = m0 + acc_row(wm, tm, v, lane);
          int64_t col = n0 + acc_col(wn, tn, lane);
          if (row < a.M && col < a.N) {
            float x = a.alpha * acc.t[tm][tn][v];
            a.C[row * a.ldc + col] += x;
            if (SYM && !diag) a.C[col * a.ldc + row] += x;
          }
        }
  }
}

// Short products (K <= 128, few output tiles): C[64 x 64 tile] += alpha * P^T Q with all K
// rows of both operand panels loaded into LDS at once.  Used for the updates inside a
// group of blocks in the column loop, where a 128 x 128 tiling would leave most of the chip
// idle and a stage loop would only add latency.  LDS: 2 x 128 x 64 floats.
template <bool VEC>
__global__ __launch_bounds__(WG_THREADS) void tn_small_kernel(TnGemmArgs a) {
  constexpr int ST = 64;                     // tile edge
  __shared__ __align__(16) float sP[128 * ST];
  __shared__ __align__(16) float sQ[128 * ST];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int ml = lane & 31, kl = lane >> 5;
  const int bi = blockIdx.x / a.tiles_n, bj = blockIdx.x - bi * a.tiles_n;   // tiles_* count 64-tiles here
  const int64_t m0 = (int64_t)bi * ST, n0 = (int64_t)bj * ST;
  const int K = (int)a.K;                    // <= 128, even

  const bool inner = VEC && (m0 + ST <= a.M) && (n0 + ST <= a.N);
  // The old values of C are fetched together with the operands (their latency passes under the
  // operands' and the MFMA loop) and all sixteen before the first store (a load after a store to a possibly aliasing
  // address would wait for it).
  const int64_t col = n0 + wn * 32 + ml;
  float oldv[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int64_t row = m0 + wm * 32 + 8 * (v >> 2) + 4 * kl + (v & 3);
    oldv[v] = (row < a.M && col < a.N) ? a.C[row * a.ldc + col] : 0.0f;
  }

  {
    // 128 rows x 16 float4 per operand = 8 per thread and operand, all in flight together
    constexpr int PER = 128 * (ST / 4) / WG_THREADS;
    float4 p[PER], q[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int f = tid + u * WG_THREADS;
      const int k = f / (ST / 4), c4 = f % (ST / 4);
      p[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      q[u] = p[u];
      if (k < K) {
        if (inner) {
          p[u] = *reinterpret_cast<const float4*>(a.P + (int64_t)k * a.ldp + m0 + 4 * c4);
          q[u] = *reinterpret_cast<const float4*>(a.Q + (int64_t)k * a.ldq + n0 + 4 * c4);
        } else {
          p[u] = tn_load_guarded<VEC>(a.P, a.ldp, k, K, m0 + 4 * c4, a.M);
          q[u] = tn_load_guarded<VEC>(a.Q, a.ldq, k, K, n0 + 4 * c4, a.N);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int f = tid + u * WG_THREADS;
      const int k = f / (ST / 4), c4 = f % (ST / 4);
      *reinterpret_cast<float4*>(sP + k * ST + 4 * c4) = p[u];
      *reinterpret_cast<float4*>(sQ + k * ST + 4 * c4) = q[u];
    }
  }
  __syncthreads();

  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  const float* pp = sP + kl * ST + wm * 32 + ml;
  const float* pq = sQ + kl * ST + wn * 32 + ml;
#pragma unroll 8
  for (int k = 0; k < 128; k += 2)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pp[k * ST], pq[k * ST], acc, 0, 0, 0);

#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int64_t row = m0 + wm * 32 + 8 * (v >> 2) + 4 * kl + (v & 3);
    if (row < a.M && col < a.N) a.C[row * a.ldc + col] = fmaf(a.alpha, acc[v], oldv[v]);
  }
}

// Sum the token-split partial tiles in split order and add alpha * sum to C, writing
// the tile at (bi, bj) and its transpose at (bj, bi).  Four workgroups per upper tile.
// Of a diagonal tile only the 32 x 32 sub-tiles on and above the diagonal are taken from the
// partial sums (the product kernel may leave the others at zero); the sub-tiles below are the
// transposes of those above.
static __global__ __launch_bounds__(WG_THREADS) void tn_reduce_sym_kernel(const float* __restrict__ partial,
                                                                  int splits, int ntiles, int T,
                                                                  float* __restrict__ C, int64_t ldc,
                                                                  int64_t M, float alpha) {
  __shared__ float st[32 * 129];
  const int tid = threadIdx.x;
  const int tile = blockIdx.x >> 2;        // four workgroups per tile, 32 rows each
  int bi, bj;
  decode_sym_tile(tile, T, bi, bj);
  const int64_t m0 = (int64_t)bi * TILE, n0 = (int64_t)bj * TILE;
  const bool vecc = (ldc % 4 == 0) && ((reinterpret_cast<uintptr_t>(C) & 15) == 0);
  {
    const int sb = blockIdx.x & 3;
    // rows sb*32 .. sb*32+31 of the tile: 32 x 128 values, 16 per thread
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      int f = tid + p * WG_THREADS;  // float4 index within the 32 x 128 slab
      int lr = f >> 5, c4 = f & 31;
      const float* src = partial + (int64_t)tile * (TILE * TILE) + (sb * 32 + lr) * TILE + 4 * c4;
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      // slices are added in order; eight loads are in flight at a time
#pragma unroll 8
      for (int sp = 0; sp < splits; ++sp) {
        float4 v = *reinterpret_cast<const float4*>(src + (int64_t)sp * ntiles * (TILE * TILE));
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      s.x *= alpha; s.y *= alpha; s.z *= alpha; s.w *= alpha;
      int64_t row = m0 + sb * 32 + lr;
      int64_t col = n0 + 4 * c4;
      if (row < M && (bi != bj || 4 * c4 >= sb * 32)) {
        float* dst = C + row * ldc + col;
        if (vecc && col + 3 < M) {
          float4 o = *reinterpret_cast<const float4*>(dst);
          o.x += s.x; o.y += s.y; o.z += s.z; o.w += s.w;
          *reinterpret_cast<float4*>(dst) = o;
        } else {
          if (col + 0 < M) dst[0] += s.x;
          if (col + 1 < M) dst[1] += s.y;
          if (col + 2 < M) dst[2] += s.z;
          if (col + 3 < M) dst[3] += s.w;
        }
      }
      float* d = st + lr * 129 + 4 * c4;
      d[0] = s.x; d[1] = s.y; d[2] = s.z; d[3] = s.w;
    }
    __syncthreads();
    {
      // transpose: target row n0 + lc, target columns m0 + sb*32 + (0..31); the sixteen old
      // values of a thread are loaded before its first store.  Diagonal tile: only the
      // columns lc of the sub-tiles to the right of sub-tile (sb, sb).
      const int lc_min = (bi != bj) ? 0 : (sb + 1) * 32;
      const int lr = tid & 31;
      const int64_t col = m0 + sb * 32 + lr;
      float oldv[TILE / 8];
#pragma unroll
      for (int q = 0; q < TILE / 8; ++q) {
        const int lc = (tid >> 5) + 8 * q;
        const int64_t row = n0 + lc;
        oldv[q] = (lc >= lc_min && row < M && col < M) ? C[row * ldc + col] : 0.0f;
      }
#pragma unroll
      for (int q = 0; q < TILE / 8; ++q) {
        const int lc = (tid >> 5) + 8 * q;
        const int64_t row = n0 + lc;
        if (lc >= lc_min && row < M && col < M) C[row * ldc + col] = oldv[q] + st[lr * 129 + lc];
      }
    }
    __syncthreads();
  }
}

}  // namespace lq
