// lq_quantize_layer: the blocked quantize-and-propagate loop (Algorithm 1 lines 10-21).
//
// Rows of W are independent problems (Section 2.2), the only sequential dimension
// is the column index.  Per block of B columns two kernels run:
//   * the column kernel: one lane owns one row and keeps that row's B weights of the
//     block in registers; for every column it quantizes against the row's grid
//     (line 13 / 15), forms E = (w - q) / U_jj (line 16) and subtracts E * U[j, j+1:]
//     from its remaining registers (line 17).  The B x B diagonal blocks of U are packed
//     once per layer and read as wave-uniform scalars.  E is written transposed so that
//   * the trailing update W[:, i+B:] -= E U[i:i+B, i+B:] (line 19) is a k-major
//     fp32 MFMA product of the same kind as the Hessian accumulation.  Blocks are taken
//     in groups of 4: after a block only the remaining columns of its group are updated
//     (they are needed next); the columns beyond the group receive the 4 blocks' updates
//     at once as one 4B-deep product.  The sums are the same, re-associated; W beyond
//     the group is read and written once per group instead of once per block.
#include "lq_common.h"
#include "lq_tn_gemm.h"

#include "lq_quantize_col.h"

namespace {
#ifndef LQ_GROUP8_ROWS
#define LQ_GROUP8_ROWS 16384
#endif

constexpr int KT = 16;      // rows of E^T and U per stage of the trailing product
constexpr int MINW = 3;    // resident workgroups per CU the kernel is compiled for
// blocks whose far-field updates are applied together: more for layers with many rows, where
// the far field is large and each pass over it costs its read-modify-write traffic
inline int group_blocks(int64_t r) { return r >= LQ_GROUP8_ROWS ? 8 : 4; }

// Pack the diagonal B x B blocks of U: ud[blk][j][jj] = U[i0+j][i0+jj] for jj >= j inside the
// matrix, zero elsewhere; urinv[blk][j] = 1 / U[i0+j][i0+j] (0 outside the matrix).
__global__ __launch_bounds__(256) void pack_diag_blocks_kernel(const float* __restrict__ U, int64_t ldu,
                                                               int64_t c, int B, float* __restrict__ ud,
                                                               float* __restrict__ urinv) {
  const int64_t i0 = (int64_t)blockIdx.x * B;
  float* dst = ud + (int64_t)blockIdx.x * B * B;
  for (int f = threadIdx.x; f < B * B; f += 256) {
    int j = f / B, jj = f - j * B;
    float v = 0.0f;
    if (jj >= j && i0 + jj < c) v = U[(i0 + j) * ldu + i0 + jj];
    dst[f] = v;
  }
  for (int j = threadIdx.x; j < B; j += 256)
    urinv[(int64_t)blockIdx.x * B + j] = (i0 + j < c) ? 1.0f / U[(i0 + j) * ldu + i0 + j] : 0.0f;
}

struct QuantPlan {
  int64_t rpad, nblk;
  size_t off_ud, off_rinv, total;
};

QuantPlan make_plan(int64_t r, int64_t c, int B) {
  QuantPlan p;
  p.rpad = lq::ceil_div(r > 0 ? r : 1, lq::QT) * lq::QT;   // one slot per lane of the column kernel
  p.nblk = lq::ceil_div(c, B);
  p.off_ud = lq::align_up((size_t)p.rpad * B * group_blocks(r) * sizeof(float), 256);
  p.off_rinv = p.off_ud + lq::align_up((size_t)p.nblk * B * B * sizeof(float), 256);
  p.total = p.off_rinv + lq::align_up((size_t)p.nblk * B * sizeof(float), 256);
  return p;
}

}  // namespace

namespace lq {
size_t quantize_workspace_bytes(int64_t r, int64_t c, int block) {
  return make_plan(r, c, block > 0 ? block : 128).total;
}
}  // namespace lq

extern "C" lq_status lq_quantize_layer(float* W, int64_t r, int64_t c, int64_t ldw, const float* U,
                                       int64_t ldu, const float* grid, const lq_params* P,
                                       uint8_t* codes, float* row_loss, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (r == 0 && c >= 1) return LQ_OK;   // nothing to do; empty buffers may be null
  if (!W || !U || !grid || !codes) return lq::fail(LQ_ERR_INVALID_ARG, "lq_quantize_layer: null pointer");
  if (!lq::aligned(grid, 16)) return lq::fail(LQ_ERR_INVALID_ARG, "lq_quantize_layer: grid must be 16-byte aligned");
  if (r < 0 || c < 1 || ldw < c || ldu < c)
    return lq::fail(LQ_ERR_INVALID_ARG, "lq_quantize_layer: r=%lld c=%lld ldw=%lld ldu=%lld", (long long)r, (long long)c, (long long)ldw, (long long)ldu);
  lq_status stt = lq::check_params(P, c);
  if (stt != LQ_OK) return stt;
  const int B = P->block;
  if (B != 32 && B != 64 && B != 128)
    return lq::fail(LQ_ERR_UNSUPPORTED, "lq_quantize_layer: block=%d (supported: 32, 64, 128)", B);
  const QuantPlan plan = make_plan(r, c, B);
  size_t need = plan.total;
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < need)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_quantize_layer: workspace needs %zu bytes, 256-byte aligned", need);
  if (r == 0) return LQ_OK;

  hipStream_t st = (hipStream_t)stream;
  const int64_t rpad = plan.rpad;
  float* ud = (float*)((char*)ws + plan.off_ud);
  float* urinv = (float*)((char*)ws + plan.off_rinv);
  lq::ColArgs a;
  a.W = W; a.ldw = ldw; a.r = r; a.c = c;
  a.grid = grid;
  a.group = (P->mode == LQ_GRID_AFFINE) ? (P->group_size > 0 ? P->group_size : (int)c) : (int)c;
  a.ngroups = (int)(c / a.group);
  a.codes = codes;
  a.Et = (float*)ws; a.rpad = rpad;
  a.row_loss = row_loss;
  a.vecw = (ldw % 4 == 0) && lq::aligned(W, 16);
  a.vecc = (c % 4 == 0) && lq::aligned(codes, 4);

  const size_t gemm_lds = 4 * KT * lq::TILE * sizeof(float);
  static lq::DeviceOnce attr_once;
  if (lq::DeviceOnceGuard once(attr_once); once.first()) {
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)lq::tn_gemm_kernel<KT, false, false, true, MINW>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)lq::tn_gemm_kernel<KT, false, false, false, MINW>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)lq::tn_gemm_kernel<KT, false, false, true, MINW, true>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds));
    once.done();
  }

  hipLaunchKernelGGL(pack_diag_blocks_kernel, dim3((unsigned)plan.nblk), dim3(256), 0, st, U, ldu, c, B,
                     ud, urinv);
  LQ_CHECK_LAUNCH("pack_diag_blocks_kernel");

  // C[:, col0 : col0+ncols] -= Et[0:K, :]^T * U[urow0 : urow0+K, col0 : col0+ncols]
  auto update = [&](const float* et, int64_t K, int64_t urow0, int64_t col0, int64_t ncols) -> lq_status {
    lq::TnGemmArgs t;
    t.P = et; t.ldp = rpad;
    t.Q = U + urow0 * ldu + col0; t.ldq = ldu;
    t.C = W + col0; t.ldc = ldw;
    t.M = r; t.N = ncols; t.K = K;
    t.alpha = -1.0f;
    t.tiles_m = (int)lq::ceil_div(r, lq::TILE);
    t.tiles_n = (int)lq::ceil_div(ncols, lq::TILE);
    t.ntiles = t.tiles_m * t.tiles_n;
    t.splits = 1;
    t.k_per_split = K;
    t.partial = nullptr;
    const bool vec = (ldu % 4 == 0) && lq::aligned(t.Q, 16);
    dim3 block2(lq::WG_THREADS);
    if (K <= 128 && t.ntiles <= 512) {
      // short and narrow: 64 x 64 tiles, one LDS fill per workgroup
      t.tiles_m = (int)lq::ceil_div(r, 64);
      t.tiles_n = (int)lq::ceil_div(ncols, 64);
      dim3 grid3((unsigned)(t.tiles_m * t.tiles_n));
      if (vec) hipLaunchKernelGGL(lq::tn_small_kernel<true>, grid3, block2, 0, st, t);
      else hipLaunchKernelGGL(lq::tn_small_kernel<false>, grid3, block2, 0, st, t);
      LQ_CHECK_LAUNCH("tn_small_kernel(trailing)");
      return LQ_OK;
    }
    // Few tiles (layers with few rows, the last groups of any layer): a compute unit's share of
    // the launch is ceil(tiles / 256) whole tiles, or ceil(2 tiles / 256) halves if every tile is
    // split between two workgroups.  The halves are taken where that share is smaller, and
    // wherever not every compute unit gets a whole tile.
    constexpr int64_t CUS = 256;
    const int64_t whole = lq::ceil_div((int64_t)t.ntiles, CUS) * 2, halves = lq::ceil_div(2 * (int64_t)t.ntiles, CUS);
    if (vec && t.ntiles <= 8 * CUS && (halves < whole || t.ntiles <= CUS)) {
      hipLaunchKernelGGL((lq::tn_gemm_kernel<KT, false, false, true, MINW, true>), dim3((unsigned)(2 * t.ntiles)),
                         block2, gemm_lds, st, t);
      LQ_CHECK_LAUNCH("tn_gemm_kernel(trailing, split tiles)");
      return LQ_OK;
    }
    dim3 grid2((unsigned)t.ntiles);
    if (vec)
      hipLaunchKernelGGL((lq::tn_gemm_kernel<KT, false, false, true, MINW>), grid2, block2, gemm_lds, st, t);
    else
      hipLaunchKernelGGL((lq::tn_gemm_kernel<KT, false, false, false, MINW>), grid2, block2, gemm_lds, st, t);
    LQ_CHECK_LAUNCH("tn_gemm_kernel(trailing)");
    return LQ_OK;
  };

  float* const et_base = a.Et;
  const int GROUP = group_blocks(r);
  for (int64_t i0 = 0; i0 < c; i0 += B) {
    const int64_t blk = i0 / B;
    const int64_t li = blk % GROUP;                       // position inside the group
    const int64_t gbase = (blk - li) * B;                 // first column of the group
    const int64_t gend = (gbase + (int64_t)GROUP * B < c) ? gbase + (int64_t)GROUP * B : c;
    const float* udb = ud + blk * B * B;
    const float* rib = urinv + blk * B;
    a.i0 = i0;
    a.nb = (int)((c - i0) < B ? (c - i0) : B);
    a.first = (i0 == 0);
    a.Et = et_base + li * B * rpad;
    lq_status s2 = (B == 128) ? lq::launch_column_128(a, udb, rib, P, st)
                 : (B == 64)  ? lq::launch_column_64(a, udb, rib, P, st)
                              : lq::launch_column_32(a, udb, rib, P, st);
    if (s2 != LQ_OK) return s2;
    const int64_t next = i0 + B;
    if (next < gend) {                                    // rest of the group: needed next
      s2 = update(a.Et, B, i0, next, gend - next);
      if (s2 != LQ_OK) return s2;
    } else if (gend < c) {                                // group finished: everything beyond it
      s2 = update(et_base, (li + 1) * B, gbase, gend, c - gend);
      if (s2 != LQ_OK) return s2;
    }
  }
  return LQ_OK;
}
