// lq_hessian_accumulate: H += 2 X^T X  (Algorithm 1 line 3; Section 2.2, H = 2 X X^T
// with the paper's X being channels x tokens).
//
// Symmetric rank-n update on fp32 MFMA: only the tiles on or above the diagonal
// are computed.  The token range is cut into slices so that the launch has many
// more workgroups than the chip has compute units; every (slice, tile) pair
// writes a partial tile into the workspace and a second kernel adds the slices
// in order into both triangles of H.
#include "lq_common.h"
#include "lq_tn_gemm.h"

namespace {

constexpr int KT = 16;                       // tokens per LDS stage: 32 KB of LDS and <= 168 registers put
constexpr int MINW = 3;                      // three workgroups on a CU (1.4 % faster than 32-token
                                             // stages at two per CU; four per CU is slower again)
constexpr int MAX_SPLITS = 64;

struct HessianPlan {
  int T;        // tiles per dimension
  int ntiles;   // tiles on or above the diagonal
  int splits;
  int64_t k_per_split;
  size_t ws_bytes;
};

// The token range is cut into `splits` slices.  More slices mean more, shorter workgroups:
// a shorter tail at the end of the launch, but a larger share of each workgroup spent on its
// first loads and its partial-tile store, and more partial tiles for the reduce kernel to
// read.  The number of slices is the one that minimizes a small time model of these three
// effects (constants measured on MI355X: 2.67 us per 16-token stage of a workgroup that
// shares its compute unit with two others, about 6 us of fixed cost per workgroup, half a
// round of tail unless the workgroups fill a whole number of rounds, 3 TB/s for the reduce kernel).
HessianPlan make_plan(int64_t c, int64_t n_tokens) {
  HessianPlan p;
  p.T = (int)lq::ceil_div(c, lq::TILE);
  p.ntiles = p.T * (p.T + 1) / 2;
  const int64_t n = n_tokens > 0 ? n_tokens : 1;
  const double slots = 256.0 * MINW;           // compute units x resident workgroups
  const double stage_us = 2.67, fixed_us = 6.0;
  int best_s = 1;
  double best_t = 0.0;
  for (int s = 1; s <= MAX_SPLITS; ++s) {
    int64_t per = lq::ceil_div(lq::ceil_div(n, (int64_t)s), (int64_t)KT) * KT;
    const int64_t used = lq::ceil_div(n, per);
    if (used != s) continue;                   // the same slicing as a smaller s
    const double stages = (double)per / KT;
    const double wgs = (double)p.ntiles * (double)used;
    // equal workgroups in a whole number of rounds end nearly together (a quarter round of
    // drift); otherwise the last round is partly empty and costs about half a round
    const bool whole = ((int64_t)wgs % (int64_t)slots) == 0;
    const double rounds = wgs <= slots ? 1.0 : wgs / slots + (whole ? 0.25 : 0.5);
    const double t_main = rounds * (stages * stage_us + fixed_us);
    const double t_reduce = wgs * (lq::TILE * lq::TILE * 4.0) / 3.0e6;   // bytes / (3 TB/s) in us
    const double t = t_main + t_reduce;
    if (s == 1 || t < best_t) { best_t = t; best_s = s; }
  }
  int64_t per = lq::ceil_div(lq::ceil_div(n, (int64_t)best_s), (int64_t)KT) * KT;
  p.k_per_split = per;
  p.splits = (int)lq::ceil_div(n, per);
  p.ws_bytes = (size_t)p.splits * p.ntiles * lq::TILE * lq::TILE * sizeof(float);
  return p;
}

}  // namespace

namespace lq {
size_t hessian_workspace_bytes(int64_t c, int64_t n_tokens) { return make_plan(c, n_tokens).ws_bytes; }
}  // namespace lq

static lq_status accumulate_device(float* H, int64_t ldh, const float* X, int64_t n_tokens,
                                   int64_t c, int64_t ldx, void* ws, size_t ws_bytes,
                                   hipStream_t st) {
  if (!H || (!X && n_tokens > 0)) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hessian_accumulate: null pointer");
  if (c < 1 || n_tokens < 0) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hessian_accumulate: c=%lld n_tokens=%lld", (long long)c, (long long)n_tokens);
  if (ldh < c || ldx < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hessian_accumulate: leading dimension smaller than c");
  if (c > (int64_t)lq::TILE * 1024) return lq::fail(LQ_ERR_UNSUPPORTED, "lq_hessian_accumulate: c > 131072");
  if (n_tokens == 0) return LQ_OK;
  HessianPlan plan = make_plan(c, n_tokens);
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < plan.ws_bytes)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_hessian_accumulate: workspace needs %zu bytes, 256-byte aligned", plan.ws_bytes);

  lq::TnGemmArgs a;
  a.P = X; a.ldp = ldx;
  a.Q = X; a.ldq = ldx;
  a.C = H; a.ldc = ldh;
  a.M = c; a.N = c; a.K = n_tokens;
  a.alpha = 2.0f;
  a.tiles_m = plan.T; a.tiles_n = plan.T;
  a.ntiles = plan.ntiles;
  a.splits = plan.splits;
  a.k_per_split = plan.k_per_split;
  a.partial = (float*)ws;

  const bool vec = (ldx % 4 == 0) && lq::aligned(X, 16);
  const size_t lds = 4 * KT * lq::TILE * sizeof(float);
  dim3 grid((unsigned)((int64_t)plan.splits * plan.ntiles)), block(lq::WG_THREADS);
  static lq::DeviceOnce attr_once;
  if (lq::DeviceOnceGuard once(attr_once); once.first()) {
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)lq::tn_gemm_kernel<KT, true, true, true, MINW>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    LQ_CHECK_HIP(hipFuncSetAttribute((const void*)lq::tn_gemm_kernel<KT, true, true, false, MINW>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    once.done();
  }
  if (vec)
    hipLaunchKernelGGL((lq::tn_gemm_kernel<KT, true, true, true, MINW>), grid, block, lds, st, a);
  else
    hipLaunchKernelGGL((lq::tn_gemm_kernel<KT, true, true, false, MINW>), grid, block, lds, st, a);
  LQ_CHECK_LAUNCH("tn_gemm_kernel(hessian)");
  hipLaunchKernelGGL(lq::tn_reduce_sym_kernel, dim3(4 * plan.ntiles), block, 0, st, (const float*)ws,
                     plan.splits, plan.ntiles, plan.T, H, ldh, c, 2.0f);
  LQ_CHECK_LAUNCH("tn_reduce_sym_kernel");
  return LQ_OK;
}

extern "C" lq_status lq_hessian_accumulate(float* H, int64_t ldh, const float* X, int64_t n_tokens,
                                           int64_t c, int64_t ldx, void* ws, size_t ws_bytes,
                                           void* stream) {
  return accumulate_device(H, ldh, X, n_tokens, c, ldx, ws, ws_bytes, (hipStream_t)stream);
}

// Layout of the host-streaming call's workspace: the partial-sum scratch of the larger of the
// two chunk sizes that occur (whole chunks and the tail), then two chunk buffers.
namespace {
struct HostPlan {
  size_t partial_bytes;
  size_t chunk_bytes;     // one staging buffer, 256-byte multiple
  size_t total;
};
HostPlan make_host_plan(int64_t c, int64_t n_tokens, int64_t chunk_tokens) {
  HostPlan hp;
  const int64_t whole = n_tokens < chunk_tokens ? n_tokens : chunk_tokens;
  const int64_t tail = n_tokens > chunk_tokens ? n_tokens % chunk_tokens : 0;
  size_t part = make_plan(c, whole).ws_bytes;
  if (tail > 0) { const size_t t = make_plan(c, tail).ws_bytes; part = t > part ? t : part; }
  hp.partial_bytes = lq::align_up(part, 256);
  hp.chunk_bytes = lq::align_up((size_t)whole * (size_t)c * sizeof(float), 256);
  hp.total = hp.partial_bytes + 2 * hp.chunk_bytes;
  return hp;
}
}  // namespace

extern "C" size_t lq_hessian_host_workspace_bytes(int64_t c, int64_t n_tokens, int64_t chunk_tokens) {
  if (c < 1 || n_tokens < 1 || chunk_tokens < 1) return 0;
  return make_host_plan(c, n_tokens, chunk_tokens).total;
}

extern "C" lq_status lq_hessian_accumulate_host(float* H, int64_t ldh, const float* X_host,
                                                int64_t n_tokens, int64_t c, int64_t ldx,
                                                int64_t chunk_tokens, void* ws, size_t ws_bytes,
                                                void* stream) {
  if (!H || (!X_host && n_tokens > 0)) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hessian_accumulate_host: null pointer");
  if (c < 1 || n_tokens < 0 || chunk_tokens < 1)
    return lq::fail(LQ_ERR_INVALID_ARG, "lq_hessian_accumulate_host: c=%lld n_tokens=%lld chunk_tokens=%lld",
                    (long long)c, (long long)n_tokens, (long long)chunk_tokens);
  if (ldh < c || ldx < c) return lq::fail(LQ_ERR_INVALID_ARG, "lq_hessian_accumulate_host: leading dimension smaller than c");
  if (n_tokens == 0) return LQ_OK;
  const HostPlan hp = make_host_plan(c, n_tokens, chunk_tokens);
  if (!ws || !lq::aligned(ws, 256) || ws_bytes < hp.total)
    return lq::fail(LQ_ERR_WORKSPACE, "lq_hessian_accumulate_host: workspace needs %zu bytes, 256-byte aligned", hp.total);
  lq::SideStream* side = lq::side_stream(1);
  if (!side) return lq::fail(LQ_ERR_HIP, "lq_hessian_accumulate_host: cannot create the copy stream");

  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)ws;
  float* buf[2] = {(float*)(base + hp.partial_bytes), (float*)(base + hp.partial_bytes + hp.chunk_bytes)};
  // the copy stream starts after everything enqueued before this call (the workspace may be in use)
  LQ_CHECK_HIP(hipEventRecord(side->fork[2], st));
  LQ_CHECK_HIP(hipStreamWaitEvent(side->stream, side->fork[2], 0));
  const int64_t nchunks = lq::ceil_div(n_tokens, chunk_tokens);
  // (a lambda, so that an error in the middle still joins the copy stream below)
  auto chunk_chain = [&]() -> lq_status {
  for (int64_t k = 0; k < nchunks; ++k) {
    const int64_t t0 = k * chunk_tokens;
    const int64_t nt = (n_tokens - t0) < chunk_tokens ? (n_tokens - t0) : chunk_tokens;
    float* dst = buf[k & 1];
    // chunk k overwrites the buffer of chunk k - 2: wait until that one is accumulated
    if (k >= 2) LQ_CHECK_HIP(hipStreamWaitEvent(side->stream, side->fork[k & 1], 0));
    // rows are packed on the device (leading dimension c)
    if (ldx == c)
      LQ_CHECK_HIP(hipMemcpyAsync(dst, X_host + t0 * ldx, (size_t)nt * (size_t)c * sizeof(float),
                                  hipMemcpyHostToDevice, side->stream));
    else
      LQ_CHECK_HIP(hipMemcpy2DAsync(dst, (size_t)c * sizeof(float), X_host + t0 * ldx, (size_t)ldx * sizeof(float),
                                    (size_t)c * sizeof(float), (size_t)nt, hipMemcpyHostToDevice, side->stream));
    LQ_CHECK_HIP(hipEventRecord(side->join, side->stream));
    LQ_CHECK_HIP(hipStreamWaitEvent(st, side->join, 0));
    lq_status rc = accumulate_device(H, ldh, dst, nt, c, c, base, hp.partial_bytes, st);
    if (rc != LQ_OK) return rc;
    if (k + 2 < nchunks) LQ_CHECK_HIP(hipEventRecord(side->fork[k & 1], st));
  }
  return LQ_OK;
  };
  const lq_status rc = chunk_chain();
  if (rc != LQ_OK) {
    // a copy may be in flight that `stream` has not been told to wait for: join it
    if (hipEventRecord(side->join, side->stream) == hipSuccess) (void)hipStreamWaitEvent(st, side->join, 0);
  }
  return rc;
}
