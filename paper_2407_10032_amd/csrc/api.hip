// Host-only part of the C ABI: parameter defaults and checks, workspace sizes,
// error text.  No kernels here.
#include <string.h>

#include "lq_common.h"

namespace lq {

size_t hessian_workspace_bytes(int64_t c, int64_t n_tokens);
size_t cholesky_workspace_bytes(int64_t c);
size_t fit_grid_workspace_bytes(int64_t c);
size_t quantize_workspace_bytes(int64_t r, int64_t c, int block);
size_t exact_workspace_bytes(int64_t r, int64_t c);

char* error_buffer() {
  static thread_local char buf[512] = {0};
  return buf;
}

lq_status fail(lq_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), 512, fmt, ap);
  va_end(ap);
  return code;
}

SideStream* side_stream(int which) {
  struct Slot { bool tried = false; bool ok = false; SideStream s; };
  static thread_local Slot slots[16][2];
  int dev = 0;
  if (which < 0 || which > 1) return nullptr;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
  Slot& sl = slots[dev][which];
  if (!sl.tried) {
    sl.tried = true;
    bool ok = hipStreamCreateWithFlags(&sl.s.stream, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; ok && i < 4; ++i)
      ok = hipEventCreateWithFlags(&sl.s.fork[i], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&sl.s.join, hipEventDisableTiming) == hipSuccess;
    sl.ok = ok;
    if (!ok) (void)hipGetLastError();
  }
  return sl.ok ? &sl.s : nullptr;
}

int resolve_t(const lq_params* P) {
  if (P->t_override >= 0) return P->t_override;
  // Eq. 8: t = 0.2 T, 0.3 T, 0.4 T for b = 4, 3, 2; floored (2048 is not divisible by 5).
  int64_t num = (P->bits == 4) ? 2 : (P->bits == 3) ? 3 : 4;
  return (int)((num * (int64_t)P->T) / 10);
}

lq_status check_params(const lq_params* P, int64_t c) {
  if (!P) return fail(LQ_ERR_INVALID_ARG, "lq_params pointer is null");
  if (P->bits < 2 || P->bits > 4) return fail(LQ_ERR_INVALID_ARG, "bits=%d, must be 2, 3 or 4", P->bits);
  if (P->mode != LQ_GRID_NONUNIFORM && P->mode != LQ_GRID_AFFINE)
    return fail(LQ_ERR_INVALID_ARG, "mode=%d is not a grid mode", P->mode);
  if (P->group_size < 0) return fail(LQ_ERR_INVALID_ARG, "group_size=%d is negative", P->group_size);
  if (P->mode == LQ_GRID_NONUNIFORM && P->group_size != 0)
    return fail(LQ_ERR_INVALID_ARG, "non-uniform grids are per row: group_size must be 0");
  if (P->mode == LQ_GRID_AFFINE && P->group_size > 0 && (c % P->group_size) != 0)
    return fail(LQ_ERR_INVALID_ARG, "group_size=%d does not divide c=%lld", P->group_size, (long long)c);
  if (P->block < 1) return fail(LQ_ERR_INVALID_ARG, "block=%d, must be >= 1", P->block);
  if (!(P->p >= 0.0f)) return fail(LQ_ERR_INVALID_ARG, "p must be >= 0");
  if (P->mode == LQ_GRID_AFFINE) {
    if (P->T < 1) return fail(LQ_ERR_INVALID_ARG, "T=%d, must be >= 1", P->T);
    int t = resolve_t(P);
    if (t < 0 || 2 * t > P->T) return fail(LQ_ERR_INVALID_ARG, "t=%d outside 0..T/2", t);
  } else if (P->kmeans_max_iter < 1) {
    return fail(LQ_ERR_INVALID_ARG, "kmeans_max_iter=%d, must be >= 1", P->kmeans_max_iter);
  }
  return LQ_OK;
}

}  // namespace lq

extern "C" void lq_params_default(lq_params* P) {
  if (!P) return;
  memset(P, 0, sizeof(*P));
  P->bits = 4;
  P->mode = LQ_GRID_NONUNIFORM;
  P->group_size = 0;
  P->block = 128;
  P->damp = 0.01f;
  P->p = 4.0f;
  P->T = 2048;
  P->t_override = -1;
  P->kmeans_max_iter = 100;
}

extern "C" size_t lq_workspace_bytes(int which_call, int64_t r, int64_t c, int64_t n_tokens,
                                     const lq_params* P) {
  if (c < 1) return 0;
  switch (which_call) {
    case LQ_CALL_HESSIAN: return lq::hessian_workspace_bytes(c, n_tokens);
    case LQ_CALL_CHOLESKY: return lq::cholesky_workspace_bytes(c);
    case LQ_CALL_FIT_GRID: return lq::fit_grid_workspace_bytes(c);
    case LQ_CALL_QUANTIZE: return lq::quantize_workspace_bytes(r, c, P ? P->block : 128);
    case LQ_CALL_EXACT: return lq::exact_workspace_bytes(r, c);
    default: return 0;
  }
}

extern "C" const char* lq_last_error(void) { return lq::error_buffer(); }

extern "C" const char* lq_version(void) { return "0.1"; }
