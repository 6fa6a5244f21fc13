// Column kernel instances for block width B = 128.
#include "lq_quantize_col.h"

namespace lq {
lq_status launch_column_128(const ColArgs& a, const float* ud, const float* urinv, const lq_params* P,
                           hipStream_t st) {
  return launch_column<128>(a, ud, urinv, P, st);
}
}  // namespace lq
