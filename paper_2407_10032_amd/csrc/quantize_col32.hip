// Column kernel instances for block width B = 32.
#include "lq_quantize_col.h"

namespace lq {
lq_status launch_column_32(const ColArgs& a, const float* ud, const float* urinv, const lq_params* P,
                           hipStream_t st) {
  return launch_column<32>(a, ud, urinv, P, st);
}
}  // namespace lq
