// Column kernel instances for block width B = 128.
#include "lq_quantize_col.h"

namespace lq {
lq_status launch_column_128(const ColArgs& a, const lq_params* P, hipStream_t st) {
  return launch_column<128>(a, P, st);
}
}  // namespace lq
