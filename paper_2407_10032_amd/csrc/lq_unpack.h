// Reading the stored form of a quantized layer (lq_pack_layer's layout): a row's codes are a
// little-endian bit stream, code j in bits [j b, (j + 1) b).  A "unit" is 32 consecutive codes
// = b 32-bit words (16 / 12 / 8 bytes at 4 / 3 / 2 bits), the piece one lane loads at a time.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lq {

constexpr int UNIT = 32;      // codes per unit

template <int BITS>
__device__ __forceinline__ void load_unit(const uint8_t* p, uint32_t (&w)[BITS]) {
  if constexpr (BITS == 4) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else if constexpr (BITS == 2) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    w[0] = v.x; w[1] = v.y;
  } else {
    const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
    w[0] = q[0]; w[1] = q[1]; w[2] = q[2];
  }
}

// code j (0..31) of a unit held as BITS 32-bit words of the little-endian bit stream
template <int BITS, int J>
__device__ __forceinline__ uint32_t unit_code(const uint32_t (&w)[BITS]) {
  constexpr int pos = BITS * J, idx = pos / 32, sh = pos % 32;
  if constexpr (sh + BITS <= 32) return (w[idx] >> sh) & ((1u << BITS) - 1u);
  else return ((w[idx] >> sh) | (w[idx + 1] << (32 - sh))) & ((1u << BITS) - 1u);
}

}  // namespace lq
