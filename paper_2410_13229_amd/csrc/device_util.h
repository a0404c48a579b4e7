// Device-side helpers shared by the kernels: MFMA operand types and the int32 -> int8
// requantization of Eq. 2 applied to accumulators.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace quamba {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Four accumulators -> four int8 codes in one word: round-to-nearest-even of float(acc) * m,
// saturated.  Clamping to [-128, 127] first and then adding 1.5 * 2^23 leaves the rounded
// integer in the low mantissa bits (the sum's unit in the last place is 1 and the constant is
// even, so ties go to even exactly as rintf would send them); the low byte is the code.
__device__ __forceinline__ unsigned requant_pack4(const int (&a)[4], float m) {
  unsigned b[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float v = __builtin_amdgcn_fmed3f(static_cast<float>(a[e]) * m, -128.f, 127.f);
    b[e] = __float_as_uint(v + 12582912.f);
  }
  const unsigned lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);  // [b0, b1, 0, 0]
  const unsigned hi = __builtin_amdgcn_perm(b[3], b[2], 0x04000c0cu);  // [0, 0, b2, b3]
  return lo | hi;
}

}  // namespace quamba
