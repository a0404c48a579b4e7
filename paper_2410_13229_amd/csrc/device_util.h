// Device-side helpers shared by the kernels: MFMA operand types and the int32 -> int8
// requantization of Eq. 2 applied to accumulators.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace quamba {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Four already scaled values -> four int8 codes (Eq. 2) in one word, first value in the low
// byte.  Clamping to [-128, 127] first and then adding 1.5 * 2^23 leaves the rounded integer in
// the low mantissa bits (the sum's unit in the last place is 1 and the constant is even, so ties
// go to even exactly as rintf would send them); the low byte is the two's-complement code.
__device__ __forceinline__ unsigned pack_q8x4(float v0, float v1, float v2, float v3) {
  const unsigned b0 = __float_as_uint(__builtin_amdgcn_fmed3f(v0, -128.f, 127.f) + 12582912.f);
  const unsigned b1 = __float_as_uint(__builtin_amdgcn_fmed3f(v1, -128.f, 127.f) + 12582912.f);
  const unsigned b2 = __float_as_uint(__builtin_amdgcn_fmed3f(v2, -128.f, 127.f) + 12582912.f);
  const unsigned b3 = __float_as_uint(__builtin_amdgcn_fmed3f(v3, -128.f, 127.f) + 12582912.f);
  return __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u) | __builtin_amdgcn_perm(b3, b2, 0x04000c0cu);
}

// Four int32 accumulators -> int8 codes of float(acc) * m.
__device__ __forceinline__ unsigned requant_pack4(const int (&a)[4], float m) {
  return pack_q8x4(static_cast<float>(a[0]) * m, static_cast<float>(a[1]) * m, static_cast<float>(a[2]) * m,
                   static_cast<float>(a[3]) * m);
}

}  // namespace quamba
