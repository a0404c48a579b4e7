// Device-side helpers shared by the kernels: MFMA operand types and the int32 -> int8
// requantization of Eq. 2 applied to accumulators.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cstdint>

namespace quamba {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Sum of an int over the 64 lanes of the wave, the same value returned to every lane.  Four DPP steps
// (inside quads, half rows, rows of 16: plain VALU operand swizzles, no LDS round trip as a shuffle
// would take) and the four row sums read out as scalars.
__device__ __forceinline__ int wave_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);   // quad_perm [1, 0, 3, 2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);   // quad_perm [2, 3, 0, 1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);  // row_half_mirror
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);  // row_mirror
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

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

// One generation step of the causal conv + SiLU + requantization (Section 4.3 "Fused causal
// convolution") for four adjacent channels of one sequence: window = [state (3, fp16),
// s_xpre * xpre_q] in fp32, weights s_cw * w_q, products and sums rounded one by one in tap order;
// the window then shifts by one.  `xin`: the four new int8 codes; `cs`: 12 fp16 of state
// (channel-major, oldest first), updated in place.  Returns the four int8 output codes.
// conv_step4_values leaves SiLU(conv) of the four channels in sv; conv_step4 quantizes them.
struct ConvWindow4 {  // the fp16 windows of four adjacent channels: 12 halves, channel-major, oldest first
  uint2 u[3];
};
__device__ __forceinline__ void conv_step4_core(unsigned xin, const uint4 &wv, const float4 &bv, ConvWindow4 &win,
                                                float s_cw, float s_xpre, float (&sv)[4]) {
  const unsigned wword[4] = {wv.x, wv.y, wv.z, wv.w};
  const float bb[4] = {bv.x, bv.y, bv.z, bv.w};
  union {
    uint2 u[3];
    __half h[12];
  } st;
  st.u[0] = win.u[0];
  st.u[1] = win.u[1];
  st.u[2] = win.u[2];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const float xn = __fmul_rn(s_xpre, static_cast<float>(static_cast<int8_t>(xin >> (8 * c))));
    const float w4[4] = {__half2float(st.h[3 * c]), __half2float(st.h[3 * c + 1]), __half2float(st.h[3 * c + 2]), xn};
    float v = bb[c];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float wj = __fmul_rn(s_cw, static_cast<float>(static_cast<int8_t>(wword[c] >> (8 * j))));
      v = __fadd_rn(v, __fmul_rn(wj, w4[j]));
    }
    sv[c] = v / (1.f + __builtin_amdgcn_exp2f(-v * 1.44269504088896340736f));
    st.h[3 * c] = st.h[3 * c + 1];
    st.h[3 * c + 1] = st.h[3 * c + 2];
    st.h[3 * c + 2] = __float2half_rn(xn);
  }
  win.u[0] = st.u[0];
  win.u[1] = st.u[1];
  win.u[2] = st.u[2];
}

__device__ __forceinline__ void conv_step4_values(unsigned xin, const int8_t *wq4, const float *bias4, __half *cs,
                                                  float s_cw, float s_xpre, float (&sv)[4]) {
  const uint4 wv = *reinterpret_cast<const uint4 *>(wq4);
  const float4 bv = *reinterpret_cast<const float4 *>(bias4);
  ConvWindow4 win;
  win.u[0] = reinterpret_cast<const uint2 *>(cs)[0];
  win.u[1] = reinterpret_cast<const uint2 *>(cs)[1];
  win.u[2] = reinterpret_cast<const uint2 *>(cs)[2];
  conv_step4_core(xin, wv, bv, win, s_cw, s_xpre, sv);
  reinterpret_cast<uint2 *>(cs)[0] = win.u[0];
  reinterpret_cast<uint2 *>(cs)[1] = win.u[1];
  reinterpret_cast<uint2 *>(cs)[2] = win.u[2];
}

__device__ __forceinline__ unsigned conv_step4(unsigned xin, const int8_t *wq4, const float *bias4, __half *cs,
                                               float s_cw, float s_xpre, float inv_s_x) {
  float sv[4];
  conv_step4_values(xin, wq4, bias4, cs, s_cw, s_xpre, sv);
  return pack_q8x4(sv[0] * inv_s_x, sv[1] * inv_s_x, sv[2] * inv_s_x, sv[3] * inv_s_x);
}

// ---- non-uniform 8-bit formats of the scan input (Appendix K: log2, and the E4M3 float it names) ----
// E4M3 (1-4-3 bits, bias 7, subnormals m 2^-9, largest finite value 448 = 0x7e, no infinities):
// nearest representable value of t, ties to the even mantissa, saturating; the sign bit of t is kept.
__device__ __forceinline__ unsigned encode_e4m3(float t) {
  const unsigned tb = __float_as_uint(t);
  const float a = fminf(__uint_as_float(tb & 0x7fffffffu), 448.f);
  int E = static_cast<int>(__float_as_uint(a) >> 23) - 127;
  E = E < -6 ? -6 : E;  // below the smallest normal the subnormal spacing 2^-9 holds
  // a / 2^(E-3): an exact scaling by a power of two, then round to nearest even
  int q = static_cast<int>(__builtin_rintf(a * __uint_as_float(static_cast<unsigned>(130 - E) << 23)));
  if (q == 16) {  // rounded up into the next binade
    q = 8;
    ++E;
  }
  unsigned field = q >= 8 ? ((static_cast<unsigned>(E + 7) << 3) | static_cast<unsigned>(q - 8)) : static_cast<unsigned>(q);
  field = field > 0x7eu ? 0x7eu : field;
  return field | ((tb >> 24) & 0x80u);
}
__device__ __forceinline__ float decode_e4m3(unsigned c) {
  const unsigned mag = c & 0x7fu;
  const float normal = __uint_as_float((mag << 20) + 0x3c000000u);  // exponent field + 120, mantissa in the top bits
  const float sub = static_cast<float>(mag) * 0.001953125f;          // m 2^-9
  return __uint_as_float(__float_as_uint(mag < 8u ? sub : normal) | ((c & 0x80u) << 24));
}
// log2: t = f 2^E with 1 <= f < 2 goes to 2^k, k = E + (f >= fp32(sqrt 2)) (nearest in the log domain);
// code = sign bit | e with e = -k in 0..126 (larger t saturates at e = 0), 127 for zero and for
// anything below 2^-126.5.  Integer work on the bits of t, so subnormal t needs no care elsewhere.
__device__ __forceinline__ unsigned encode_log2(float t) {
  const unsigned tb = __float_as_uint(t);
  const unsigned ab = tb & 0x7fffffffu;
  const int ef = static_cast<int>(ab >> 23);
  const unsigned man = ab & 0x7fffffu;
  int k;
  if (ef != 0) {
    k = ef - 127 + (man >= 0x3504f3u ? 1 : 0);
  } else {  // subnormal: only [2^-127 sqrt 2, 2^-126) still reaches e = 126
    k = (man >= 0x5a827au) ? -126 : -200;  // man 2^-149 >= 2^-127 fp32(sqrt 2), i.e. man >= 0xb504f3 / 2 rounded up
  }
  int e = -k;
  const bool zero = ab == 0u || e > 126;
  e = e < 0 ? 0 : e;
  return zero ? 127u : (static_cast<unsigned>(e) | ((tb >> 24) & 0x80u));
}
__device__ __forceinline__ float decode_log2(unsigned c) {
  const unsigned e = c & 0x7fu;
  const unsigned bits = e == 127u ? 0u : ((127u - e) << 23);
  return __uint_as_float(bits | ((c & 0x80u) << 24));
}

// ---- per-call scale of the scan input (Appendix K, dynamic row).  One device word holds the bits of
// max|x| of the call; every reader derives what it needs from it with the same correctly rounded
// operations, so all of them (and the CPU check) agree bit for bit:
//   s = max / 127 (1 if max is 0),  1 / s,  multiplier = (s * s_W) / s_out
__device__ __forceinline__ float dyn_scale(const unsigned *slot) {
  const float mx = __uint_as_float(*slot);
  return mx > 0.f ? __fdiv_rn(mx, 127.f) : 1.f;
}
__device__ __forceinline__ float dyn_inv_scale(const unsigned *slot) { return __fdiv_rn(1.f, dyn_scale(slot)); }
__device__ __forceinline__ float dyn_multiplier(const unsigned *slot, float s_W, float s_out) {
  return __fdiv_rn(__fmul_rn(dyn_scale(slot), s_W), s_out);
}

// four floats -> four fp16 in one 8-byte word
__device__ __forceinline__ uint2 pack_f16x4(float v0, float v1, float v2, float v3) {
  union {
    uint2 u;
    __half h[4];
  } o;
  o.h[0] = __float2half_rn(v0);
  o.h[1] = __float2half_rn(v1);
  o.h[2] = __float2half_rn(v2);
  o.h[3] = __float2half_rn(v3);
  return o.u;
}

// Buffer descriptor over [base, base + bytes).  An access takes a scalar byte offset plus a 32-bit
// lane offset, so its address costs no vector arithmetic (a 64-bit vector address is a quarter-rate
// multiply-add per access); a lane offset past the end reads as zero and is not written (the range
// test looks at the lane offset only), so a lane is switched off by an offset >= bytes and a whole
// output by bytes = 0.  `base` must be wave-uniform and bytes < 2^31.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_over(const void *base, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ int buffer_load_i8(__amdgpu_buffer_rsrc_t r, unsigned lane_off, int wave_off) {
  return static_cast<int>(static_cast<int8_t>(__builtin_amdgcn_raw_buffer_load_b8(r, lane_off, wave_off, 0)));
}
__device__ __forceinline__ unsigned buffer_load_u16(__amdgpu_buffer_rsrc_t r, unsigned lane_off, int wave_off) {
  return __builtin_amdgcn_raw_buffer_load_b16(r, lane_off, wave_off, 0);
}
__device__ __forceinline__ void buffer_store_f32(__amdgpu_buffer_rsrc_t r, unsigned lane_off, int wave_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, lane_off, wave_off, 0);
}
__device__ __forceinline__ void buffer_store_f16(__amdgpu_buffer_rsrc_t r, unsigned lane_off, int wave_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b16(__half_as_ushort(__float2half_rn(v)), r, lane_off, wave_off, 0);
}

// ---- read-ahead: workgroups appended to a launch that is not bound by memory read ranges the following kernels
// will need (the weights of the next projections), so that the lines wait in the last-level cache.  Plain loads,
// 16 per thread in flight; nothing is written, the sum only keeps the loads alive.
struct WarmRanges {
  const uint4 *ptr[3];
  unsigned n16[3];  // length in 16-byte words
  int blocks;       // workgroups of the launch that do this (0: none)
};
__device__ __forceinline__ void warm_read(const WarmRanges &w, int part, int nparts) {
  unsigned acc = 0;
  const size_t step = (size_t)nparts * blockDim.x;
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const uint4 *q = w.ptr[r];
    const size_t n = w.n16[r];
    size_t i = (size_t)part * blockDim.x + threadIdx.x;
    for (; i + 15 * step < n; i += 16 * step) {
      uint4 v[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) v[j] = q[i + j * step];
#pragma unroll
      for (int j = 0; j < 16; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    }
    for (; i < n; i += step) {
      const uint4 v = q[i];
      acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
  }
  asm volatile("" ::"v"(acc));
}

}  // namespace quamba
