// Bandwidth-bound stages around the GEMMs: input quantization (Eq. 2), the fused int8 causal
// conv + SiLU + requantization in its prefill and decode forms (Section 4.3 "Fused causal
// convolution"), and the fused residual add + RMSNorm + quantization (Section 4.3 "Fused
// RMSNorm").  Every kernel reads and writes each byte once, with 4- to 16-byte accesses per
// lane that are contiguous across the wavefront.
#include <algorithm>

#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

__device__ __forceinline__ int q8(float v) {
  v = __builtin_rintf(v);
  v = __builtin_amdgcn_fmed3f(v, -128.f, 127.f);
  return static_cast<int>(v);
}

// ------------------------------------------------------------------ quantize fp16 -> int8
__global__ __launch_bounds__(256) void quantize_f16_kernel(const __half *__restrict__ x,
                                                           int8_t *__restrict__ q, size_t n,
                                                           float inv_s) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i + 8 <= n) {
    union {
      uint4 u;
      __half h[8];
    } in;
    in.u = *reinterpret_cast<const uint4 *>(x + i);
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = __half2float(in.h[e]) * inv_s;
    *reinterpret_cast<uint2 *>(q + i) = make_uint2(pack_q8x4(v[0], v[1], v[2], v[3]), pack_q8x4(v[4], v[5], v[6], v[7]));
  } else {
    for (size_t j = i; j < n; ++j) q[j] = static_cast<int8_t>(q8(__half2float(x[j]) * inv_s));
  }
}

// ------------------------------------------------------------------ conv, prefill
// One thread owns 4 adjacent channels (one 32-bit word per token) and TT consecutive tokens of
// one sequence.  All TT+3 words are requested up front; a pair of byte permutes per channel
// turns "4 channels of one tap" into "4 taps of one channel", which v_dot4_i32_i8 multiplies
// with that channel's packed weights.

__device__ __forceinline__ float silu_fast(float v) {
  return v * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-v * 1.44269504088896340736f));
}

// OUT_F16 (the Appendix H comparison variant): the SiLU output is stored in half precision into
// x16 instead of being quantized into xq.  OUT_ASYM (Appendix K): codes on an asymmetric grid,
// clamp(rne(v / s + zero point)).  OUT_E4M3 / OUT_LOG2 (Appendix K): one-byte codes of v / s in that format.
enum ConvOut { OUT_SYM, OUT_F16, OUT_ASYM, OUT_E4M3, OUT_LOG2 };
template <ConvOut MODE>
__device__ __forceinline__ unsigned conv_pack4(const float (&sv)[4]) {
  if constexpr (MODE == OUT_E4M3)
    return encode_e4m3(sv[0]) | (encode_e4m3(sv[1]) << 8) | (encode_e4m3(sv[2]) << 16) | (encode_e4m3(sv[3]) << 24);
  else if constexpr (MODE == OUT_LOG2)
    return encode_log2(sv[0]) | (encode_log2(sv[1]) << 8) | (encode_log2(sv[2]) << 16) | (encode_log2(sv[3]) << 24);
  else
    return pack_q8x4(sv[0], sv[1], sv[2], sv[3]);
}
template <ConvOut MODE, int CONV_TT>
__global__ __launch_bounds__(256) void conv_prefill_kernel(
    const int8_t *__restrict__ xpre, int ldx, const int8_t *__restrict__ wq,
    const float *__restrict__ bias, int L, int Di, float m_conv, float inv_s_x, float s_xpre,
    int8_t *__restrict__ xq, __half *__restrict__ x16, float x_zp, __half *__restrict__ conv_state) {
  constexpr bool F16OUT = MODE == OUT_F16;
  const int c4 = blockIdx.x * 256 + threadIdx.x;  // channel group
  if (c4 * 4 >= Di) return;
  const int d0 = c4 * 4;
  const int b = blockIdx.z;
  const int t0 = blockIdx.y * CONV_TT;
  const int t1 = min(t0 + CONV_TT, L);

  const uint4 wv = *reinterpret_cast<const uint4 *>(wq + (size_t)d0 * 4);  // [channel][tap]
  const int wword[4] = {(int)wv.x, (int)wv.y, (int)wv.z, (int)wv.w};
  const float4 bv = *reinterpret_cast<const float4 *>(bias + d0);
  const float bb[4] = {bv.x, bv.y, bv.z, bv.w};

  const int8_t *src = xpre + (size_t)b * L * ldx + d0;
  int8_t *dst = xq + (size_t)b * L * Di + d0;
  unsigned h[CONV_TT + 3];
#pragma unroll
  for (int i = 0; i < CONV_TT + 3; ++i) {
    const int t = t0 - 3 + i;
    h[i] = (t >= 0 && t < t1) ? *reinterpret_cast<const unsigned *>(src + (size_t)t * ldx) : 0u;
  }
  unsigned outw[CONV_TT];  // the codes are stored after the last token is computed (0.7 us faster at 2048 x 5120 than storing each as it is ready)
#pragma unroll
  for (int i = 0; i < CONV_TT; ++i) {
    outw[i] = 0u;
    if (t0 + i < t1) {
      // bytes of h[i..i+3]: taps oldest..newest, 4 channels each -> per channel its 4 taps
      const unsigned ta = __builtin_amdgcn_perm(h[i + 1], h[i], 0x05010400u);
      const unsigned tb = __builtin_amdgcn_perm(h[i + 1], h[i], 0x07030602u);
      const unsigned ua = __builtin_amdgcn_perm(h[i + 3], h[i + 2], 0x05010400u);
      const unsigned ub = __builtin_amdgcn_perm(h[i + 3], h[i + 2], 0x07030602u);
      const unsigned taps[4] = {__builtin_amdgcn_perm(ua, ta, 0x05040100u), __builtin_amdgcn_perm(ua, ta, 0x07060302u),
                                __builtin_amdgcn_perm(ub, tb, 0x05040100u), __builtin_amdgcn_perm(ub, tb, 0x07060302u)};
      float sv[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int a = __builtin_amdgcn_sdot4((int)taps[c], wword[c], 0, false);
        const float v = __fadd_rn(__fmul_rn(static_cast<float>(a), m_conv), bb[c]);
        sv[c] = F16OUT ? silu_fast(v) : silu_fast(v) * inv_s_x;
        if constexpr (MODE == OUT_ASYM) sv[c] = __fadd_rn(sv[c], x_zp);
      }
      if constexpr (F16OUT)
        *reinterpret_cast<uint2 *>(x16 + ((size_t)b * L + t0 + i) * Di + d0) = pack_f16x4(sv[0], sv[1], sv[2], sv[3]);
      else
        outw[i] = conv_pack4<MODE>(sv);
    }
  }
  if constexpr (!F16OUT) {
#pragma unroll
    for (int i = 0; i < CONV_TT; ++i)
      if (t0 + i < t1) *reinterpret_cast<unsigned *>(dst + (size_t)(t0 + i) * Di) = outw[i];
  }
  // the tile holding the sequence end also emits the carried window [L-3, L-2, L-1]
  if (conv_state != nullptr && t1 == L) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int tj = L - 3 + j;
      unsigned w = 0u;
      if (tj >= 0) {
        // tj >= t0 - 3 always holds for the last tile; pick the word out of the preloaded window
#pragma unroll
        for (int i = 0; i < CONV_TT + 3; ++i)
          if (t0 - 3 + i == tj) w = h[i];
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float v = tj >= 0 ? s_xpre * static_cast<float>(static_cast<int8_t>(w >> (8 * c))) : 0.f;
        conv_state[((size_t)b * Di + d0 + c) * 3 + j] = __float2half_rn(v);
      }
    }
  }
}

// ------------------------------------------------------------------ conv, decode step
template <ConvOut MODE>
__global__ __launch_bounds__(256) void conv_step_kernel(const int8_t *__restrict__ xpre, int ldx,
                                                        const int8_t *__restrict__ wq,
                                                        const float *__restrict__ bias, int Bt, int Di,
                                                        float s_cw, float s_xpre, float inv_s_x,
                                                        int8_t *__restrict__ xq, __half *__restrict__ x16,
                                                        float x_zp, __half *__restrict__ conv_state) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // (b, channel group of 4)
  const int groups = Di / 4;
  if (idx >= (size_t)Bt * groups) return;
  const int b = static_cast<int>(idx / groups);
  const int d0 = static_cast<int>(idx % groups) * 4;
  const unsigned xin = *reinterpret_cast<const unsigned *>(xpre + (size_t)b * ldx + d0);
  __half *cs = conv_state + ((size_t)b * Di + d0) * 3;
  if constexpr (MODE == OUT_SYM) {
    *reinterpret_cast<unsigned *>(xq + (size_t)b * Di + d0) =
        conv_step4(xin, wq + (size_t)d0 * 4, bias + d0, cs, s_cw, s_xpre, inv_s_x);
  } else {
    float sv[4];
    conv_step4_values(xin, wq + (size_t)d0 * 4, bias + d0, cs, s_cw, s_xpre, sv);
    if constexpr (MODE == OUT_F16) {  // half-precision output, no quantizer
      *reinterpret_cast<uint2 *>(x16 + (size_t)b * Di + d0) = pack_f16x4(sv[0], sv[1], sv[2], sv[3]);
    } else if constexpr (MODE == OUT_ASYM) {
      *reinterpret_cast<unsigned *>(xq + (size_t)b * Di + d0) =
          pack_q8x4(__fadd_rn(sv[0] * inv_s_x, x_zp), __fadd_rn(sv[1] * inv_s_x, x_zp),
                    __fadd_rn(sv[2] * inv_s_x, x_zp), __fadd_rn(sv[3] * inv_s_x, x_zp));
    } else {
      const float tv[4] = {sv[0] * inv_s_x, sv[1] * inv_s_x, sv[2] * inv_s_x, sv[3] * inv_s_x};
      *reinterpret_cast<unsigned *>(xq + (size_t)b * Di + d0) = conv_pack4<MODE>(tv);
    }
  }
}

// ------------------------------------------------------------------ add + RMSNorm + quant
// One workgroup per token row; each thread keeps its share of the row in registers between
// the reduction and the normalisation, so the row is read once.
constexpr int RMS_MAX_PER_THREAD = 4;  // groups of 8 halves per thread: Dm <= 8192

// PART: x_out is not stored but given as the int32 partial sums of a GEMM whose K was split over the
// grid, [splits][rows][Dm]: x_out = fp16(m_out * sum), the rounding the reduce kernel would have done.
template <bool PART>
__global__ __launch_bounds__(256) void add_rmsnorm_quant_kernel(const __half *__restrict__ x_out,
                                                                __half *__restrict__ res,
                                                                const __half *__restrict__ weight,
                                                                float eps, float inv_s,
                                                                int8_t *__restrict__ u_q, int Dm,
                                                                const int32_t *__restrict__ partial, int splits,
                                                                float m_out) {
  const size_t row = blockIdx.x;
  const int ngroups = Dm / 8;
  float vals[RMS_MAX_PER_THREAD][8];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < RMS_MAX_PER_THREAD; ++i) {
    const int g = threadIdx.x + i * 256;
    if (g < ngroups) {
      union {
        uint4 u;
        __half h[8];
      } a, r;
      if constexpr (PART) {
        const size_t rows = gridDim.x;
        v4i v[8][2];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          v[s][0] = v[s][1] = v4i{0, 0, 0, 0};
          if (s < splits) {
            const v4i *src = reinterpret_cast<const v4i *>(partial + ((size_t)s * rows + row) * Dm + (size_t)g * 8);
            v[s][0] = src[0];
            v[s][1] = src[1];
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          int sum = 0;
#pragma unroll
          for (int s = 0; s < 8; ++s) sum += v[s][e >> 2][e & 3];
          a.h[e] = __float2half_rn(static_cast<float>(sum) * m_out);
        }
      } else {
        a.u = *reinterpret_cast<const uint4 *>(x_out + row * Dm + (size_t)g * 8);
      }
      r.u = *reinterpret_cast<const uint4 *>(res + row * Dm + (size_t)g * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const __half s = __float2half_rn(__half2float(a.h[e]) + __half2float(r.h[e]));
        r.h[e] = s;
        const float f = __half2float(s);
        vals[i][e] = f;
        ss += f * f;
      }
      *reinterpret_cast<uint4 *>(res + row * Dm + (size_t)g * 8) = r.u;
    }
  }
  __shared__ float part[4];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = part[0] + part[1] + part[2] + part[3];
  const float rinv = 1.f / sqrtf(tot / static_cast<float>(Dm) + eps);
#pragma unroll
  for (int i = 0; i < RMS_MAX_PER_THREAD; ++i) {
    const int g = threadIdx.x + i * 256;
    if (g < ngroups) {
      union {
        uint4 u;
        __half h[8];
      } wv;
      wv.u = *reinterpret_cast<const uint4 *>(weight + (size_t)g * 8);
      unsigned lo = 0, hi = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        lo |= (static_cast<unsigned>(q8(vals[i][e] * rinv * __half2float(wv.h[e]) * inv_s)) & 0xffu) << (8 * e);
        hi |= (static_cast<unsigned>(q8(vals[i][e + 4] * rinv * __half2float(wv.h[e + 4]) * inv_s)) & 0xffu)
              << (8 * e);
      }
      *reinterpret_cast<uint2 *>(u_q + row * Dm + (size_t)g * 8) = make_uint2(lo, hi);
    }
  }
}

// ------------------------------------------------------------------ per-call scale of x (Appendix K, dynamic row)
__global__ __launch_bounds__(64) void dyn_reset_kernel(unsigned *slot) {
  if (threadIdx.x == 0) *slot = 0u;
}

// max|x| over n halves -> *slot (bits of a non-negative float order like unsigned integers)
__global__ __launch_bounds__(256) void absmax_f16_kernel(const __half *__restrict__ x, size_t n, unsigned *__restrict__ slot) {
  float m = 0.f;
  const size_t stride = (size_t)gridDim.x * 256 * 8;
  for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8; i < n; i += stride) {
    if (i + 8 <= n) {
      union {
        uint4 u;
        __half h[8];
      } v;
      v.u = *reinterpret_cast<const uint4 *>(x + i);
#pragma unroll
      for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(__half2float(v.h[e])));
    } else {
      for (size_t j = i; j < n; ++j) m = fmaxf(m, fabsf(__half2float(x[j])));
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  __shared__ float part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) atomicMax(slot, __float_as_uint(fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]))));
}

// x_q = clamp(rne(fp32(x16) * (1 / s))) with the call's scale
__global__ __launch_bounds__(256) void quantize_f16_dyn_kernel(const __half *__restrict__ x, int8_t *__restrict__ q, size_t n,
                                                               const unsigned *__restrict__ slot) {
  const float inv_s = dyn_inv_scale(slot);
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  if (i + 8 <= n) {
    union {
      uint4 u;
      __half h[8];
    } in;
    in.u = *reinterpret_cast<const uint4 *>(x + i);
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = __half2float(in.h[e]) * inv_s;
    *reinterpret_cast<uint2 *>(q + i) = make_uint2(pack_q8x4(v[0], v[1], v[2], v[3]), pack_q8x4(v[4], v[5], v[6], v[7]));
  } else {
    for (size_t j = i; j < n; ++j) q[j] = static_cast<int8_t>(q8(__half2float(x[j]) * inv_s));
  }
}

// x_proj sums [M, N] int32 -> int8 codes, the multipliers formed from the call's scale:
// columns [0, e0) (s s_W) / so0, [e0, e1) (s s_W) / so1, [e1, N) (s s_W) / so2
__global__ __launch_bounds__(256) void requant_dyn_kernel(const int32_t *__restrict__ acc, int8_t *__restrict__ out, size_t groups,
                                                          int N, int e0, int e1, const unsigned *__restrict__ slot, float s_W,
                                                          float so0, float so1, float so2) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= groups) return;
  const int gn = static_cast<int>(g % (N / 4)) * 4;
  const float m = dyn_multiplier(slot, s_W, gn < e0 ? so0 : (gn < e1 ? so1 : so2));
  const v4i a = *reinterpret_cast<const v4i *>(acc + g * 4);
  const int r[4] = {a[0], a[1], a[2], a[3]};
  *reinterpret_cast<unsigned *>(out + g * 4) = requant_pack4(r, m);
}

// *out = the scale the call used (for callers that want to see it)
__global__ __launch_bounds__(64) void dyn_export_kernel(const unsigned *slot, float *out) {
  if (threadIdx.x == 0) *out = dyn_scale(slot);
}

}  // namespace

int launch_dyn_absmax_f16(const __half *x, size_t n, unsigned *slot, hipStream_t st) {
  hipLaunchKernelGGL(dyn_reset_kernel, dim3(1), dim3(64), 0, st, slot);
  // (few blocks: every block ends in one atomic on the same word, and those serialise)
  const size_t blocks = std::min<size_t>((n + 2047) / 2048, 256);
  hipLaunchKernelGGL(absmax_f16_kernel, dim3((unsigned)(blocks ? blocks : 1)), dim3(256), 0, st, x, n, slot);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_quantize_f16_dyn(const __half *x, int8_t *q, size_t n, const unsigned *slot, hipStream_t st) {
  if (n == 0) return QUAMBA_OK;
  hipLaunchKernelGGL(quantize_f16_dyn_kernel, dim3((unsigned)((n + 2047) / 2048)), dim3(256), 0, st, x, q, n, slot);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_requant_dyn(const int32_t *acc, int8_t *out, int M, int N, int e0, int e1, const unsigned *slot, float s_W,
                       float so0, float so1, float so2, hipStream_t st) {
  const size_t groups = (size_t)M * (N / 4);
  if (groups == 0) return QUAMBA_OK;
  hipLaunchKernelGGL(requant_dyn_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, acc, out, groups, N, e0, e1,
                     slot, s_W, so0, so1, so2);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_dyn_export(const unsigned *slot, float *out, hipStream_t st) {
  hipLaunchKernelGGL(dyn_export_kernel, dim3(1), dim3(64), 0, st, slot, out);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_quantize_f16(const __half *x, int8_t *q, size_t n, float inv_s, hipStream_t st) {
  if (n == 0) return QUAMBA_OK;
  const size_t blocks = (n + 2047) / 2048;
  hipLaunchKernelGGL(quantize_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, q, n, inv_s);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

namespace {
template <int TT>
void conv_prefill_launch(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b, int Bt, int L, int Di,
                         float m_conv, float inv_s_x, float s_xpre, int8_t *x_q, __half *conv_state, hipStream_t st,
                         __half *x16, int x_zero_point, int x_format) {
  dim3 grid((Di / 4 + 255) / 256, (L + TT - 1) / TT, Bt);
  const float zp = static_cast<float>(x_zero_point);
  if (x_format == QUAMBA_XFMT_E4M3)
    hipLaunchKernelGGL((conv_prefill_kernel<OUT_E4M3, TT>), grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, L, Di,
                       m_conv, inv_s_x, s_xpre, x_q, x16, zp, conv_state);
  else if (x_format == QUAMBA_XFMT_LOG2)
    hipLaunchKernelGGL((conv_prefill_kernel<OUT_LOG2, TT>), grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, L, Di,
                       m_conv, inv_s_x, s_xpre, x_q, x16, zp, conv_state);
  else if (x16)
    hipLaunchKernelGGL((conv_prefill_kernel<OUT_F16, TT>), grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, L, Di,
                       m_conv, inv_s_x, s_xpre, x_q, x16, zp, conv_state);
  else if (x_zero_point != 0)
    hipLaunchKernelGGL((conv_prefill_kernel<OUT_ASYM, TT>), grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, L, Di,
                       m_conv, inv_s_x, s_xpre, x_q, x16, zp, conv_state);
  else
    hipLaunchKernelGGL((conv_prefill_kernel<OUT_SYM, TT>), grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, L, Di,
                       m_conv, inv_s_x, s_xpre, x_q, x16, zp, conv_state);
}
}  // namespace

int launch_conv_prefill(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b, int Bt,
                        int L, int Di, float m_conv, float inv_s_x, float s_xpre, int8_t *x_q,
                        __half *conv_state, hipStream_t st, __half *x16, int x_zero_point, int x_format) {
  // Tokens per thread: 8 re-reads the least of the 3-token window and is best when the launch has
  // many waves per SIMD anyway or is tiny; in between (about 4 to 16 M elements, 2048 tokens of the
  // 2.8B shape) 4 gives twice the waves and is 0.5 us faster (measured 8.9 vs 9.4 us; 47.5 vs 46.3 us
  // at 16384 tokens the other way round).
  const size_t elems = (size_t)Bt * L * Di;
  if (elems >= ((size_t)4 << 20) && elems <= ((size_t)16 << 20))
    conv_prefill_launch<4>(xpre_q, ldx, w_q, conv_b, Bt, L, Di, m_conv, inv_s_x, s_xpre, x_q, conv_state, st, x16,
                           x_zero_point, x_format);
  else
    conv_prefill_launch<8>(xpre_q, ldx, w_q, conv_b, Bt, L, Di, m_conv, inv_s_x, s_xpre, x_q, conv_state, st, x16,
                           x_zero_point, x_format);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_conv_step(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b, int Bt,
                     int Di, float s_cw, float s_xpre, float inv_s_x, int8_t *x_q, __half *conv_state,
                     hipStream_t st, __half *x16, int x_zero_point, int x_format) {
  const size_t n = (size_t)Bt * (Di / 4);
  const dim3 grid((unsigned)((n + 255) / 256));
  const float zp = static_cast<float>(x_zero_point);
  if (x_format == QUAMBA_XFMT_E4M3)
    hipLaunchKernelGGL(conv_step_kernel<OUT_E4M3>, grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw,
                       s_xpre, inv_s_x, x_q, x16, zp, conv_state);
  else if (x_format == QUAMBA_XFMT_LOG2)
    hipLaunchKernelGGL(conv_step_kernel<OUT_LOG2>, grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw,
                       s_xpre, inv_s_x, x_q, x16, zp, conv_state);
  else if (x16)
    hipLaunchKernelGGL(conv_step_kernel<OUT_F16>, grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw,
                       s_xpre, inv_s_x, x_q, x16, zp, conv_state);
  else if (x_zero_point != 0)
    hipLaunchKernelGGL(conv_step_kernel<OUT_ASYM>, grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw,
                       s_xpre, inv_s_x, x_q, x16, zp, conv_state);
  else
    hipLaunchKernelGGL(conv_step_kernel<OUT_SYM>, grid, dim3(256), 0, st, xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw,
                       s_xpre, inv_s_x, x_q, x16, zp, conv_state);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_add_rmsnorm_quant(const __half *x_out, __half *res, const __half *weight, float eps,
                             float inv_s, int8_t *u_q, int M, int Dm, hipStream_t st) {
  if (Dm % 8 != 0 || Dm > 8 * 256 * RMS_MAX_PER_THREAD)
    return fail(QUAMBA_EUNSUPPORTED, "add_rmsnorm_quant: d_model=%d must be a multiple of 8 and <= %d", Dm,
                8 * 256 * RMS_MAX_PER_THREAD);
  hipLaunchKernelGGL(add_rmsnorm_quant_kernel<false>, dim3(M), dim3(256), 0, st, x_out, res, weight, eps, inv_s,
                     u_q, Dm, nullptr, 0, 0.f);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_add_rmsnorm_quant_partial(const int32_t *partial, int splits, float m_out, __half *res, const __half *weight,
                                     float eps, float inv_s, int8_t *u_q, int M, int Dm, hipStream_t st) {
  if (Dm % 8 != 0 || Dm > 8 * 256 * RMS_MAX_PER_THREAD)
    return fail(QUAMBA_EUNSUPPORTED, "add_rmsnorm_quant: d_model=%d must be a multiple of 8 and <= %d", Dm,
                8 * 256 * RMS_MAX_PER_THREAD);
  if (!partial || splits < 1 || splits > 8 || !aligned(partial, 16))
    return fail(QUAMBA_EINVAL, "add_rmsnorm_quant: %d partial sums", splits);
  hipLaunchKernelGGL(add_rmsnorm_quant_kernel<true>, dim3(M), dim3(256), 0, st, nullptr, res, weight, eps, inv_s, u_q,
                     Dm, partial, splits, m_out);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace quamba
