// x_proj for a scan input stored in a non-uniform 8-bit format (Appendix K: log2, and the E4M3
// float it names).  The appendix calls the log2 matrix product unsupported by the frameworks it
// used; on this part it has a plain form: every decoded value (a power of two, or a float with four
// significant bits) and every int8 weight code is exact in bfloat16, so the product runs on the
// bf16 matrix units (v_mfma_f32_32x32x16_bf16), products exact, sums in fp32:
//   acc[m, n] = sum_k W_q[n, k] value(x_code[m, k]);   out = clamp(rne(acc * mult)) int8
// The output is skinny (N = dt_rank + 2 d_state <= 320) and K deep, so K is cut over grid.y into
// equal ranges whose fp32 partial sums a second kernel adds in ascending order (a fixed order:
// the result does not depend on scheduling).  A workgroup is 64 rows x all columns: wave w takes
// row tile w % 2 and the column tiles w / 2, w / 2 + 2, ...; operands come straight from global
// memory (a 128-byte line of W holds the 64 k the four k-steps of a slice use, so the cache serves
// three of four requests), the codes are decoded in registers.
#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int FMT>
__device__ __forceinline__ float value_of(unsigned c) {
  return FMT == QUAMBA_XFMT_E4M3 ? decode_e4m3(c) : decode_log2(c);
}

// eight code bytes -> eight bf16 (the upper halves of the fp32 values: exact for these formats)
template <int FMT>
__device__ __forceinline__ bf8 decode8(uint2 c) {
  bf8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const unsigned byte = ((e < 4 ? c.x : c.y) >> (8 * (e & 3))) & 0xffu;
    o[e] = __builtin_bit_cast(__bf16, static_cast<unsigned short>(__float_as_uint(value_of<FMT>(byte)) >> 16));
  }
  return o;
}

struct XfmtEpi {
  int8_t *out_q;
  float *acc;  // optional fp32 sums [M, N]
  int e0, e1;
  float m0, m1, m2;
};

__device__ __forceinline__ void xfmt_emit4(const XfmtEpi &epi, int gm, int gn, int N, const float (&a)[4]) {
  if (epi.acc) *reinterpret_cast<float4 *>(epi.acc + (size_t)gm * N + gn) = make_float4(a[0], a[1], a[2], a[3]);
  const float m = gn < epi.e0 ? epi.m0 : (gn < epi.e1 ? epi.m1 : epi.m2);
  *reinterpret_cast<unsigned *>(epi.out_q + (size_t)gm * N + gn) = pack_q8x4(a[0] * m, a[1] * m, a[2] * m, a[3] * m);
}

// NTW: column tiles per wave (N <= 64 NTW).  partial != nullptr: fp32 sums of this k range go to
// partial[blockIdx.y][M][N]; otherwise the epilogue runs here.
template <int FMT, int NTW>
__global__ __launch_bounds__(256) void xfmt_proj_kernel(const uint8_t *__restrict__ x, const uint16_t *__restrict__ Wb,
                                                        int M, int N, int K, int kc, float *__restrict__ partial,
                                                        XfmtEpi epi) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rt = wave & 1, ch = wave >> 1;
  const int m0 = blockIdx.x * 64 + rt * 32;
  const int k_lo = blockIdx.y * kc, k_hi = min(K, k_lo + kc);
  const int koff = 8 * (lane >> 5);
  // rows and columns past the end are clamped: loaded and multiplied, never stored
  const uint8_t *xrow = x + (size_t)min(m0 + (lane & 31), M - 1) * K + koff;
  const uint16_t *wrow[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j) wrow[j] = Wb + (size_t)min((ch + 2 * j) * 32 + (lane & 31), N - 1) * K + koff;

  f32x16 acc[NTW];
#pragma unroll
  for (int j = 0; j < NTW; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

#pragma unroll 4
  for (int kk = k_lo; kk < k_hi; kk += 16) {
    const bf8 xb = decode8<FMT>(*reinterpret_cast<const uint2 *>(xrow + kk));
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
      if ((ch + 2 * j) * 32 < N) {  // wave-uniform
        const bf8 wb = *reinterpret_cast<const bf8 *>(wrow[j] + kk);
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb, xb, acc[j], 0, 0, 0);
      }
    }
  }
  // register r of lane l: column 8 (r / 4) + 4 (l / 32) + r % 4 of the tile, row l % 32
  const int gm = m0 + (lane & 31);
  if (gm >= M) return;
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int gn = (ch + 2 * j) * 32 + 8 * g + 4 * (lane >> 5);
      if (gn >= N) continue;  // N is a multiple of 4: a group is all in or all out
      const float a[4] = {acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]};
      if (partial)
        *reinterpret_cast<float4 *>(partial + ((size_t)blockIdx.y * M + gm) * N + gn) = make_float4(a[0], a[1], a[2], a[3]);
      else
        xfmt_emit4(epi, gm, gn, N, a);
    }
  }
}

// Sum of the k-range partials in ascending order + epilogue; one thread per group of four columns.
__global__ __launch_bounds__(256) void xfmt_reduce_kernel(const float *__restrict__ partial, int splits, int M, int N,
                                                          XfmtEpi epi) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t groups = (size_t)M * (N / 4);
  if (g >= groups) return;
  const int gm = static_cast<int>(g / (N / 4));
  const int gn = static_cast<int>(g % (N / 4)) * 4;
  float4 v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    v[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s < splits) v[s] = *reinterpret_cast<const float4 *>(partial + ((size_t)s * M + gm) * N + gn);
  }
  float a[4] = {v[0].x, v[0].y, v[0].z, v[0].w};
#pragma unroll
  for (int s = 1; s < 8; ++s) {
    if (s < splits) {
      a[0] = __fadd_rn(a[0], v[s].x);
      a[1] = __fadd_rn(a[1], v[s].y);
      a[2] = __fadd_rn(a[2], v[s].z);
      a[3] = __fadd_rn(a[3], v[s].w);
    }
  }
  xfmt_emit4(epi, gm, gn, N, a);
}

__global__ __launch_bounds__(256) void x_encode_kernel(const float *__restrict__ v, size_t n, float inv_s, int fmt,
                                                       uint8_t *__restrict__ codes) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float t = __fmul_rn(v[i], inv_s);
  codes[i] = static_cast<uint8_t>(fmt == QUAMBA_XFMT_E4M3 ? encode_e4m3(t) : encode_log2(t));
}

__global__ __launch_bounds__(256) void i8_to_bf16_kernel(const int8_t *__restrict__ q, size_t n, uint16_t *__restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  out[i] = static_cast<uint16_t>(__float_as_uint(static_cast<float>(q[i])) >> 16);  // |q| <= 128: exact in 8 bits
}

template <int FMT>
int run_xfmt(const uint8_t *x, const uint16_t *Wb, int M, int N, int K, int kc, int splits, float *partial,
             const XfmtEpi &epi, hipStream_t st) {
  const dim3 grid((unsigned)((M + 63) / 64), (unsigned)splits);
  const int ntw = (N + 63) / 64;
  switch (ntw) {
    case 1: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 1>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    case 2: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 2>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    case 3: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 3>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    case 4: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 4>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    default: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 5>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
  }
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace

int launch_xfmt_proj(int format, const uint8_t *x_code, int M, int N, int K, const uint16_t *W_bf16, int e0, int e1,
                     float m0, float m1, float m2, int8_t *out_q, float *acc_f32, void *ws, size_t ws_bytes,
                     hipStream_t st) {
  if (format != QUAMBA_XFMT_E4M3 && format != QUAMBA_XFMT_LOG2) return fail(QUAMBA_EINVAL, "x format %d", format);
  if (!x_code || !W_bf16 || !out_q) return fail(QUAMBA_EINVAL, "xfmt_proj: NULL pointer");
  if (M < 1 || N < 4 || N > 320 || N % 4 || K < 16 || K % 16 || e0 % 4 || e1 % 4)
    return fail(QUAMBA_EUNSUPPORTED, "xfmt_proj: M=%d N=%d K=%d (N a multiple of 4 up to 320, K a multiple of 16)", M, N, K);
  if (!aligned(x_code, 16) || !aligned(W_bf16, 16) || !aligned(out_q, 4) || (acc_f32 && !aligned(acc_f32, 16)))
    return fail(QUAMBA_EINVAL, "xfmt_proj: pointers must be 16-byte aligned");
  // K ranges: enough workgroups for the chip, ranges whole multiples of 16, at most 8 and at least 64 deep
  const int row_blocks = (M + 63) / 64;
  int splits = 1;
  if (ws && aligned(ws, 256)) {
    splits = std::min(8, std::max(1, 256 / row_blocks));
    while (splits > 1 && ((K / 16) / splits < 4 || (size_t)splits * M * N * sizeof(float) > ws_bytes)) --splits;
  }
  const int kc = ((K / 16 + splits - 1) / splits) * 16;
  splits = (K + kc - 1) / kc;
  const XfmtEpi epi{out_q, acc_f32, e0, e1, m0, m1, m2};
  float *partial = splits > 1 ? static_cast<float *>(ws) : nullptr;
  int rc = format == QUAMBA_XFMT_E4M3 ? run_xfmt<QUAMBA_XFMT_E4M3>(x_code, W_bf16, M, N, K, kc, splits, partial, epi, st)
                                      : run_xfmt<QUAMBA_XFMT_LOG2>(x_code, W_bf16, M, N, K, kc, splits, partial, epi, st);
  if (rc != QUAMBA_OK || splits == 1) return rc;
  const size_t groups = (size_t)M * (N / 4);
  hipLaunchKernelGGL(xfmt_reduce_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, partial, splits, M, N,
                     epi);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_x_encode(int format, const float *v, size_t n, float inv_s, uint8_t *codes, hipStream_t st) {
  if (format != QUAMBA_XFMT_E4M3 && format != QUAMBA_XFMT_LOG2) return fail(QUAMBA_EINVAL, "x format %d", format);
  if (n == 0) return QUAMBA_OK;
  if (!v || !codes) return fail(QUAMBA_EINVAL, "x_encode: NULL pointer");
  hipLaunchKernelGGL(x_encode_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, v, n, inv_s, format, codes);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_i8_to_bf16(const int8_t *q, size_t n, uint16_t *out, hipStream_t st) {
  if (n == 0) return QUAMBA_OK;
  hipLaunchKernelGGL(i8_to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, q, n, out);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace quamba
