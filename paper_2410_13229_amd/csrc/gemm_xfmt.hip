// x_proj for a scan input stored in a non-uniform 8-bit format (Appendix K: log2, and the E4M3
// float it names).  The appendix calls the log2 matrix product unsupported by the frameworks it
// used; on this part it has a plain form: every decoded value (a power of two, or a float with four
// significant bits) and every int8 weight code is exact in bfloat16, so the product runs on the
// bf16 matrix units (v_mfma_f32_32x32x16_bf16), products exact, sums in fp32:
//   acc[m, n] = sum_k W_q[n, k] value(x_code[m, k]);   out = clamp(rne(acc * mult)) int8
// The output is skinny (N = dt_rank + 2 d_state <= 320) and K deep, so K is cut over grid.y into
// equal ranges whose fp32 partial sums a second kernel adds in ascending order (a fixed order:
// the result does not depend on scheduling).  A workgroup is 64 (or 128) rows x all columns: wave w
// takes row tile(s) w % 2 and the column tiles w / 2, w / 2 + 2, ...; operands come straight from global
// memory and the codes are decoded in registers.  So that those loads are whole cache lines, the
// bf16 weight is stored in the order the matrix unit consumes it (the calibration writes it):
//   W_blk[(s N + n) 16 + 8 h + j] = W_q[n, 32 (s / 2) + 16 h + 8 (s % 2) + j],  s = k-step, h = lane / 32, j < 8
// a wave-level load of one k-step and column tile is then 1 KB contiguous, and a lane's 16 code bytes
// x[m, 32 q + 16 h ..] serve the two k-steps 2 q and 2 q + 1 (a sum does not care in which order the
// k are visited as long as both operands agree).
#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// eight code bytes -> eight bf16 (the upper halves of the fp32 values: exact for these formats).
// E4M3 is the float8 format this part's converter implements (v_cvt_pk_f32_fp8: two codes -> two fp32);
// a byte permute then gathers the two upper halves.  log2: the exponent field is 127 - e.
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <int FMT>
__device__ __forceinline__ bf8 decode8(uint2 c) {
  union {
    bf8 v;
    unsigned w[4];
  } o;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const unsigned word = q < 2 ? c.x : c.y;
    if constexpr (FMT == QUAMBA_XFMT_E4M3) {
      const f32x2 f = (q & 1) ? __builtin_amdgcn_cvt_pk_f32_fp8(word, true) : __builtin_amdgcn_cvt_pk_f32_fp8(word, false);
      o.w[q] = __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);
    } else {
      // two codes at once, one per 16-bit half: bf16 bits = (127 - e) << 7 | sign << 15 (e = 127, the zero code, gives 0)
      const unsigned pair = __builtin_amdgcn_perm(0u, word, (q & 1) ? 0x0c030c02u : 0x0c010c00u);
      o.w[q] = ((0x007f007fu - (pair & 0x007f007fu)) << 7) | ((pair & 0x00800080u) << 8);
    }
  }
  return o.v;
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

// NTW: column tiles per wave (a workgroup covers 64 NTW columns, grid.z walks the column groups);
// RT: row tiles per wave (a workgroup covers 64 RT rows).
// The loop takes U k-steps at a time and requests all their operands before the first product, so
// a wave has (RT + 2 NTW) U loads in flight instead of paying one memory round trip per k-step.
// partial != nullptr: fp32 sums of this k range go to partial[blockIdx.y][M][N]; otherwise the
// epilogue runs here.
template <int FMT, int NTW, int RT>
__global__ __launch_bounds__(256) void xfmt_proj_kernel(const uint8_t *__restrict__ x, const uint16_t *__restrict__ Wb,
                                                        int M, int N, int K, int kc, float *__restrict__ partial,
                                                        XfmtEpi epi) {
  constexpr int U = RT == 1 ? 4 : 2;  // pairs of k-steps (32 k) taken at a time
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int rt = wave & 1, ch = wave >> 1;
  const int ct0 = blockIdx.z * (2 * NTW);  // first column tile of this workgroup
  const int m0 = blockIdx.x * (64 * RT) + rt * (32 * RT);
  const int k_lo = blockIdx.y * kc, k_hi = min(K, k_lo + kc);
  const int half = lane >> 5;
  // rows and columns past the end are clamped: loaded and multiplied, never stored
  const uint8_t *xrow[RT];
#pragma unroll
  for (int i = 0; i < RT; ++i) xrow[i] = x + (size_t)min(m0 + 32 * i + (lane & 31), M - 1) * K + 16 * half;
  const uint16_t *wcol[NTW];  // + (k-step) N 16
#pragma unroll
  for (int j = 0; j < NTW; ++j) wcol[j] = Wb + (size_t)min((ct0 + ch + 2 * j) * 32 + (lane & 31), N - 1) * 16 + 8 * half;
  const size_t wstep = (size_t)N * 16;

  f32x16 acc[RT][NTW];
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int j = 0; j < NTW; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  auto load = [&](int k0, uint4 (&xc)[U][RT], bf8 (&wb)[2 * U][NTW]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kk = min(k0 + 32 * u, k_hi - 32);  // past the range: a valid address, loaded, not used
#pragma unroll
      for (int i = 0; i < RT; ++i) xc[u][i] = *reinterpret_cast<const uint4 *>(xrow[i] + kk);
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
          if ((ct0 + ch + 2 * j) * 32 < N)  // wave-uniform
            wb[2 * u + e][j] = *reinterpret_cast<const bf8 *>(wcol[j] + (size_t)(kk / 16 + e) * wstep);
    }
  };
  auto compute = [&](int k0, const uint4 (&xc)[U][RT], const bf8 (&wb)[2 * U][NTW]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (k0 + 32 * u < k_hi) {  // wave-uniform
#pragma unroll
        for (int i = 0; i < RT; ++i) {
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const bf8 xb = decode8<FMT>(e == 0 ? make_uint2(xc[u][i].x, xc[u][i].y) : make_uint2(xc[u][i].z, xc[u][i].w));
#pragma unroll
            for (int j = 0; j < NTW; ++j)
              if ((ct0 + ch + 2 * j) * 32 < N)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[2 * u + e][j], xb, acc[i][j], 0, 0, 0);
          }
        }
      }
    }
  };
  // two operand sets: the loads of the next U pairs of k-steps are in flight under the products of these
  uint4 xc0[U][RT], xc1[U][RT];
  bf8 wb0[2 * U][NTW], wb1[2 * U][NTW];
  int k0 = k_lo;
  if (k0 < k_hi) load(k0, xc0, wb0);
  while (k0 < k_hi) {
    const int k1 = k0 + 32 * U;
    if (k1 < k_hi) load(k1, xc1, wb1);
    compute(k0, xc0, wb0);
    if (k1 >= k_hi) break;
    const int k2 = k1 + 32 * U;
    if (k2 < k_hi) load(k2, xc0, wb0);
    compute(k1, xc1, wb1);
    k0 = k2;
  }
  // register r of lane l: column 8 (r / 4) + 4 (l / 32) + r % 4 of the tile, row l % 32
#pragma unroll
  for (int i = 0; i < RT; ++i) {
    const int gm = m0 + 32 * i + (lane & 31);
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int gn = (ct0 + ch + 2 * j) * 32 + 8 * g + 4 * (lane >> 5);
        if (gn >= N) continue;  // N is a multiple of 4: a group is all in or all out
        const float a[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        if (partial)
          *reinterpret_cast<float4 *>(partial + ((size_t)blockIdx.y * M + gm) * N + gn) = make_float4(a[0], a[1], a[2], a[3]);
        else
          xfmt_emit4(epi, gm, gn, N, a);
      }
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

// int8 codes [N, K] -> bfloat16 in the order the product kernel consumes (see the top of this file)
__global__ __launch_bounds__(256) void i8_to_bf16_kernel(const int8_t *__restrict__ q, int N, int K, uint16_t *__restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;  // index into out
  if (i >= (size_t)N * K) return;
  const int p = static_cast<int>(i & 15), n = static_cast<int>((i >> 4) % N), s = static_cast<int>((i >> 4) / N);
  const int k = 32 * (s >> 1) + 16 * (p >> 3) + 8 * (s & 1) + (p & 7);
  out[i] = static_cast<uint16_t>(__float_as_uint(static_cast<float>(q[(size_t)n * K + k])) >> 16);  // |q| <= 128: exact in 8 bits
}

template <int FMT, int RT>
int run_xfmt(const uint8_t *x, const uint16_t *Wb, int M, int N, int K, int kc, int splits, float *partial,
             const XfmtEpi &epi, hipStream_t st) {
  // few workgroups: one column tile per wave and the column groups spread over grid.z
  const int row_blocks = (M + 64 * RT - 1) / (64 * RT);
  const int ntw = (row_blocks * splits < 128) ? 1 : (N + 63) / 64;
  const dim3 grid((unsigned)row_blocks, (unsigned)splits, (unsigned)((N + 64 * ntw - 1) / (64 * ntw)));
  switch (ntw) {
    case 1: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 1, RT>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    case 2: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 2, RT>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    case 3: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 3, RT>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    case 4: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 4, RT>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
    default: hipLaunchKernelGGL((xfmt_proj_kernel<FMT, 5, RT>), grid, dim3(256), 0, st, x, Wb, M, N, K, kc, partial, epi); break;
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
  if (M < 1 || N < 4 || N > 320 || N % 4 || K < 32 || K % 32 || e0 % 4 || e1 % 4)
    return fail(QUAMBA_EUNSUPPORTED, "xfmt_proj: M=%d N=%d K=%d (N a multiple of 4 up to 320, K a multiple of 32)", M, N, K);
  if (!aligned(x_code, 16) || !aligned(W_bf16, 16) || !aligned(out_q, 4) || (acc_f32 && !aligned(acc_f32, 16)))
    return fail(QUAMBA_EINVAL, "xfmt_proj: pointers must be 16-byte aligned");
  // K ranges: enough workgroups for the chip, ranges whole multiples of 32, at most 8 and at least 128 deep
  // many rows: two row tiles per wave halve the weight traffic (every row block streams all of W)
  const int rt = M >= 4096 ? 2 : 1;
  const int row_blocks = (M + 64 * rt - 1) / (64 * rt);
  int splits = 1;
  if (ws && aligned(ws, 256)) {
    splits = std::min(8, std::max(1, 256 / row_blocks));
    while (splits > 1 && ((K / 32) / splits < 4 || (size_t)splits * M * N * sizeof(float) > ws_bytes)) --splits;
  }
  const int kc = ((K / 32 + splits - 1) / splits) * 32;
  splits = (K + kc - 1) / kc;
  const XfmtEpi epi{out_q, acc_f32, e0, e1, m0, m1, m2};
  float *partial = splits > 1 ? static_cast<float *>(ws) : nullptr;
  int rc;
  if (format == QUAMBA_XFMT_E4M3)
    rc = rt == 2 ? run_xfmt<QUAMBA_XFMT_E4M3, 2>(x_code, W_bf16, M, N, K, kc, splits, partial, epi, st)
                 : run_xfmt<QUAMBA_XFMT_E4M3, 1>(x_code, W_bf16, M, N, K, kc, splits, partial, epi, st);
  else
    rc = rt == 2 ? run_xfmt<QUAMBA_XFMT_LOG2, 2>(x_code, W_bf16, M, N, K, kc, splits, partial, epi, st)
                 : run_xfmt<QUAMBA_XFMT_LOG2, 1>(x_code, W_bf16, M, N, K, kc, splits, partial, epi, st);
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

int launch_i8_to_bf16(const int8_t *q, int N, int K, uint16_t *out, hipStream_t st) {
  if (N < 1 || K < 32 || K % 32) return fail(QUAMBA_EUNSUPPORTED, "bf16 weight copy: K=%d must be a multiple of 32", K);
  const size_t n = (size_t)N * K;
  hipLaunchKernelGGL(i8_to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, q, N, K, out);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace quamba
