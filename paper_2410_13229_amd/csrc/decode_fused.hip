// First kernel of a block in generation with few sequences (M <= 4): residual add + RMSNorm +
// quantization (Section 4.3 "Fused RMSNorm"), the int8 input projection, and the causal conv step
// with SiLU and requantization (Section 4.3 "Fused causal convolution") in one launch.  With a
// handful of rows every one of these is a few microseconds of launch latency and almost no work,
// and each output column of in_proj needs only its own conv window, so the three chain inside
// one workgroup:
//   s = fp16(out_prev + res_in)            (workgroup 0 stores it as the new residual)
//   u_q = q(RMSNorm(s) * w, 1/s_u)         (recomputed by every workgroup into LDS: M rows only)
//   acc[m, n] = sum_k u_q[m, k] W_in[n, k]  for the workgroup's 16 columns n (4 per wave)
//   n <  Di: xpre_q = q(acc m_in_x) -> conv step on that channel's window -> x_q[m, n]
//   n >= Di: z_q[m, n - Di] = q(acc m_in_z)
// The weights stream once, 1 KB of a row per wave-level load, multiplied with v_dot4_i32_i8.
#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

template <int MB>
__global__ __launch_bounds__(256) void decode_in_kernel(DecodeInArgs p) {
  extern __shared__ __attribute__((aligned(16))) int8_t sA[];  // [MB][Dm] int8 codes of u, rows past M zero
  __shared__ float part[4][MB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Dm = p.Dm, Di = p.Di, M = p.M;
  const int groups = Dm / 8;  // pieces of 8 halves
  const int n0 = blockIdx.x * 16 + wave * 4;  // wave w owns columns n0 .. n0+3 of in_proj
  const int N = 2 * Di;
  const int nchunks = Dm / 16;
  // The first weight pieces (up to three rounds: all of K up to 3072) are requested before anything
  // else, so that they stream in while the block input is normalised and quantized.
  constexpr int PF = 3;
  v4i wpre[PF][4];
#pragma unroll
  for (int r = 0; r < PF; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ch = min(lane + 64 * r, nchunks - 1);
      wpre[r][j] = *reinterpret_cast<const v4i *>(p.W_in + (size_t)min(n0 + j, N - 1) * Dm + ch * 16);
    }

  if (p.u_q) {  // already quantized input
#pragma unroll
    for (int m = 0; m < MB; ++m)
      for (int ch = tid; ch < Dm / 16; ch += 256) {
        v4i v = {0, 0, 0, 0};
        if (m < M) v = *reinterpret_cast<const v4i *>(p.u_q + (size_t)m * Dm + ch * 16);
        *reinterpret_cast<v4i *>(sA + (size_t)m * Dm + ch * 16) = v;
      }
  } else {
    // One sweep: the fp16 sums s = fp16(out + res) stay in registers (8 halves per 16-byte word) between
    // the reduction and the scaling; a thread owns at most SW words per row (d_model <= 4096 with 2).
    constexpr int SW = 2;
    const bool one_sweep = groups <= SW * 256;
    uint4 keep[MB][SW];
    float ss[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) ss[m] = 0.f;
    auto load_sum = [&](int m, int g) -> uint4 {
      union {
        uint4 u;
        __half h[8];
      } a, r;
      a.u = *reinterpret_cast<const uint4 *>(p.out_prev + (size_t)m * Dm + (size_t)g * 8);
      r.u = *reinterpret_cast<const uint4 *>(p.res_in + (size_t)m * Dm + (size_t)g * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) r.h[e] = __float2half_rn(__half2float(a.h[e]) + __half2float(r.h[e]));
      return r.u;
    };
#pragma unroll
    for (int it = 0; it < (SW > 1 ? SW : 1); ++it) {
      const int g = tid + it * 256;
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        keep[m][it] = make_uint4(0u, 0u, 0u, 0u);
        if (one_sweep && m < M && g < groups) keep[m][it] = load_sum(m, g);
      }
    }
    if (one_sweep) {
#pragma unroll
      for (int it = 0; it < SW; ++it) {
        const int g = tid + it * 256;
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          if (m < M && g < groups) {
            union {
              uint4 u;
              __half h[8];
            } r;
            r.u = keep[m][it];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float f = __half2float(r.h[e]);
              ss[m] += f * f;
            }
            if (blockIdx.x == 0) *reinterpret_cast<uint4 *>(p.res_out + (size_t)m * Dm + (size_t)g * 8) = r.u;
          }
        }
      }
    } else {
      for (int g = tid; g < groups; g += 256) {
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          if (m < M) {
            union {
              uint4 u;
              __half h[8];
            } r;
            r.u = load_sum(m, g);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float f = __half2float(r.h[e]);
              ss[m] += f * f;
            }
            if (blockIdx.x == 0) *reinterpret_cast<uint4 *>(p.res_out + (size_t)m * Dm + (size_t)g * 8) = r.u;
          }
        }
      }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      float v = ss[m];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
      if (lane == 0) part[wave][m] = v;
    }
    __syncthreads();
    float rinv[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
      rinv[m] = 1.f / sqrtf((part[0][m] + part[1][m] + part[2][m] + part[3][m]) / static_cast<float>(Dm) + p.eps);
    // normalise, scale, quantize into LDS (rows past M: zero codes)
    auto emit = [&](int m, int g, uint4 sum, const uint4 &wword) {
      union {
        uint4 u;
        __half h[8];
      } r, wv;
      r.u = sum;
      wv.u = wword;
      float v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = __half2float(r.h[e]) * rinv[m] * __half2float(wv.h[e]) * p.inv_s_u;
      *reinterpret_cast<uint2 *>(sA + (size_t)m * Dm + (size_t)g * 8) =
          make_uint2(pack_q8x4(v[0], v[1], v[2], v[3]), pack_q8x4(v[4], v[5], v[6], v[7]));
    };
    if (one_sweep) {
#pragma unroll
      for (int it = 0; it < SW; ++it) {
        const int g = tid + it * 256;
        if (g < groups) {
          const uint4 wword = *reinterpret_cast<const uint4 *>(p.norm_w + (size_t)g * 8);
#pragma unroll
          for (int m = 0; m < MB; ++m) {
            if (m < M) emit(m, g, keep[m][it], wword);
            else *reinterpret_cast<uint2 *>(sA + (size_t)m * Dm + (size_t)g * 8) = make_uint2(0u, 0u);
          }
        }
      }
    } else {  // second sweep over the same (cache-resident) rows
      for (int g = tid; g < groups; g += 256) {
        const uint4 wword = *reinterpret_cast<const uint4 *>(p.norm_w + (size_t)g * 8);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          if (m < M) emit(m, g, load_sum(m, g), wword);
          else *reinterpret_cast<uint2 *>(sA + (size_t)m * Dm + (size_t)g * 8) = make_uint2(0u, 0u);
        }
      }
    }
  }
  __syncthreads();

  // in_proj for 16 columns: the lanes of a wave split K in 16-byte pieces
  int acc[MB][4];
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[m][j] = 0;
  auto mac = [&](int ch, const v4i (&w)[4]) {
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      const v4i a = *reinterpret_cast<const v4i *>(sA + (size_t)m * Dm + ch * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[m][j] = __builtin_amdgcn_sdot4(a[e], w[j][e], acc[m][j], false);
    }
  };
  if (n0 < N) {
#pragma unroll
    for (int r = 0; r < PF; ++r)
      if (lane + 64 * r < nchunks) mac(lane + 64 * r, wpre[r]);
    for (int ch = lane + 64 * PF; ch < nchunks; ch += 64) {
      v4i w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = *reinterpret_cast<const v4i *>(p.W_in + (size_t)(n0 + j) * Dm + ch * 16);
      mac(ch, w);
    }
  }
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[m][j] = wave_sum(acc[m][j]);  // every lane holds the sum
  // lane m finishes row m of this wave's four columns
  if (n0 < N && lane < M) {
    int a[4] = {0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < MB; ++m)
      if (lane == m) {
        a[0] = acc[m][0];
        a[1] = acc[m][1];
        a[2] = acc[m][2];
        a[3] = acc[m][3];
      }
    const int m = lane;
    if (p.acc_in) *reinterpret_cast<v4i *>(p.acc_in + (size_t)m * N + n0) = v4i{a[0], a[1], a[2], a[3]};
    if (n0 < Di) {
      const unsigned xpre = requant_pack4(a, p.m_in_x);
      *reinterpret_cast<unsigned *>(p.xz_q + (size_t)m * N + n0) = xpre;
      *reinterpret_cast<unsigned *>(p.x_q + (size_t)m * Di + n0) =
          conv_step4(xpre, p.conv_w + (size_t)n0 * 4, p.conv_b + n0, p.conv_state + ((size_t)m * Di + n0) * 3, p.s_cw,
                     p.s_xpre, p.inv_s_x);
    } else {
      *reinterpret_cast<unsigned *>(p.xz_q + (size_t)m * N + n0) = requant_pack4(a, p.m_in_z);
    }
  }
}

}  // namespace

int launch_decode_in(const DecodeInArgs &a, hipStream_t st) {
  if (a.M < 1 || a.M > 4) return fail(QUAMBA_EUNSUPPORTED, "decode_in: M=%d outside 1..4", a.M);
  if (a.Dm % 16 || a.Di % 4 || a.Dm > 8192)
    return fail(QUAMBA_EUNSUPPORTED, "decode_in: d_model=%d must be a multiple of 16 and <= 8192, d_inner a multiple of 4",
                a.Dm);
  const int mb = a.M <= 1 ? 1 : (a.M <= 2 ? 2 : 4);
  const size_t lds = (size_t)mb * a.Dm;
  const dim3 grid((2 * a.Di + 15) / 16), block(256);
  switch (mb) {
    case 1: hipLaunchKernelGGL(decode_in_kernel<1>, grid, block, lds, st, a); break;
    case 2: hipLaunchKernelGGL(decode_in_kernel<2>, grid, block, lds, st, a); break;
    default: hipLaunchKernelGGL(decode_in_kernel<4>, grid, block, lds, st, a); break;
  }
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace quamba
