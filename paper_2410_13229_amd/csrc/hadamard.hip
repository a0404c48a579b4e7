// Fused fast Hadamard transform + int8 quantization of the gated scan output (Section 4.2
// "SSM outputs", Eq. 3; Section 3.3): per token row, yH = H_n g, yH_q = clamp(rne(yH / s_y)).
//
// n = k * 2^m with k in {1, 12, 20} and H_n = H_k (x) H_{2^m} (index = a * 2^m + b): the
// 2^m part is the Sylvester / natural-order Walsh-Hadamard matrix, done as butterflies; the
// k part (Section 3.3: a known Hadamard matrix of non-power-of-two order) is the first Paley
// construction for q = k - 1 prime, applied as a dense +-1 product of order k.
//
// One workgroup per row.  The row sits in LDS as fp32; each pass gathers 2^r (or k) elements
// per work item at a power-of-two stride, transforms them in registers and scatters them back.
// The last pass covers the lowest four index bits, so every work item ends with 16 adjacent
// outputs, which it scales, rounds, clamps and stores as one 16-byte word.  The LDS row is
// padded by 4 floats every 16 so that this 16-byte-per-lane pass is bank-conflict free.
#include "common.h"

namespace quamba {
namespace {

constexpr int HT = 256;  // threads per row

__device__ __forceinline__ int pad(int i) { return i + ((i >> 4) << 2); }

// Sign pattern of the Paley-I Hadamard matrix of order Q+1, Q prime, Q = 3 (mod 4):
// H = I + S, S[0][j] = +1, S[i][0] = -1, S[i+1][j+1] = chi(i - j) (Legendre symbol mod Q).
// neg[a] has bit b set when H[a][b] = -1.
template <int Q>
struct Paley {
  unsigned neg[Q + 1];
  constexpr Paley() : neg{} {
    bool residue[Q] = {};
    for (int i = 1; i < Q; ++i) residue[(i * i) % Q] = true;
    for (int a = 0; a <= Q; ++a) {
      unsigned bits = 0;
      for (int b = 0; b <= Q; ++b) {
        bool minus = false;
        if (a == 0) {
          minus = false;
        } else if (b == 0) {
          minus = true;
        } else if (a != b) {
          const int diff = ((a - 1) - (b - 1) + Q) % Q;
          minus = !residue[diff];
        }
        if (minus) bits |= 1u << b;
      }
      neg[a] = bits;
    }
  }
};

template <int K>
__device__ __forceinline__ void order_k_pass(float *row, int logm) {
  if constexpr (K > 1) {
    constexpr Paley<K - 1> tab{};
    const int items = 1 << logm;
    for (int w = threadIdx.x; w < items; w += HT) {
      float v[K], o[K];
#pragma unroll
      for (int a = 0; a < K; ++a) v[a] = row[pad((a << logm) | w)];
#pragma unroll
      for (int a = 0; a < K; ++a) {
        float s = 0.f;
#pragma unroll
        for (int b = 0; b < K; ++b) s += ((tab.neg[a] >> b) & 1u) ? -v[b] : v[b];
        o[a] = s;
      }
#pragma unroll
      for (int a = 0; a < K; ++a) row[pad((a << logm) | w)] = o[a];
    }
    __syncthreads();
  }
}

template <int R>
__device__ __forceinline__ void butterflies(float (&v)[1 << R]) {
#pragma unroll
  for (int len = 1; len < (1 << R); len <<= 1)
#pragma unroll
    for (int i = 0; i < (1 << R); ++i)
      if ((i & len) == 0) {
        const float a = v[i], b = v[i + len];
        v[i] = a + b;
        v[i + len] = a - b;
      }
}

// Butterflies over index bits [s, s+R) of the whole row.
template <int R>
__device__ __forceinline__ void radix_pass(float *row, int n, int s) {
  if constexpr (R > 0) {
    const int items = n >> R;
    for (int w = threadIdx.x; w < items; w += HT) {
      const int low = w & ((1 << s) - 1);
      const int base = ((w >> s) << (s + R)) | low;
      float v[1 << R];
#pragma unroll
      for (int j = 0; j < (1 << R); ++j) v[j] = row[pad(base + (j << s))];
      butterflies<R>(v);
#pragma unroll
      for (int j = 0; j < (1 << R); ++j) row[pad(base + (j << s))] = v[j];
    }
    __syncthreads();
  }
}

__device__ __forceinline__ unsigned q8u(float v) {
  v = __builtin_rintf(v);
  v = fminf(fmaxf(v, -128.f), 127.f);
  return static_cast<unsigned>(static_cast<int>(v)) & 0xffu;
}

template <int K, int LOGM, typename TIn>
__global__ __launch_bounds__(HT) void hadamard_quant_kernel(const TIn *__restrict__ g, float inv_s,
                                                            int8_t *__restrict__ out,
                                                            float *__restrict__ out_f32) {
  static_assert(LOGM >= 4, "the last pass owns the low four index bits");
  constexpr int n = K << LOGM;
  extern __shared__ __attribute__((aligned(16))) float row[];
  const size_t r = blockIdx.x;
  const TIn *src = g + r * n;

  for (int i = threadIdx.x * 8; i < n; i += HT * 8) {
    float *dst = row + pad(i);
    if constexpr (sizeof(TIn) == 2) {
      union {
        uint4 u;
        __half h[8];
      } in;
      in.u = *reinterpret_cast<const uint4 *>(src + i);
      *reinterpret_cast<float4 *>(dst) = make_float4(__half2float(in.h[0]), __half2float(in.h[1]),
                                                     __half2float(in.h[2]), __half2float(in.h[3]));
      *reinterpret_cast<float4 *>(dst + 4) = make_float4(__half2float(in.h[4]), __half2float(in.h[5]),
                                                         __half2float(in.h[6]), __half2float(in.h[7]));
    } else {
      *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src + i);
      *reinterpret_cast<float4 *>(dst + 4) = *reinterpret_cast<const float4 *>(src + i + 4);
    }
  }
  __syncthreads();

  order_k_pass<K>(row, LOGM);

  // index bits [4, LOGM) in up to three passes of at most 5 bits, high bits first
  constexpr int HI = LOGM - 4;
  constexpr int NP = (HI + 4) / 5;
  constexpr int R0 = NP > 0 ? (HI + NP - 1) / NP : 0;
  constexpr int R1 = NP > 1 ? (HI - R0 + NP - 2) / (NP - 1) : 0;
  constexpr int R2 = NP > 2 ? HI - R0 - R1 : 0;
  static_assert(R0 + R1 + R2 == HI && NP <= 3, "pass schedule");
  radix_pass<R0>(row, n, LOGM - R0);
  radix_pass<R1>(row, n, LOGM - R0 - R1);
  radix_pass<R2>(row, n, 4);

  // last pass: bits [0, 4), fused with scale / round / clamp / pack
  for (int w = threadIdx.x; w < n / 16; w += HT) {
    float v[16];
    const float *p = row + pad(w * 16);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 f = reinterpret_cast<const float4 *>(p)[q];
      v[4 * q] = f.x;
      v[4 * q + 1] = f.y;
      v[4 * q + 2] = f.z;
      v[4 * q + 3] = f.w;
    }
    butterflies<4>(v);
    if (out) {
      unsigned pk[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        pk[q] = q8u(v[4 * q] * inv_s) | (q8u(v[4 * q + 1] * inv_s) << 8) | (q8u(v[4 * q + 2] * inv_s) << 16) |
                (q8u(v[4 * q + 3] * inv_s) << 24);
      *reinterpret_cast<uint4 *>(out + r * n + (size_t)w * 16) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
    if (out_f32) {
      float *o = out_f32 + r * n + (size_t)w * 16;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        reinterpret_cast<float4 *>(o)[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
  }
}

template <int K, int LOGM, typename TIn>
int run(const TIn *g, int M, float inv_s, int8_t *out, float *out_f32, hipStream_t st) {
  constexpr int n = K << LOGM;
  constexpr size_t lds = (size_t)(n + n / 4) * sizeof(float);
  static bool attr_set = false;
  if (lds > 64 * 1024 && !attr_set) {
    QUAMBA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&hadamard_quant_kernel<K, LOGM, TIn>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL((hadamard_quant_kernel<K, LOGM, TIn>), dim3(M), dim3(HT), lds, st, g, inv_s, out, out_f32);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

template <int K, typename TIn>
int dispatch_m(int m, const TIn *g, int M, float inv_s, int8_t *out, float *out_f32, hipStream_t st) {
  switch (m) {
#define QUAMBA_CASE(LM) \
  case LM:              \
    return run<K, LM, TIn>(g, M, inv_s, out, out_f32, st);
    QUAMBA_CASE(4)
    QUAMBA_CASE(5)
    QUAMBA_CASE(6)
    QUAMBA_CASE(7)
    QUAMBA_CASE(8)
    QUAMBA_CASE(9)
    QUAMBA_CASE(10)
    default:
      break;
  }
  if constexpr (K == 1) {
    switch (m) {
      QUAMBA_CASE(11)
      QUAMBA_CASE(12)
      QUAMBA_CASE(13)
      QUAMBA_CASE(14)
      default:
        break;
    }
  }
#undef QUAMBA_CASE
  return fail(QUAMBA_EUNSUPPORTED, "hadamard: order %d*2^%d is outside the supported range", K, m);
}

}  // namespace

bool hadamard_factor(int n, int *k, int *m) {
  if (n <= 0) return false;
  int odd = n, p = 0;
  while ((odd & 1) == 0) {
    odd >>= 1;
    ++p;
  }
  if (odd == 1) {
    *k = 1;
    *m = p;
    return true;
  }
  if ((odd == 3 || odd == 5) && p >= 2) {
    *k = odd * 4;
    *m = p - 2;
    return true;
  }
  return false;
}

namespace {
template <typename TIn>
int dispatch_k(const TIn *g, int M, int n, float inv_s_y, int8_t *yH_q, float *yH_f32, hipStream_t st) {
  int k = 0, m = 0;
  if (!hadamard_factor(n, &k, &m) || m < 4)
    return fail(QUAMBA_EUNSUPPORTED, "hadamard: n=%d is not k*2^m with k in (1,12,20) and m >= 4", n);
  if (M == 0) return QUAMBA_OK;
  switch (k) {
    case 1:
      return dispatch_m<1, TIn>(m, g, M, inv_s_y, yH_q, yH_f32, st);
    case 12:
      return dispatch_m<12, TIn>(m, g, M, inv_s_y, yH_q, yH_f32, st);
    default:
      return dispatch_m<20, TIn>(m, g, M, inv_s_y, yH_q, yH_f32, st);
  }
}
}  // namespace

int launch_hadamard_quant(const __half *g, int M, int n, float inv_s_y, int8_t *yH_q, float *yH_f32,
                          hipStream_t st) {
  return dispatch_k<__half>(g, M, n, inv_s_y, yH_q, yH_f32, st);
}

// fp32 rows in, fp32 rows out, no quantization (used by calibration)
int launch_hadamard_f32(const float *x, int M, int n, float *y, hipStream_t st) {
  return dispatch_k<float>(x, M, n, 1.f, nullptr, y, st);
}

}  // namespace quamba
