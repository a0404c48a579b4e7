// Fused fast Hadamard transform + int8 quantization of the gated scan output (Section 4.2
// "SSM outputs", Eq. 3; Section 3.3): per token row, yH = H_n g, yH_q = clamp(rne(yH / s_y)).
//
// n = k * 2^m with k in {1, 12, 20} and H_n = H_k (x) H_{2^m} (index = a * 2^m + b): the
// 2^m part is the Sylvester / natural-order Walsh-Hadamard matrix, done as butterflies; the
// k part (Section 3.3: a known Hadamard matrix of non-power-of-two order) is the first Paley
// construction for q = k - 1 prime, applied as a dense +-1 product of order k.
//
// For fp16 input the order-k factor runs on the matrix cores: y[a, w] = sum_b H_k[a, b] x[b, w]
// is a (k x k) by (k x 2^m) product whose operands (+-1 and fp16 values) are exact in fp16 and
// whose sums accumulate in fp32, so only the order of the fp32 additions differs from the
// scalar form.  H_k is zero-padded to 32 x 32.
//
// One workgroup per row.  The row sits in LDS as fp32; each pass gathers 2^r (or k) elements
// per work item at a power-of-two stride, transforms them in registers and scatters them back.
// The last pass covers the lowest four index bits, so every work item ends with 16 adjacent
// outputs, which it scales, rounds, clamps and stores as one 16-byte word.  The LDS row is
// padded by 4 floats every 16 so that this 16-byte-per-lane pass is bank-conflict free.
#include <atomic>

#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

// Threads per row: one per 16 elements (every pass then gives each thread one work item), in
// whole waves, at most 1024.
constexpr int threads_for(int n) { return n / 16 >= 1024 ? 1024 : (n / 16 + 63) / 64 * 64; }

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

// H_k as fp16 bit patterns (+1 = 0x3C00, -1 = 0xBC00), zero-padded to 32 x 32: the A operand of
// the MFMA form, read 16 bytes per lane.
// TR: the table of H_k^T (the Paley matrices are not symmetric; the backward transform needs it).
template <int K, bool TR>
struct PaleyHalf {
  uint16_t h[32][32];
  constexpr PaleyHalf() : h{} {
    constexpr Paley<K - 1> tab{};
    for (int a = 0; a < K; ++a)
      for (int b = 0; b < K; ++b) {
        const bool minus = TR ? ((tab.neg[b] >> a) & 1u) : ((tab.neg[a] >> b) & 1u);
        h[a][b] = minus ? 0xBC00 : 0x3C00;
      }
  }
};
template <int K, bool TR>
__device__ const PaleyHalf<K, TR> g_paley_half{};

template <int K, int HT, bool TR>
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
        for (int b = 0; b < K; ++b) s += (TR ? ((tab.neg[b] >> a) & 1u) : ((tab.neg[a] >> b) & 1u)) ? -v[b] : v[b];
        o[a] = s;
      }
#pragma unroll
      for (int a = 0; a < K; ++a) row[pad((a << logm) | w)] = o[a];
    }
    __syncthreads();
  }
}

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// fp16 row in global memory -> order-k transform -> fp32 row in LDS (padded layout), using
// v_mfma_f32_32x32x16_f16.  The row is first staged as fp16 [K][2^LOGM + 8] in the same LDS
// bytes (the pitch keeps the two half-waves of a fragment read on different banks).  Operand
// element e of lane l at k step s is b = 16 s + 8 (l / 32) + e for both operands: H_k[l % 32, b]
// on the A side, x[b, 32 t + l % 32] on the B side; register r of the result is row
// a = 8 (r / 4) + 4 (l / 32) + r % 4, column 32 t + l % 32.
// int8 input (the backward transform of quantized codes) is widened to fp16 while staging, which is exact.
template <int K, int LOGM, int HT, typename TIn, bool TR>
__device__ __forceinline__ void order_k_load_mfma(const TIn *__restrict__ src, float *row) {
  static_assert(K > 1 && K <= 32 && LOGM >= 5, "one 32-row tile of H_k, whole 32-column tiles");
  static_assert(sizeof(TIn) <= 2, "fp16 or int8 rows");
  constexpr int W = 1 << LOGM, PITCH = W + 8, n = K << LOGM;
  _Float16 *hx = reinterpret_cast<_Float16 *>(row);
  for (int i = threadIdx.x * 8; i < n; i += HT * 8) {
    uint4 *dst = reinterpret_cast<uint4 *>(hx + (i >> LOGM) * PITCH + (i & (W - 1)));
    if constexpr (sizeof(TIn) == 2) {
      *dst = *reinterpret_cast<const uint4 *>(src + i);
    } else {
      const uint2 in = *reinterpret_cast<const uint2 *>(src + i);
      union {
        uint4 u;
        _Float16 h[8];
      } w;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        w.h[e] = static_cast<_Float16>(static_cast<int>(static_cast<int8_t>((e < 4 ? in.x : in.y) >> (8 * (e & 3)))));
      *dst = w.u;
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int a = lane & 31, bhalf = 8 * (lane >> 5);
  h8 ha[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) ha[s] = *reinterpret_cast<const h8 *>(&g_paley_half<K, TR>.h[a][16 * s + bhalf]);
  __syncthreads();
  constexpr int NWAVE = HT / 64, TILES = W / 32, TPW = (TILES + NWAVE - 1) / NWAVE;  // column tiles, per wave
  f32x16 acc[TPW];
#pragma unroll
  for (int q = 0; q < TPW; ++q) {
    const int t = wave + NWAVE * q;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
    if (t < TILES) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        if (16 * s >= K) continue;
        h8 hb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int b = 16 * s + bhalf + e;
          hb[e] = b < K ? hx[b * PITCH + 32 * t + a] : static_cast<_Float16>(0.f);
        }
        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ha[s], hb, acc[q], 0, 0, 0);
      }
    }
  }
  __syncthreads();  // every fragment is in registers: the fp16 staging may be overwritten
#pragma unroll
  for (int q = 0; q < TPW; ++q) {
    const int t = wave + NWAVE * q;
    if (t < TILES) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int oa = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (oa < K) row[pad((oa << LOGM) | (32 * t + a))] = acc[q][r];
      }
    }
  }
  __syncthreads();
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
template <int R, int HT>
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

// One row of n = K 2^LOGM values from global memory through every pass but the last, left in LDS
// (padded fp32 layout); ends with a barrier.
template <int K, int LOGM, typename TIn, bool TR>
__device__ __forceinline__ void transform_row(const TIn *__restrict__ src, float *row) {
  static_assert(LOGM >= 4, "the last pass owns the low four index bits");
  constexpr int n = K << LOGM;
  constexpr int HT = threads_for(n);
  if constexpr (sizeof(TIn) <= 2 && K > 1 && LOGM >= 5) {
    order_k_load_mfma<K, LOGM, HT, TIn, TR>(src, row);
  } else {
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
      } else if constexpr (sizeof(TIn) == 1) {
        const uint2 in = *reinterpret_cast<const uint2 *>(src + i);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          dst[e] = static_cast<float>(static_cast<int>(static_cast<int8_t>((e < 4 ? in.x : in.y) >> (8 * (e & 3)))));
      } else {
        *reinterpret_cast<float4 *>(dst) = *reinterpret_cast<const float4 *>(src + i);
        *reinterpret_cast<float4 *>(dst + 4) = *reinterpret_cast<const float4 *>(src + i + 4);
      }
    }
    __syncthreads();
    order_k_pass<K, HT, TR>(row, LOGM);
  }

  // index bits [4, LOGM) in up to three passes of at most 5 bits, high bits first
  constexpr int HI = LOGM - 4;
  constexpr int NP = (HI + 4) / 5;
  constexpr int R0 = NP > 0 ? (HI + NP - 1) / NP : 0;
  constexpr int R1 = NP > 1 ? (HI - R0 + NP - 2) / (NP - 1) : 0;
  constexpr int R2 = NP > 2 ? HI - R0 - R1 : 0;
  static_assert(R0 + R1 + R2 == HI && NP <= 3, "pass schedule");
  radix_pass<R0, HT>(row, n, LOGM - R0);
  radix_pass<R1, HT>(row, n, LOGM - R0 - R1);
  radix_pass<R2, HT>(row, n, 4);
}

// last pass of item w: bits [0, 4) of elements [16 w, 16 w + 16)
__device__ __forceinline__ void last_pass(const float *row, int w, float (&v)[16]) {
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
}

// Outputs (any may be null): out = int8 codes of scale * y; out_f32 = y; out_f16 = fp16(scale * y).
// TR applies H_n^T = H_k^T (x) H_{2^m} (the Sylvester factor is symmetric).
template <int K, int LOGM, typename TIn, bool TR>
__global__ __launch_bounds__(threads_for(K << LOGM)) void hadamard_quant_kernel(const TIn *__restrict__ g, float inv_s,
                                                            int8_t *__restrict__ out,
                                                            float *__restrict__ out_f32,
                                                            __half *__restrict__ out_f16) {
  constexpr int n = K << LOGM;
  constexpr int HT = threads_for(n);
  extern __shared__ __attribute__((aligned(16))) float row[];
  const size_t r = blockIdx.x;
  transform_row<K, LOGM, TIn, TR>(g + r * n, row);

  // last pass: bits [0, 4), fused with scale / round / clamp / pack
  for (int w = threadIdx.x; w < n / 16; w += HT) {
    float v[16];
    last_pass(row, w, v);
    if (out) {
      unsigned pk[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        pk[q] = pack_q8x4(v[4 * q] * inv_s, v[4 * q + 1] * inv_s, v[4 * q + 2] * inv_s, v[4 * q + 3] * inv_s);
      *reinterpret_cast<uint4 *>(out + r * n + (size_t)w * 16) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
    if (out_f32) {
      float *o = out_f32 + r * n + (size_t)w * 16;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        reinterpret_cast<float4 *>(o)[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    }
    if (out_f16) {
      union {
        uint4 u[2];
        __half h[16];
      } o;
#pragma unroll
      for (int e = 0; e < 16; ++e) o.h[e] = __float2half_rn(v[e] * inv_s);
      uint4 *dst = reinterpret_cast<uint4 *>(out_f16 + r * n + (size_t)w * 16);
      dst[0] = o.u[0];
      dst[1] = o.u[1];
    }
  }
}

// Generation with up to three sequences: Hadamard + quantization + out_proj in one launch.  Two launches
// of a few microseconds each, almost all of it latency, become one: every workgroup owns one row and OC
// output columns, asks for its pieces of their weight rows first (one 16-byte piece per thread and column:
// n / 16 threads), transforms its row itself while they arrive (redundantly: the row is 10 KB
// and stays in the cache), and multiplies the 16 codes each thread ends up holding with exactly the
// weight pieces it asked for.  The codes are the stand-alone kernel's bit for bit (same passes, same
// order); the workgroups of column group 0 also store them.  out[r, n] = fp16(acc[r, n] * m_out).
constexpr int OC = 16;  // output columns per workgroup (8: +2 %, 4: +3 %, 32: +12 % on the 64-block step)

template <int K, int LOGM>
__global__ __launch_bounds__(threads_for(K << LOGM)) void hadamard_out_proj_kernel(
    const __half *__restrict__ g, int M, float inv_s, const int8_t *__restrict__ W, int Dm, float m_out,
    __half *__restrict__ out, int8_t *__restrict__ codes_out) {
  constexpr int n = K << LOGM;
  constexpr int HT = threads_for(n);
  static_assert(HT == n / 16, "one item per thread");
  extern __shared__ __attribute__((aligned(16))) float row[];
  __shared__ int red[HT / 64][OC];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // One workgroup per (row, column group).  Workgroups go to the 8 XCDs round-robin by index, so the
  // M workgroups of a column group are spaced 8 apart: same L2, launched together, one HBM read.
  const int ncg = gridDim.x / M, bid = blockIdx.x;
  int cg, r;
  if (ncg % 8 == 0) {
    const int slot = bid >> 3;
    r = slot % M;
    cg = (slot / M) * 8 + (bid & 7);
  } else {
    r = bid % M;
    cg = bid / M;
  }
  const int n0 = cg * OC;
  v4i wv[OC];
#pragma unroll
  for (int j = 0; j < OC; ++j)  // the clamp only bounds the address of a ragged last group
    wv[j] = *reinterpret_cast<const v4i *>(W + (size_t)min(n0 + j, Dm - 1) * n + (size_t)tid * 16);
  transform_row<K, LOGM, __half, false>(g + (size_t)r * n, row);
  float v[16];
  last_pass(row, tid, v);
  v4i c;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    c[q] = static_cast<int>(pack_q8x4(v[4 * q] * inv_s, v[4 * q + 1] * inv_s, v[4 * q + 2] * inv_s, v[4 * q + 3] * inv_s));
  if (cg == 0 && codes_out) *reinterpret_cast<v4i *>(codes_out + (size_t)r * n + (size_t)tid * 16) = c;
#pragma unroll
  for (int j = 0; j < OC; ++j) {
    int acc = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_sdot4(c[e], wv[j][e], acc, false);
    acc = wave_sum(acc);
    if (lane == 0) red[wave][j] = acc;
  }
  __syncthreads();
  if (tid < OC && n0 + tid < Dm) {
    int a = 0;
#pragma unroll
    for (int w = 0; w < HT / 64; ++w) a += red[w][tid];
    out[(size_t)r * Dm + n0 + tid] = __float2half_rn(static_cast<float>(a) * m_out);
  }
}

template <int K, int LOGM, typename TIn, bool TR>
int run(const TIn *g, int M, float inv_s, int8_t *out, float *out_f32, __half *out_f16, hipStream_t st) {
  constexpr int n = K << LOGM;
  constexpr size_t lds = (size_t)(n + n / 4) * sizeof(float);
  if (lds > 64 * 1024) {  // the attribute is per device: one bit per device index
    static std::atomic<unsigned long long> attr_set{0};
    int dev = 0;
    QUAMBA_HIP(hipGetDevice(&dev));
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(attr_set.load(std::memory_order_acquire) & bit)) {
      QUAMBA_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&hadamard_quant_kernel<K, LOGM, TIn, TR>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      attr_set.fetch_or(bit, std::memory_order_release);
    }
  }
  hipLaunchKernelGGL((hadamard_quant_kernel<K, LOGM, TIn, TR>), dim3(M), dim3(threads_for(n)), lds, st, g, inv_s, out,
                     out_f32, out_f16);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

template <int K, typename TIn, bool TR>
int dispatch_m(int m, const TIn *g, int M, float inv_s, int8_t *out, float *out_f32, __half *out_f16, hipStream_t st) {
  switch (m) {
#define QUAMBA_CASE(LM) \
  case LM:              \
    return run<K, LM, TIn, TR>(g, M, inv_s, out, out_f32, out_f16, st);
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
template <typename TIn, bool TR>
int dispatch_k(const TIn *g, int M, int n, float inv_s_y, int8_t *yH_q, float *yH_f32, __half *y_f16, hipStream_t st) {
  int k = 0, m = 0;
  if (!hadamard_factor(n, &k, &m) || m < 4)
    return fail(QUAMBA_EUNSUPPORTED, "hadamard: n=%d is not k*2^m with k in (1,12,20) and m >= 4", n);
  if (M == 0) return QUAMBA_OK;
  switch (k) {
    case 1:
      return dispatch_m<1, TIn, false>(m, g, M, inv_s_y, yH_q, yH_f32, y_f16, st);  // H_{2^m} is symmetric
    case 12:
      return dispatch_m<12, TIn, TR>(m, g, M, inv_s_y, yH_q, yH_f32, y_f16, st);
    default:
      return dispatch_m<20, TIn, TR>(m, g, M, inv_s_y, yH_q, yH_f32, y_f16, st);
  }
}
}  // namespace

int launch_hadamard_quant(const __half *g, int M, int n, float inv_s_y, int8_t *yH_q, float *yH_f32,
                          hipStream_t st) {
  return dispatch_k<__half, false>(g, M, n, inv_s_y, yH_q, yH_f32, nullptr, st);
}

namespace {
template <int K, int LOGM>
int run_out_proj(const __half *g, int M, float inv_s, const int8_t *W, int Dm, float m_out, __half *out, int8_t *codes,
                 hipStream_t st) {
  constexpr int n = K << LOGM;
  constexpr size_t lds = (size_t)(n + n / 4) * sizeof(float);
  static_assert(lds <= 64 * 1024, "fits the default dynamic LDS limit");
  hipLaunchKernelGGL((hadamard_out_proj_kernel<K, LOGM>), dim3((Dm + OC - 1) / OC * M), dim3(threads_for(n)), lds, st, g, M,
                     inv_s, W, Dm, m_out, out, codes);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}
}  // namespace

// orders for which one thread per 16 elements is a whole number of waves and the row fits 64 KB of LDS
bool hadamard_fuses_out_proj(int n, int Dm) {
  int k = 0, m = 0;
  if (Dm < 1 || !hadamard_factor(n, &k, &m)) return false;
  return (k == 1 && m >= 10 && m <= 13) || (k == 12 && m >= 8 && m <= 10) || (k == 20 && m >= 8 && m <= 9);
}

// M rows (a few: with four the separate kernels are faster, and two rows per workgroup, the transforms one
// after the other, cost 5-9 us more than they save): out[r, 0..Dm) = fp16(m_out * W codes(H_n g[r])), codes as launch_hadamard_quant's (stored to codes if given)
int launch_hadamard_out_proj(const __half *g, int M, int n, float inv_s_y, const int8_t *W, int Dm, float m_out,
                             __half *out, int8_t *codes, hipStream_t st) {
  if (M < 1 || M > 64) return fail(QUAMBA_EINVAL, "hadamard + out_proj: M=%d", M);
  if (!hadamard_fuses_out_proj(n, Dm)) return fail(QUAMBA_EUNSUPPORTED, "hadamard + out_proj: n=%d Dm=%d", n, Dm);
  int k = 0, m = 0;
  hadamard_factor(n, &k, &m);
#define QUAMBA_CASE(KK, LM) \
  if (k == KK && m == LM) return run_out_proj<KK, LM>(g, M, inv_s_y, W, Dm, m_out, out, codes, st);
  QUAMBA_CASE(1, 10) QUAMBA_CASE(1, 11) QUAMBA_CASE(1, 12) QUAMBA_CASE(1, 13)
  QUAMBA_CASE(12, 8) QUAMBA_CASE(12, 9) QUAMBA_CASE(12, 10)
  QUAMBA_CASE(20, 8) QUAMBA_CASE(20, 9)
#undef QUAMBA_CASE
  return fail(QUAMBA_EUNSUPPORTED, "hadamard + out_proj: n=%d", n);
}

// fp32 rows in, fp32 rows out, no quantization (used by calibration)
int launch_hadamard_f32(const float *x, int M, int n, float *y, hipStream_t st) {
  return dispatch_k<float, false>(x, M, n, 1.f, nullptr, y, nullptr, st);
}

// Backward transform of quantized codes (Appendix H, the comparison variant's scan input):
// x_hat = fp16(scale * H_n^T xH_q).  The integer sums are exact in fp32 for n * 128 < 2^24.
int launch_hadamard_inverse(const int8_t *xH_q, int M, int n, float scale, __half *x_hat, hipStream_t st) {
  return dispatch_k<int8_t, true>(xH_q, M, n, scale, nullptr, nullptr, x_hat, st);
}

}  // namespace quamba
