// int8 x int8 -> int32 GEMM on the gfx950 matrix cores with fused requantization
// (Section 4.3 "Projection layers": 8-bit linear layers, int8 out except the output
// projection, which writes half precision).
//
//   acc[m, j] = sum_k A[m, k] * Wt[j, k]          A [M, K], Wt [N, K], both K-contiguous
//
// One workgroup of 4 wave64s owns a BM x BN tile of the output.  K is walked in slices of 64
// bytes: each slice of A and Wt is fetched with 16-byte global loads into registers, parked in
// LDS (double buffered, XOR-swizzled so both the 16-byte writes and the MFMA operand reads are
// bank-conflict free) and consumed by v_mfma_i32_32x32x32_i8.  The weight fragment is the
// MFMA "A" operand and the activation fragment the "B" operand, so each lane ends up holding
// four consecutive output columns of one token row and can requantize, pack and store them as
// one 32-bit (int8) or 64-bit (fp16) word.
#include "common.h"

namespace quamba {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int BK = 64;  // bytes of K per LDS tile row

// Byte offset of 16-byte chunk `chunk` (0..3) of tile row `row`.  Rows are 64 bytes, so four
// rows span the 64 LDS banks once; XOR-ing the chunk index with bits 2..3 of the row spreads
// any 16 consecutive rows read at one logical chunk over all banks.
__device__ __forceinline__ int swz(int row, int chunk) {
  return row * BK + ((chunk ^ ((row >> 2) & 3)) << 4);
}

__device__ __forceinline__ int requant1(int acc, float m) {
  float v = __builtin_rintf(static_cast<float>(acc) * m);
  v = fminf(fmaxf(v, -128.f), 127.f);
  return static_cast<int>(v);
}

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_i8_kernel(const int8_t *__restrict__ A, int lda,
                                                      const int8_t *__restrict__ Wt, int ldw,
                                                      int M, int N, int K, GemmEpilogue epi,
                                                      int tiles_m, int tiles_n) {
  static_assert(WGM * WGN == 4, "four waves per workgroup");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1 && BM % 64 == 0 && BN % 64 == 0, "tile shape");
  constexpr int A_CH = BM * 4 / 256, W_CH = BN * 4 / 256;  // 16-byte chunks per thread per slice

  __shared__ __attribute__((aligned(16))) int8_t lds[2][(BM + BN) * BK];

  // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // tiles (same weight columns, consecutive token rows) so its L2 sees each weight slice once.
  const int nwg = tiles_m * tiles_n;
  const int per = nwg >> 3;
  const int wg = blockIdx.x;
  const int id = (wg < (per << 3)) ? (wg & 7) * per + (wg >> 3) : wg;
  const int m0 = (id % tiles_m) * BM;
  const int n0 = (id / tiles_m) * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;

  v16i acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  v4i ra[A_CH], rw[W_CH];

  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * 256;
      const int row = c >> 2, ch = c & 3;
      const int gm = m0 + row, gk = k0 + ch * 16;
      v4i v = {0, 0, 0, 0};
      if (gm < M && gk < K) v = *reinterpret_cast<const v4i *>(A + (size_t)gm * lda + gk);
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
      const int c = tid + i * 256;
      const int row = c >> 2, ch = c & 3;
      const int gn = n0 + row, gk = k0 + ch * 16;
      v4i v = {0, 0, 0, 0};
      if (gn < N && gk < K) v = *reinterpret_cast<const v4i *>(Wt + (size_t)gn * ldw + gk);
      rw[i] = v;
    }
  };
  auto park = [&](int buf) {
    int8_t *la = lds[buf];
    int8_t *lw = lds[buf] + BM * BK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<v4i *>(la + swz(c >> 2, c & 3)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<v4i *>(lw + swz(c >> 2, c & 3)) = rw[i];
    }
  };

  const int nk = (K + BK - 1) / BK;
  fetch(0);
  park(0);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * BK);
    const int8_t *la = lds[buf];
    const int8_t *lw = lds[buf] + BM * BK;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int chunk = ks * 2 + (lane >> 5);
      v4i fa[TM], fw[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fa[j] = *reinterpret_cast<const v4i *>(la + swz(wm * WM + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fw[i] = *reinterpret_cast<const v4i *>(lw + swz(wn * WN + i * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[i], fa[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) park(buf ^ 1);
    __syncthreads();
  }

  // Epilogue.  Register r of lane l in tile (i, j) holds
  //   column n = n0 + wn*WN + i*32 + 8*(r/4) + 4*(l/32) + r%4,  row m = m0 + wm*WM + j*32 + l%32.
#pragma unroll
  for (int i = 0; i < TN; ++i) {
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int gm = m0 + wm * WM + j * 32 + (lane & 31);
      if (gm >= M) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int gn = n0 + wn * WN + i * 32 + 8 * g + 4 * (lane >> 5);
        if (gn >= N) continue;  // N is a multiple of 4: a group is all in or all out
        int a[4];
        float mlt[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[e] = acc[i][j][4 * g + e];
          const int c = gn + e;
          mlt[e] = c < epi.e0 ? epi.m0 : (c < epi.e1 ? epi.m1 : epi.m2);
        }
        if (epi.acc) {
          v4i v = {a[0], a[1], a[2], a[3]};
          *reinterpret_cast<v4i *>(epi.acc + (size_t)gm * N + gn) = v;
        }
        if (epi.out_i8) {
          unsigned p = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) p |= (static_cast<unsigned>(requant1(a[e], mlt[e])) & 0xffu) << (8 * e);
          *reinterpret_cast<unsigned *>(epi.out_i8 + (size_t)gm * epi.ldo + gn) = p;
        } else if (epi.out_f16) {
          union {
            __half h[4];
            uint2 u;
          } pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk.h[e] = __float2half_rn(static_cast<float>(a[e]) * mlt[e]);
          *reinterpret_cast<uint2 *>(epi.out_f16 + (size_t)gm * epi.ldo + gn) = pk.u;
        }
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN>
int run(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
        const GemmEpilogue &epi, hipStream_t st) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL((gemm_i8_kernel<BM, BN, WGM, WGN>), dim3(tiles_m * tiles_n), dim3(256), 0, st,
                     A, lda, Wt, ldw, M, N, K, epi, tiles_m, tiles_n);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace

int launch_gemm_i8(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
                   const GemmEpilogue &epi, hipStream_t st) {
  if (M <= 64 || N <= 512) return run<64, 64, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, st);
  return run<128, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, st);
}

}  // namespace quamba
