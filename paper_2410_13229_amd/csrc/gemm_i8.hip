// int8 x int8 -> int32 GEMM on the gfx950 matrix cores with fused requantization
// (Section 4.3 "Projection layers": 8-bit linear layers, int8 out except the output
// projection, which writes half precision).
//
//   acc[m, j] = sum_k A[m, k] * Wt[j, k]          A [M, K], Wt [N, K], both K-contiguous
//
// One workgroup of 4 wave64s owns a BM x BN tile of the output and walks K in slices that are
// parked in LDS (XOR-swizzled 16-byte chunks, so the fills and the MFMA operand reads are free
// of bank conflicts) and consumed by v_mfma_i32_32x32x32_i8.  The weight fragment is the MFMA
// "A" operand and the activation fragment the "B" operand, so each lane ends up holding four
// consecutive output columns of one token row and can requantize, pack and store them as one
// 32-bit (int8) or 64-bit (fp16) word.
//
// Two kernels share that tiling:
//   gemm_i8_dma_kernel   K a multiple of the slice width.  Slices travel with gfx950's 16-byte
//                        direct-to-LDS loads (global_load_lds_dwordx4): no staging registers, no
//                        LDS write instructions, a ring of LDS stages whose arrival is tracked
//                        with an explicit vmcnt wait in front of one barrier per slice.
//   gemm_i8_kernel       register-staged, zero-fills ragged K, serves small / ragged shapes.
// Skinny problems (few output tiles, deep K) are split along K over grid.y; the int32 partial
// sums go to a workspace and a second kernel adds them and applies the epilogue (integer
// addition, so the result does not depend on the order).
#include <atomic>

#include "common.h"
#include "device_util.h"

namespace quamba {

namespace {

// Byte offset of 16-byte chunk `chunk` of tile row `row` for rows of BKB bytes.  With 64-byte
// rows four rows span the 64 LDS banks and the chunk index is XOR-ed with bits 2..3 of the row;
// with 128-byte rows two rows span them and bits 1..3 are used.  Either way any 16 consecutive
// rows read at one logical chunk hit 16 different bank groups.
template <int BKB>
__device__ __forceinline__ int swzk(int row, int chunk) {
  if constexpr (BKB == 64) return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4);
  else if constexpr (BKB == 128) return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
  else return row * 256 + ((chunk ^ (row & 15)) << 4);  // 256-byte rows: one row spans the 64 banks
}

// Epilogue for four consecutive columns gn..gn+3 of row gm.  The column ranges end on multiples
// of 4, so one multiplier serves the group.
// The conv step on the four x_pre codes `xin` of row gm, channels gn..gn+3.
__device__ __forceinline__ void conv_emit(const GemmEpilogue &epi, int gm, int gn, unsigned xin) {
  const size_t at = (size_t)gm * epi.e0 + gn;
  const unsigned xq = conv_step4(xin, epi.conv.w_q + (size_t)gn * 4, epi.conv.bias + gn, epi.conv.state + at * 3,
                                 epi.conv.s_cw, epi.conv.s_xpre, epi.conv.inv_s_x);
  *reinterpret_cast<unsigned *>(epi.conv.x_q + at) = xq;
}

template <bool CONV = false>
__device__ __forceinline__ void emit4(const GemmEpilogue &epi, int gm, int gn, int N, const int (&raw)[4]) {
  if (epi.acc) {
    v4i v = {raw[0], raw[1], raw[2], raw[3]};
    *reinterpret_cast<v4i *>(epi.acc + (size_t)gm * N + gn) = v;
  }
  int a[4] = {raw[0], raw[1], raw[2], raw[3]};
  if (epi.col_bias) {
    const v4i b = *reinterpret_cast<const v4i *>(epi.col_bias + gn);
#pragma unroll
    for (int e = 0; e < 4; ++e) a[e] += b[e];
  }
  const float m = gn < epi.e0 ? epi.m0 : (gn < epi.e1 ? epi.m1 : epi.m2);
  if (epi.out_i8) {
    const unsigned word = requant_pack4(a, m);
    *reinterpret_cast<unsigned *>(epi.out_i8 + (size_t)gm * epi.ldo + gn) = word;
    if constexpr (CONV)
      if (gn < epi.e0) conv_emit(epi, gm, gn, word);
  } else if (epi.out_f16) {
    union {
      __half h[4];
      uint2 u;
    } pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) pk.h[e] = __float2half_rn(static_cast<float>(a[e]) * m);
    *reinterpret_cast<uint2 *>(epi.out_f16 + (size_t)gm * epi.ldo + gn) = pk.u;
  }
}

// Register r of lane l in MFMA tile (i, j) holds
//   column n = n_base + i*32 + 8*(r/4) + 4*(l/32) + r%4,   row m = m_base + j*32 + l%32.
// `partial` != nullptr: split-K launch, raw sums go to partial[M, N].
template <int TM, int TN, bool CONV = false>
__device__ __forceinline__ void store_tiles(const v16i (&acc)[TN][TM], int m_base, int n_base, int lane,
                                            int M, int N, const GemmEpilogue &epi, int32_t *partial) {
#pragma unroll
  for (int i = 0; i < TN; ++i) {
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int gm = m_base + j * 32 + (lane & 31);
      if (gm >= M) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int gn = n_base + i * 32 + 8 * g + 4 * (lane >> 5);
        if (gn >= N) continue;  // N is a multiple of 4: a group is all in or all out
        const int a[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        if (partial) {
          v4i v = {a[0], a[1], a[2], a[3]};
          *reinterpret_cast<v4i *>(partial + (size_t)gm * N + gn) = v;
        } else {
          emit4<CONV>(epi, gm, gn, N, a);
        }
      }
    }
  }
}

// Same result, but the wave first lays its (TM*32) x (TN*32) block of finished int8 / fp16
// values out row-major in a private LDS region and then writes it with 16 bytes per lane, so a
// wave-level store covers whole runs of a row instead of 8-byte pieces of 32 different rows.
// Needs N, ldo and the output base aligned to 16 bytes; `scratch` is this wave's region of
// TM*32 * (TN*32 * sizeof(element) + 16) bytes, free of other use (callers barrier before).
template <int TM, int TN, bool CONV = false>
__device__ __forceinline__ void store_tiles_rows(const v16i (&acc)[TN][TM], int m_base, int n_base, int lane,
                                                 int M, int N, const GemmEpilogue &epi, int8_t *scratch) {
  const bool f16 = epi.out_f16 != nullptr;
  const int esz = f16 ? 2 : 1;
  const int rowb = TN * 32 * esz;  // bytes per block row
  const int pitch = rowb + 16;     // staged rows sit 16 bytes further apart: fewer lanes per LDS bank
  const int cpr = rowb / 16;  // 16-byte chunks per block row
  int8_t *out = f16 ? reinterpret_cast<int8_t *>(epi.out_f16) : epi.out_i8;
  // one band of 32 rows at a time: its global stores are under way while the next band is requantized
#pragma unroll
  for (int j = 0; j < TM; ++j) {
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      const int row = j * 32 + (lane & 31);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = i * 32 + 8 * g + 4 * (lane >> 5);
        const int gn = n_base + col;
        int a[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        if (epi.col_bias && gn < N) {
          const v4i b = *reinterpret_cast<const v4i *>(epi.col_bias + gn);
#pragma unroll
          for (int e = 0; e < 4; ++e) a[e] += b[e];
        }
        const float m = gn < epi.e0 ? epi.m0 : (gn < epi.e1 ? epi.m1 : epi.m2);
        if (f16) {
          union {
            __half h[4];
            uint2 u;
          } pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk.h[e] = __float2half_rn(static_cast<float>(a[e]) * m);
          *reinterpret_cast<uint2 *>(scratch + row * pitch + col * 2) = pk.u;
        } else {
          *reinterpret_cast<unsigned *>(scratch + row * pitch + col) = requant_pack4(a, m);
        }
      }
    }
    // the region is private to this wave: its own LDS writes are ordered before its reads
    for (int q = lane; q < 32 * cpr; q += 64) {
      const int row = j * 32 + q / cpr, cc = q % cpr;
      const int gm = m_base + row;
      const int gcol = n_base + cc * (16 / esz);
      if (gm < M && gcol < N) {
        const v4i v = *reinterpret_cast<const v4i *>(scratch + row * pitch + cc * 16);
        *reinterpret_cast<v4i *>(out + ((size_t)gm * epi.ldo + gcol) * esz) = v;
      }
    }
  }
  if constexpr (CONV) {
    // conv step on the x_pre columns, from the staged codes: consecutive lanes take consecutive
    // groups of four channels of one row, so the 24-byte windows they touch are adjacent.  All
    // windows, weights and biases of the wave's block are requested before the first is used.
    constexpr int GPR = TN * 8;            // groups per block row (int8 output)
    constexpr int IT = TM * 32 * GPR / 64;  // groups per lane
    ConvWindow4 win[IT];
    uint4 wv[IT];
    float4 bv[IT];
    bool on[IT];
    size_t at[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int q = lane + 64 * it;
      const int row = q / GPR, cg = q % GPR;
      const int gm = m_base + row, gn = n_base + cg * 4;
      on[it] = gm < M && gn < N && gn < epi.e0;
      const int cm = on[it] ? gm : 0, cn = on[it] ? gn : 0;  // off: a valid address, loaded, never stored
      at[it] = (size_t)cm * epi.e0 + cn;
      const uint2 *cs = reinterpret_cast<const uint2 *>(epi.conv.state + at[it] * 3);
      win[it].u[0] = cs[0];
      win[it].u[1] = cs[1];
      win[it].u[2] = cs[2];
      wv[it] = *reinterpret_cast<const uint4 *>(epi.conv.w_q + (size_t)cn * 4);
      bv[it] = *reinterpret_cast<const float4 *>(epi.conv.bias + cn);
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int q = lane + 64 * it;
      const int row = q / GPR, cg = q % GPR;
      float sv[4];
      conv_step4_core(*reinterpret_cast<const unsigned *>(scratch + row * pitch + cg * 4), wv[it], bv[it], win[it],
                      epi.conv.s_cw, epi.conv.s_xpre, sv);
      if (on[it]) {
        uint2 *cs = reinterpret_cast<uint2 *>(epi.conv.state + at[it] * 3);
        cs[0] = win[it].u[0];
        cs[1] = win[it].u[1];
        cs[2] = win[it].u[2];
        *reinterpret_cast<unsigned *>(epi.conv.x_q + at[it]) =
            pack_q8x4(sv[0] * epi.conv.inv_s_x, sv[1] * epi.conv.inv_s_x, sv[2] * epi.conv.inv_s_x, sv[3] * epi.conv.inv_s_x);
      }
    }
  }
}

template <int TM, int TN, bool BARRIER, bool CONV = false>
__device__ __forceinline__ void finish(const v16i (&acc)[TN][TM], int m_base, int n_base, int lane,
                                       int M, int N, const GemmEpilogue &epi, int32_t *partial,
                                       int8_t *scratch, int scratch_bytes) {
  const bool f16 = epi.out_f16 != nullptr;
  const int per = f16 ? 8 : 16;  // elements per 16-byte store
  const int region = TM * 32 * (TN * 32 * (f16 ? 2 : 1) + 16);  // bytes one wave stages (padded rows)
  const uintptr_t base = reinterpret_cast<uintptr_t>(f16 ? (const void *)epi.out_f16 : (const void *)epi.out_i8);
  const bool rows_ok = !partial && !epi.acc && base != 0 && (N % per) == 0 && (epi.ldo % per) == 0 &&
                       (base % 16) == 0 && region <= scratch_bytes;
  if (rows_ok) {
    if (BARRIER) __syncthreads();
    store_tiles_rows<TM, TN, CONV>(acc, m_base, n_base, lane, M, N, epi, scratch);
  } else {
    store_tiles<TM, TN, CONV>(acc, m_base, n_base, lane, M, N, epi, partial);
  }
}

// Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles
// (same weight columns, consecutive token rows) so its L2 sees each weight slice once.
__device__ __forceinline__ int xcd_tile_id(int wg, int nwg) {
  const int per = nwg >> 3;
  return (wg < (per << 3)) ? (wg & 7) * per + (wg >> 3) : wg;
}

// Tile id -> (m tile, n tile), walking the output in bands of 8 m tiles with m fastest inside a
// band: a run of 32 consecutive ids (one XCD's share of 256 tiles) is then an 8 x 4 block, which
// touches the fewest distinct operand rows, instead of a 16 x 2 or 32 x 1 strip.
__device__ __forceinline__ void tile_coords(int id, int tiles_m, int tiles_n, int *tm, int *tn) {
  constexpr int GM = 8;
  const int width = GM * tiles_n;
  const int first = (id / width) * GM;
  const int gsz = min(tiles_m - first, GM);
  const int r = id % width;
  *tm = first + r % gsz;
  *tn = r / gsz;
}

struct KSplit {
  int slices_per_split;  // K slices handled by one grid.y index
  int32_t *partial;      // [splits, M, N] when splitting, else nullptr
};

// ------------------------------------------------------------------------------------------
// Register-staged kernel: 16-byte global loads into registers, parked in a double-buffered LDS
// tile after the MFMAs of the current slice; chunks past K are zero-filled.
// ------------------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_i8_kernel(const int8_t *__restrict__ A, int lda,
                                                      const int8_t *__restrict__ Wt, int ldw, int M, int N,
                                                      int K, GemmEpilogue epi, int tiles_m, int tiles_n,
                                                      KSplit ks) {
  static_assert(WGM * WGN == 4, "four waves per workgroup");
  constexpr int BK = 64;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1 && BM % 64 == 0 && BN % 64 == 0, "tile shape");
  constexpr int A_CH = BM * 4 / 256, W_CH = BN * 4 / 256;  // 16-byte chunks per thread per slice

  __shared__ __attribute__((aligned(16))) int8_t lds[2][(BM + BN) * BK];

  int tile_m, tile_n;
  tile_coords(xcd_tile_id(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, &tile_m, &tile_n);
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  const int k_lo = blockIdx.y * ks.slices_per_split * BK;
  const int k_hi = min(K, k_lo + ks.slices_per_split * BK);

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
      if (gm < M && gk < k_hi) v = *reinterpret_cast<const v4i *>(A + (size_t)gm * lda + gk);
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
      const int c = tid + i * 256;
      const int row = c >> 2, ch = c & 3;
      const int gn = n0 + row, gk = k0 + ch * 16;
      v4i v = {0, 0, 0, 0};
      if (gn < N && gk < k_hi) v = *reinterpret_cast<const v4i *>(Wt + (size_t)gn * ldw + gk);
      rw[i] = v;
    }
  };
  auto park = [&](int buf) {
    int8_t *la = lds[buf];
    int8_t *lw = lds[buf] + BM * BK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<v4i *>(la + swzk<64>(c >> 2, c & 3)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
      const int c = tid + i * 256;
      *reinterpret_cast<v4i *>(lw + swzk<64>(c >> 2, c & 3)) = rw[i];
    }
  };

  const int nk = (k_hi - k_lo + BK - 1) / BK;
  if (nk > 0) {
    fetch(k_lo);
    park(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) fetch(k_lo + (kt + 1) * BK);
    const int8_t *la = lds[buf];
    const int8_t *lw = lds[buf] + BM * BK;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int chunk = s * 2 + (lane >> 5);
      v4i fa[TM], fw[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fa[j] = *reinterpret_cast<const v4i *>(la + swzk<64>(wm * WM + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fw[i] = *reinterpret_cast<const v4i *>(lw + swzk<64>(wn * WN + i * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[i], fa[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) park(buf ^ 1);
    __syncthreads();
  }
  constexpr int REGION = (int)sizeof(lds) / 4;
  finish<TM, TN, true>(acc, m0 + wm * WM, n0 + wn * WN, lane, M, N, epi,
                       ks.partial ? ks.partial + (size_t)blockIdx.y * M * N : nullptr, &lds[0][0] + wave * REGION,
                       REGION);
}

// ------------------------------------------------------------------------------------------
// Direct-to-LDS kernel.  A wave-level global_load_lds_dwordx4 writes 64 lanes x 16 bytes to
// LDS base (M0) + lane * 16, i.e. 1024 / BKB consecutive tile rows; the swizzle is therefore
// applied on the global side: each lane fetches the logical chunk that belongs in its slot.
// Ring of S stages.  Iteration k: wait until this wave's loads of slice k have landed (vmcnt <=
// loads issued after them), barrier (everyone's part of slice k is in LDS and everyone is done
// reading slice k-1), refill the stage slice k-1 occupied with slice k+S-1, multiply slice k.
// Rows past M or N are clamped to the last valid row: they are loaded and multiplied but never
// stored.
// ------------------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, int S, int BKB, int OCC, int KG = 1, bool PIPE = false, bool CONV = false>
__global__ __launch_bounds__(64 * WGM * WGN * KG, OCC) void gemm_i8_dma_kernel(const int8_t *__restrict__ A, int lda,
                                                               const int8_t *__restrict__ Wt, int ldw,
                                                               int M, int N, int K, GemmEpilogue epi,
                                                               int tiles_m, int tiles_n, KSplit ks) {
  // KG wave groups share one output tile: group g multiplies the 32-byte sub-slices s with
  // s % KG == g, and the groups' sums are added through LDS before the epilogue.
  constexpr int NW = WGM * WGN * KG;  // waves per workgroup
  static_assert(NW == 2 || NW == 4 || NW == 8, "two, four or eight waves per workgroup");
  static_assert(BKB == 64 || BKB == 128 || BKB == 256, "slice width");
  static_assert(KG == 1 || KG == 2 || KG == 4, "one, two or four K groups");
  static_assert(BKB / 32 % KG == 0, "every K group gets whole sub-slices");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int RPI = 1024 / BKB;  // tile rows written by one wave-level load
  constexpr int CPR = BKB / 16;    // 16-byte chunks per row
  static_assert(TM >= 1 && TN >= 1 && WM % 32 == 0 && WN % 32 == 0 && BM % RPI == 0 && BN % RPI == 0, "tile");
  constexpr int ROWS = BM + BN;
  constexpr int NJ = ROWS / RPI;    // wave-level loads per slice
  constexpr int NI = (NJ + NW - 1) / NW;  // per wave (a short wave repeats the last group)
  constexpr int STAGE = ROWS * BKB;
  static_assert((S - 2) * NI <= 63 && S >= 2, "vmcnt is 6 bits");

  extern __shared__ __attribute__((aligned(16))) int8_t ring[];

  int tile_m, tile_n;
  tile_coords(xcd_tile_id(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, &tile_m, &tile_n);
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;
  const int slice_lo = blockIdx.y * ks.slices_per_split;
  const int nk = min(K / BKB - slice_lo, ks.slices_per_split);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave / (WGM * WGN);
  const int wtile = wave % (WGM * WGN);
  const int wm = wtile % WGM, wn = wtile / WGM;

  const int8_t *src[NI];
  int dst[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int j = min(wave + NW * i, NJ - 1);
    const int row = j * RPI + lane / CPR;
    const int lrow = row < BM ? row : row - BM;  // the swizzle phase follows the row inside its operand
    const int chunk = BKB == 64 ? ((lane % CPR) ^ ((lrow >> 2) & 3))
                                : (BKB == 128 ? ((lane % CPR) ^ ((lrow >> 1) & 7)) : ((lane % CPR) ^ (lrow & 15)));
    dst[i] = j * 1024;
    if (row < BM)
      src[i] = A + (size_t)min(m0 + row, M - 1) * lda + (size_t)slice_lo * BKB + chunk * 16;
    else
      src[i] = Wt + (size_t)min(n0 + row - BM, N - 1) * ldw + (size_t)slice_lo * BKB + chunk * 16;
  }
  auto issue = [&](int stage, int kslice) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
      __builtin_amdgcn_global_load_lds(
          (const void __attribute__((address_space(1))) *)(src[i] + (size_t)kslice * BKB),
          (void __attribute__((address_space(3))) *)(ring + stage * STAGE + dst[i]), 16, 0, 0);
  };

  v16i acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  auto compute = [&](int stage) {
    const int8_t *la = ring + stage * STAGE;
    const int8_t *lw = la + BM * BKB;
    if constexpr (PIPE) {
      // one wave per SIMD: nothing else hides the LDS latency, so the fragments of sub-slice s + 1 are
      // requested before the MFMAs of sub-slice s are issued, and the scheduler is told to keep that order
      constexpr int NSUB = BKB / 32 / KG;
      v4i fa[2][TM], fw[2][TN];
      auto load = [&](int sub, int buf) {
        const int chunk = (sub * KG + kg) * 2 + (lane >> 5);
#pragma unroll
        for (int j = 0; j < TM; ++j)
          fa[buf][j] = *reinterpret_cast<const v4i *>(la + swzk<BKB>(wm * WM + j * 32 + (lane & 31), chunk));
#pragma unroll
        for (int i = 0; i < TN; ++i)
          fw[buf][i] = *reinterpret_cast<const v4i *>(lw + swzk<BKB>(wn * WN + i * 32 + (lane & 31), chunk));
      };
      load(0, 0);
#pragma unroll
      for (int sub = 0; sub < NSUB; ++sub) {
        if (sub + 1 < NSUB) load(sub + 1, (sub + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int j = 0; j < TM; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[sub & 1][i], fa[sub & 1][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      return;
    }
#pragma unroll
    for (int s0 = 0; s0 < BKB / 32; s0 += KG) {
      const int chunk = (s0 + kg) * 2 + (lane >> 5);
      v4i fa[TM], fw[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fa[j] = *reinterpret_cast<const v4i *>(la + swzk<BKB>(wm * WM + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fw[i] = *reinterpret_cast<const v4i *>(lw + swzk<BKB>(wn * WN + i * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[i], fa[j], acc[i][j], 0, 0, 0);
    }
  };

  // s_waitcnt immediate for "vmcnt <= n, nothing else waited for" (gfx9 encoding: vmcnt in
  // bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
#define QUAMBA_VMCNT(n) (((n) & 0xF) | ((((n) >> 4) & 0x3) << 14) | (0x7 << 4) | (0xF << 8))
  // the same with lgkmcnt = 0 as well (LDS reads of this wave finished)
#define QUAMBA_VMCNT_LGKM0(n) (((n) & 0xF) | ((((n) >> 4) & 0x3) << 14) | (0x7 << 4))
  if constexpr (S == 2 && !PIPE) {
    // Ring of two: the barrier of a slice sits in front of its last sub-slice instead of in front of its first.
    // By then a wave holds the last fragments of the slice in registers, so behind the barrier it has products to
    // issue at once, and the first fragments of the next slice (certified by the same barrier) and the loads of
    // the slice after that travel under them.  With the barrier in front of a slice every wave starts the slice
    // by asking for fragments, and the matrix pipes idle until they arrive.
    constexpr int NSUB = BKB / 32 / KG;
    static_assert(NSUB >= 2, "a slice has a last sub-slice of its own");
    auto frags = [&](int stage, int sub, v4i (&fa)[TM], v4i (&fw)[TN]) {
      const int8_t *la = ring + stage * STAGE;
      const int8_t *lw = la + BM * BKB;
      const int chunk = (sub * KG + kg) * 2 + (lane >> 5);
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fa[j] = *reinterpret_cast<const v4i *>(la + swzk<BKB>(wm * WM + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fw[i] = *reinterpret_cast<const v4i *>(lw + swzk<BKB>(wn * WN + i * 32 + (lane & 31), chunk));
    };
    auto mma = [&](const v4i (&fa)[TM], const v4i (&fw)[TN]) {
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[i], fa[j], acc[i][j], 0, 0, 0);
    };
    v4i pa[TM], pw[TN];  // first fragments of the slice about to start
    if (nk > 0) {
      issue(0, 0);
      __builtin_amdgcn_s_waitcnt(QUAMBA_VMCNT(0));
      __builtin_amdgcn_s_barrier();
      if (nk > 1) issue(1, 1);
      frags(0, 0, pa, pw);
    }
    for (int kt = 0; kt + 1 < nk; ++kt) {
      const int cur = kt & 1;
      v4i fa[TM], fw[TN];
      mma(pa, pw);
#pragma unroll
      for (int sub = 1; sub + 1 < NSUB; ++sub) {
        frags(cur, sub, fa, fw);
        mma(fa, fw);
      }
      frags(cur, NSUB - 1, fa, fw);
      // this wave's loads of slice kt + 1 have landed and its reads of this slice are done: behind the barrier
      // that holds for every wave
      __builtin_amdgcn_s_waitcnt(QUAMBA_VMCNT_LGKM0(0));
      __builtin_amdgcn_s_barrier();
      frags(cur ^ 1, 0, pa, pw);
      __builtin_amdgcn_sched_barrier(0);  // the requests first: the products below are what covers their latency
      if (kt + 2 < nk) issue(cur, kt + 2);
      mma(fa, fw);
    }
    if (nk > 0) {  // the last slice (its own code: a join with the loop body would make the products above wait for pa, pw)
      const int cur = (nk - 1) & 1;
      v4i fa[TM], fw[TN];
      mma(pa, pw);
#pragma unroll
      for (int sub = 1; sub < NSUB; ++sub) {
        frags(cur, sub, fa, fw);
        mma(fa, fw);
      }
    }
  } else {
#pragma unroll
    for (int s = 0; s < S - 1; ++s)
      if (s < nk) issue(s, s);
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + S - 2 < nk)
        __builtin_amdgcn_s_waitcnt(QUAMBA_VMCNT((S - 2) * NI));  // slices kt+1 .. kt+S-2 may be in flight
      else
        __builtin_amdgcn_s_waitcnt(QUAMBA_VMCNT(0));             // tail: fewer slices were issued
      __builtin_amdgcn_s_barrier();
      if (kt + S - 1 < nk) issue(stage == 0 ? S - 1 : stage - 1, kt + S - 1);
      compute(stage);
      stage = (stage + 1 == S) ? 0 : stage + 1;
    }
  }
#undef QUAMBA_VMCNT
#undef QUAMBA_VMCNT_LGKM0

  if constexpr (KG > 1) {
    // groups 1 .. KG-1 park their sums lane-major (16 bytes per lane and register quad:
    // conflict-free), group 0 adds them; region (g - 1, tile) is PART bytes, and group 0 reuses
    // region (0, tile), which it alone reads, for staging its output
    constexpr int PART = TM * TN * 16 * 64 * 4;
    constexpr int TILES = WGM * WGN;
    static_assert(S * STAGE >= (KG - 1) * TILES * PART, "K-group sums fit in the ring");
    __syncthreads();  // operand tiles are dead
    if (kg >= 1) {
      v4i *part = reinterpret_cast<v4i *>(ring + ((kg - 1) * TILES + wtile) * PART);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            part[((i * TM + j) * 4 + g) * 64 + lane] =
                v4i{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
    }
    __syncthreads();
    if (kg >= 1) return;
#pragma unroll
    for (int o = 0; o < KG - 1; ++o) {
      const v4i *part = reinterpret_cast<const v4i *>(ring + (o * TILES + wtile) * PART);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const v4i v = part[((i * TM + j) * 4 + g) * 64 + lane];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] += v[e];
          }
    }
    finish<TM, TN, false, CONV>(acc, m0 + wm * WM, n0 + wn * WN, lane, M, N, epi,
                                ks.partial ? ks.partial + (size_t)blockIdx.y * M * N : nullptr, ring + wtile * PART, PART);
  } else {
    constexpr int REGION = S * STAGE / NW / 16 * 16;
    finish<TM, TN, true, CONV>(acc, m0 + wm * WM, n0 + wn * WN, lane, M, N, epi,
                         ks.partial ? ks.partial + (size_t)blockIdx.y * M * N : nullptr, ring + wave * REGION, REGION);
  }
}

// ------------------------------------------------------------------------------------------
// Few-row kernel (generation with a handful of sequences: M <= 4; from about 8 rows on the
// matrix-tile kernels are faster again).  A matrix tile would be
// nearly empty, and the job is to stream W once: a workgroup owns four adjacent output columns,
// its 256 threads split K in 16-byte pieces (one wave-level load covers 1 KB of a weight row),
// multiply with v_dot4_i32_i8 against the activation rows held in LDS, and reduce across lanes
// and waves.  No K split over the grid, so no second kernel.
// ------------------------------------------------------------------------------------------
template <int MB>
__global__ __launch_bounds__(256) void gemv_i8_kernel(const int8_t *__restrict__ A, int lda,
                                                      const int8_t *__restrict__ Wt, int ldw, int M, int N,
                                                      int K, GemmEpilogue epi) {
  extern __shared__ __attribute__((aligned(16))) int8_t sA[];  // [MB][K], rows past M zero
  __shared__ int red[4][MB * 4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * 4;
  const int nchunks = K / 16;
  // the first weight pieces are requested before the activations are staged: their latency
  // overlaps the staging and its barrier
  v4i w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = min(n0 + j, N - 1);  // N is a multiple of 4: the clamp never acts, it only bounds the address
    w[j] = *reinterpret_cast<const v4i *>(Wt + (size_t)n * ldw + min(tid, nchunks - 1) * 16);
  }
#pragma unroll
  for (int m = 0; m < MB; ++m)
    for (int ch = tid; ch < nchunks; ch += 256) {
      v4i v = {0, 0, 0, 0};
      if (m < M) v = *reinterpret_cast<const v4i *>(A + (size_t)m * lda + ch * 16);
      *reinterpret_cast<v4i *>(sA + (size_t)m * K + ch * 16) = v;
    }
  __syncthreads();
  int acc[MB][4];
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[m][j] = 0;
  for (int ch = tid; ch < nchunks; ch += 256) {
    v4i wn[4];
    const bool more = ch + 256 < nchunks;
    if (more) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int n = min(n0 + j, N - 1);
        wn[j] = *reinterpret_cast<const v4i *>(Wt + (size_t)n * ldw + (ch + 256) * 16);
      }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      const v4i a = *reinterpret_cast<const v4i *>(sA + (size_t)m * K + ch * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[m][j] = __builtin_amdgcn_sdot4(a[e], w[j][e], acc[m][j], false);
    }
    if (more) {
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = wn[j];
    }
  }
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int v = wave_sum(acc[m][j]);
      if (lane == 0) red[wave][m * 4 + j] = v;
    }
  __syncthreads();
  if (tid < M) {
    int a[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = red[0][tid * 4 + j] + red[1][tid * 4 + j] + red[2][tid * 4 + j] + red[3][tid * 4 + j];
    emit4(epi, tid, n0, N, a);
  }
}

// Sum of the split-K partials + epilogue; one thread per group of four columns.
template <bool CONV>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const int32_t *__restrict__ partial, int splits,
                                                            int M, int N, GemmEpilogue epi) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t groups = (size_t)M * (N / 4);
  if (g >= groups) return;
  const int gm = static_cast<int>(g / (N / 4));
  const int gn = static_cast<int>(g % (N / 4)) * 4;
  // at most 8 splits: request every partial before adding any, so the loads overlap
  v4i v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    v[s] = v4i{0, 0, 0, 0};
    if (s < splits) v[s] = *reinterpret_cast<const v4i *>(partial + ((size_t)s * M + gm) * N + gn);
  }
  int a[4] = {0, 0, 0, 0};
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    a[0] += v[s][0];
    a[1] += v[s][1];
    a[2] += v[s][2];
    a[3] += v[s][3];
  }
  emit4<CONV>(epi, gm, gn, N, a);
}

template <int BM, int BN, int WGM, int WGN, int S, int BKB, int OCC, int KG = 1, bool PIPE = false, bool CONV = false>
int run_dma(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
            const GemmEpilogue &epi, int splits, const KSplit &ks, hipStream_t st) {
  constexpr size_t lds = (size_t)S * (BM + BN) * BKB;
  // the attribute is per device: one bit per device index, set after the first successful call there
  // (two threads racing here both set it, which is harmless)
  static std::atomic<unsigned long long> attr_set{0};
  int dev = 0;
  QUAMBA_HIP(hipGetDevice(&dev));
  const unsigned long long bit = 1ull << (dev & 63);
  if (!(attr_set.load(std::memory_order_acquire) & bit)) {
    QUAMBA_HIP(hipFuncSetAttribute(
        reinterpret_cast<const void *>(&gemm_i8_dma_kernel<BM, BN, WGM, WGN, S, BKB, OCC, KG, PIPE, CONV>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set.fetch_or(bit, std::memory_order_release);
  }
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL((gemm_i8_dma_kernel<BM, BN, WGM, WGN, S, BKB, OCC, KG, PIPE, CONV>), dim3(tiles_m * tiles_n, splits),
                     dim3(64 * WGM * WGN * KG), lds, st, A, lda, Wt, ldw, M, N, K, epi, tiles_m, tiles_n, ks);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

template <int BM, int BN, int WGM, int WGN>
int run_reg(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
            const GemmEpilogue &epi, int splits, const KSplit &ks, hipStream_t st) {
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL((gemm_i8_kernel<BM, BN, WGM, WGN>), dim3(tiles_m * tiles_n, splits), dim3(256), 0, st, A,
                     lda, Wt, ldw, M, N, K, epi, tiles_m, tiles_n, ks);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

// Tuning hooks (process-wide; read once per plan).
std::atomic<int> g_gemm_variant{-1};  // >= 0 forces a kernel configuration
std::atomic<int> g_gemm_split{0};     // > 1 forces a K split over the grid
std::atomic<int> g_gemv_max_rows{2};  // the few-row streaming kernels serve M up to this (at most 4)

using GemmChoice = GemmPlan;

// The four tile forms of a large output, priced in output elements per unit rate (times 2 K / 10^6: microseconds).
struct LargePrice {
  int kind;
  double units;
};
LargePrice price_large(int M, int N) {
  auto rounds1 = [](long t) { return (double)((t + 255) / 256); };
  const long t4 = (long)((M + 255) / 256) * ((N + 319) / 320), t10 = (long)((M + 255) / 256) * ((N + 255) / 256);
  const long t2 = (long)((M + 127) / 128) * ((N + 159) / 160);
  const double e4 = rounds1(t4) * (256.0 * 320.0) / 8.7;
  const double e10 = rounds1(t10) * (256.0 * 256.0) / 8.3;
  const double e6 = rounds1(t2) * (128.0 * 160.0) / 5.8;
  const long r2 = t2 % 512;
  const double e2 = ((double)(t2 / 512) + (r2 == 0 ? 0.0 : (r2 <= 256 ? 0.6 : 1.0))) * (128.0 * 160.0) / 3.44;
  LargePrice p{4, e4};
  if (e10 < p.units * 0.97) p = LargePrice{10, e10};
  if (e6 < p.units * 0.97) p = LargePrice{6, e6};
  if (e2 < p.units * 0.97) p = LargePrice{2, e2};
  return p;
}

// Microseconds a row range of the output costs: the large forms by the prices above, smaller outputs by a fit to
// the slower of their measured rates (8 us + operations at 1.2 POP/s: a pessimistic price keeps the split to cases
// where the second part is small).
double price_rows_us(int M, int N, int K) {
  const long tiles_128 = (long)((M + 127) / 128) * ((N + 159) / 160);
  if (tiles_128 >= 192) return price_large(M, N).units * 2.0 * K * 1e-6;
  return 8.0 + 2.0 * M * N * (double)K / 1.2e9;
}

// Rows [0, Mb) and [Mb, M) as two launches when the first then fills whole rounds of CUs and the rest is cheap:
// returns Mb, or 0 to keep one launch.  (2304 x 10240 x 2560: 2048 rows in one round of 256 x 320 tiles plus 256
// rows, instead of two rounds of 256 x 256 tiles.)
int row_split(int M, int N, int K) {
  if (M < 512 || (long)((M + 127) / 128) * ((N + 159) / 160) < 192) return 0;
  const double whole = price_rows_us(M, N, K);
  double best = whole * 0.92;
  int at = 0;
  for (int Mb = (M - 1) / 256 * 256; Mb >= 256 && Mb >= M - 2048; Mb -= 256) {
    const double two = price_rows_us(Mb, N, K) + price_rows_us(M - Mb, N, K) + 3.0;
    if (two < best) {
      best = two;
      at = Mb;
    }
  }
  return at;
}

GemmChoice choose_gemm(int M, int N, int K, const void *ws, size_t ws_bytes, bool partials_wanted = false) {
  const int forced_kind = quamba::g_gemm_variant.load(std::memory_order_relaxed);
  const int forced_split = quamba::g_gemm_split.load(std::memory_order_relaxed);
  const int max_gemv_rows = quamba::g_gemv_max_rows.load(std::memory_order_relaxed);
  const bool k64 = (K % 64) == 0, k128 = (K % 128) == 0;
  // which kernel:
  //   0 = reg 64x64            1 = reg 128x128
  //   2 = dma 128x160, 4 waves, 128-byte slices, ring of 2, two workgroups per CU
  //   3 = dma 64x64, 64-byte slices, ring of 4
  //   4 = dma 256x320, 8 waves of 64x160, 128-byte slices, ring of 2 (the least operand traffic
  //       per MFMA; best when it still yields a tile for most CUs)
  //   5 = dma 64x64, 128-byte slices, ring of 3 (best weight-streaming rate for decode-sized M)
  //   6 = dma 128x160, two K groups of 4 waves (fills the SIMDs when there is only about one
  //       128x160 tile per CU)
  //   8, 9 = 6 and 5 with 256-byte slices and a ring of 2 (K a multiple of 256)
  //   10 = 4 with 256 x 256 tiles (eight waves of 64 x 128), for N that 320-wide tiles fit badly
  //   7 = dma 64x32, two K groups of 2 waves, ring of 4: decode-sized M with a wide output gets a
  //       tile per CU without splitting K over the grid (no second kernel)
  //   12 = 7 with four K groups of 2 waves and 256-byte slices, ring of 3 (K a multiple of 256): half the
  //       barriers and twice the waves per tile for the skinny output of a prefill (2048 x 192 x 5120: 8.3 against
  //       10.1 us; with a deeper ring of 128-byte slices, 6 to 12 stages, the time does not move: the loop is bound
  //       by the per-slice barrier and the latency of one round of fragment reads, not by bytes in flight)
  //   13 = dma 32x32, four K groups of one wave, 256-byte slices, ring of 3: a generation-step output of 64 to 512
  //       such tiles whose K would otherwise be split over the grid, unless the caller takes the partial sums
  //       itself (`partials_wanted`): one launch instead of GEMM + reduce (64 x 2560 x 5120: 7.4 against 9.0 us, 16 rows:
  //       6.6 against 8.0; two K groups with a ring of 4: 8.8; at K = 8192 the split form stays ahead, 11.0 against 11.3);
  //       also the wide output of a step with at most 32 sequences, where one row of tiles covers them
  //       (4 to 32 x 10240 x 2560: 5.9-6.2 against 7.3-7.5 us for the 64 x 64 form)
  //   11 = dma 64x64, two K groups of 4 waves, 256-byte slices, ring of 3: the same job when K is a
  //       multiple of 256; half as many workgroups re-read the activation rows (64 x 10240 x 2560:
  //       7.5 against 8.0 us, 64 x 16384 x 4096: 13.6 against 14.6 us)
  // the streaming kernel keeps its rows in LDS: rows x K bytes next to a static array of rows x 64 bytes
  const size_t gemv_rows = M <= 1 ? 1 : (M <= 2 ? 2 : 4);
  if (M <= max_gemv_rows && forced_kind < 0 && gemv_rows * K + gemv_rows * 64 <= 64 * 1024)
    return GemmChoice{true, 0, 1, 0};
  int kind;
  const long tiles_128 = (long)((M + 127) / 128) * ((N + 159) / 160);
  if (M <= 64)
    kind = k128 ? ((N + 31) / 32 >= 256 ? ((K % 256) == 0 ? (M <= 32 && (N + 31) / 32 <= 512 && K <= 6144 ? 13 : 11) : 7) : 5)
                : (k64 ? 3 : 0);
  else if (N <= 512) {
    kind = k128 ? 5 : (k64 ? 3 : 0);
    // A skinny output with about one 64 x 32 tile per CU and a moderately deep K: those tiles with
    // two K groups fill the chip without splitting K over the grid, which saves the reduce kernel
    // (measured at N = 192, K = 5120: 10.2 vs 12.5 us at M = 2048, 12.4 vs 15.1 at 4096; at
    // K = 8192 or with many more tiles the split-K / single-pass 64 x 64 form stays ahead).
    const long tiles_32 = (long)((M + 63) / 64) * ((N + 31) / 32);
    if (k128 && tiles_32 >= 192 && tiles_32 <= 512 && K <= 8192) kind = (K % 256) == 0 ? 12 : 7;
    // up to 400 tiles of 32 x 32, four K groups of one wave: 7.9 us at 2048 tokens, 6.9-7.1 at 96 to 1024 (the
    // 64 x 64 form: 8.4-11.0); a generation step whose scan adds up the partial sums keeps the split form (96
    // sequences: 4.1 us for the GEMM against 8.3 in one launch)
    if (!partials_wanted && (K % 256) == 0 && K <= 8192 && (long)((M + 31) / 32) * ((N + 31) / 32) <= 400) kind = 13;
    // Very many rows and an N that 160-wide tiles cover without waste: the 128 x 160 tiles with two
    // K groups (N = 320, K = 8192, 16384 tokens: 56 vs 80 us; at 8192 tokens and below the 64 x 64
    // tiles are ahead again).
    const int n160 = (N + 159) / 160 * 160;
    if (k128 && M >= 16384 && N * 10 >= n160 * 9) kind = 6;
  }
  else if (k128 && tiles_128 < 192)
    kind = 5;  // few big tiles: 64 x 64 ones
  else if (k128) {
    // Four forms compete for the large outputs; which is fastest depends on how the tile count fills rounds of
    // 256 CUs, so each is priced as rounds x operations per tile / the rate one resident workgroup sustains
    // (measured with the chip full: 256 x 320 tiles 8.7 TOP/s, 256 x 256 8.3, 128 x 160 with two K groups 5.8,
    // all one workgroup per CU; 128 x 160 with two workgroups per CU 3.44 each, and a last round that leaves
    // them alone on their CUs runs in 0.6 of a tile time).  1280 x 10240 x 2560: 39.4 us with the 256 x 256
    // tiles this picks (200 tiles, one round) against 54.0 with 128 x 160 (640 tiles); 5120 x 2560 x 5120:
    // 80.1 against 91.7; 2560 x 4096 x 8192: 108.9 against 135.4.
    kind = price_large(M, N).kind;
  } else
    kind = 1;
  // deep K in whole 256-byte slices: half as many barriers for the same bytes
  if ((K % 256) == 0 && kind == 6) kind = 8;
  // (decode-sized M measured better with 128-byte slices, and so do skinny outputs, N <= 512, with so
  // many 64 x 64 tiles that K is not split over the grid: there the deeper ring of the 128-byte form wins)
  // and so do outputs of more than 512 tiles: the 128-byte form fits three workgroups on a CU, the
  // 256-byte form two, so beyond 512 tiles it needs a second round (1024 x 2560 x 5120: 28.8 against
  // 32.7 us; 256 x 10240 x 2560: 15.3 against 18.2 us)
  const long tiles64 = (long)((M + 63) / 64) * ((N + 63) / 64);
  const bool skinny_unsplit = N <= 512 && tiles64 > 256;
  if ((K % 256) == 0 && kind == 5 && M > 64 && !skinny_unsplit && tiles64 <= 512) kind = 9;
  // More than 64 rows and still few tiles (short prompts, generation with 65 to 256 sequences): the 32 x 32 tiles
  // with four K groups cover K in one launch and fill the chip where the 64 x 64 ones would split K or leave CUs
  // idle (96 to 192 x 2560 x 5120: 7.2-9.8 against 10.3-12.4 us; from about 520 such tiles on the 64 x 64 forms are
  // ahead again: 384 x 2560 x 5120 18.2 against 12.7).
  if (!partials_wanted && M > 64 && (K % 256) == 0 && K <= 8192 && (kind == 5 || kind == 9)) {
    const long tiles_s = (long)((M + 31) / 32) * ((N + 31) / 32);
    if (N > 512 && tiles_s <= 520) kind = 13;
  }
  // At most 64 rows: the same tiles instead of 64 x 64 tiles with K split over the grid + reduce kernel, unless
  // the caller takes the partial sums itself (3 to 64 x 2560 x 5120: 6.8-7.3 against 8.4-9.2 us, x 192: 6.9-7.0
  // against 8.4-8.8)
  if (!partials_wanted && M <= 64 && (K % 256) == 0 && K <= 6144 && (kind == 5 || kind == 9)) {
    const long tiles_s = (long)((M + 31) / 32) * ((N + 31) / 32);
    if (tiles_s <= 512) kind = 13;
  }
  // 129 to 256 tiles of 64 x 64 with deep K: two K groups per tile instead of K split over the grid
  // (256 / 384 x 2560 x 5120: 12.1 / 12.7 against 13.3 / 14.1 us; 3072 / 4096 x 192 x 5120: 12.3 against 14.1 / 13.3)
  if (M > 64 && (K % 256) == 0 && K <= 8192 && (kind == 5 || kind == 9 || kind == 12) && tiles64 > 128 && tiles64 <= 256 &&
      (long)((M + 31) / 32) * ((N + 31) / 32) > (N <= 512 ? 400 : 520))
    kind = 11;
  if ((forced_kind == 12 || forced_kind == 13) && (K % 256) == 0) kind = forced_kind;
  if (forced_kind >= 0 && forced_kind <= 11 &&
      (forced_kind < 2 || (forced_kind == 3 && k64) || (forced_kind != 3 && k128)) &&
      ((forced_kind != 8 && forced_kind != 9 && forced_kind != 11) || (K % 256) == 0))  // their slices are 256 bytes
    kind = forced_kind;

  // split K when the output has too few tiles to fill 256 CUs and K is deep
  int splits = 1;
  const int slice = (kind == 8 || kind == 9 || kind == 11 || kind == 12 || kind == 13) ? 256 : ((kind == 2 || kind >= 4) ? 128 : 64);
  const int nslices = (K + slice - 1) / slice;
  if ((kind == 0 || kind == 3 || kind == 5 || kind == 9) && ws != nullptr) {
    const int tiles = ((M + 63) / 64) * ((N + 63) / 64);
    // about one workgroup per CU: every further split adds a copy of the output to write and read back
    // (64 x 2560 x 5120: 9.2 us with 6 ranges against 10.0 with 8; 64 x 4096 x 8192: 11.4 with 4 against 12.6)
    int want = (256 + tiles / 2) / (tiles > 0 ? tiles : 1);
    if (want > 8) want = 8;
    while (want > 1 && (nslices / want < 4 || (size_t)want * M * N * sizeof(int32_t) > ws_bytes)) --want;
    if (want > 1) splits = want;
  }
  if (forced_split > 1 && ws != nullptr && (size_t)forced_split * M * N * sizeof(int32_t) <= ws_bytes) splits = forced_split;
  const int per = (nslices + splits - 1) / splits;
  return GemmChoice{false, kind, (nslices + per - 1) / per, per};
}

}  // namespace

int gemv_max_rows() { return g_gemv_max_rows.load(std::memory_order_relaxed); }

size_t gemm_workspace_bytes(int M, int N) {
  // room for up to 8 int32 partial copies of a skinny output
  return (size_t)8 * M * N * sizeof(int32_t);
}

GemmPlan gemm_plan(int M, int N, int K, const void *ws, size_t ws_bytes, bool partials_wanted) {
  return choose_gemm(M, N, K, ws, ws_bytes, partials_wanted);
}

int launch_gemm_i8(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
                   const GemmEpilogue &epi, void *ws, size_t ws_bytes, hipStream_t st, const GemmPlan *plan) {
  const bool conv_in = epi.conv.state != nullptr;
  if (!conv_in && !epi.defer_reduce && g_gemm_variant.load(std::memory_order_relaxed) < 0 && (K % 128) == 0 && N > 512) {
    if (const int Mb = row_split(M, N, K)) {
      GemmEpilogue rest = epi;
      if (rest.out_i8) rest.out_i8 += (size_t)Mb * epi.ldo;
      if (rest.out_f16) rest.out_f16 += (size_t)Mb * epi.ldo;
      if (rest.acc) rest.acc += (size_t)Mb * N;
      const int rc = launch_gemm_i8(A, lda, Wt, ldw, Mb, N, K, epi, ws, ws_bytes, st, nullptr);
      if (rc != QUAMBA_OK) return rc;
      return launch_gemm_i8(A + (size_t)Mb * lda, lda, Wt, ldw, M - Mb, N, K, rest, ws, ws_bytes, st, nullptr);
    }
  }
  const GemmChoice c = plan ? *plan : choose_gemm(M, N, K, ws, ws_bytes);
  if (c.splits > 1 && (!ws || (size_t)c.splits * M * N * sizeof(int32_t) > ws_bytes))
    return fail(QUAMBA_EWORKSPACE, "gemm: %d K ranges of a %d x %d output do not fit the workspace", c.splits, M, N);
  const bool conv = epi.conv.state != nullptr;
  if (conv && (c.gemv || !(c.kind == 7 || c.kind == 11 || c.kind == 13 || c.splits > 1) || !epi.out_i8 || epi.e0 % 4 != 0))
    return fail(QUAMBA_EUNSUPPORTED, "gemm: this shape (M=%d N=%d K=%d) has no epilogue that carries the conv step", M, N, K);
  if (c.gemv) {
    const size_t lds = (size_t)(M <= 1 ? 1 : (M <= 2 ? 2 : 4)) * K;
    if (M <= 1)
      hipLaunchKernelGGL(gemv_i8_kernel<1>, dim3(N / 4), dim3(256), lds, st, A, lda, Wt, ldw, M, N, K, epi);
    else if (M <= 2)
      hipLaunchKernelGGL(gemv_i8_kernel<2>, dim3(N / 4), dim3(256), lds, st, A, lda, Wt, ldw, M, N, K, epi);
    else
      hipLaunchKernelGGL(gemv_i8_kernel<4>, dim3(N / 4), dim3(256), lds, st, A, lda, Wt, ldw, M, N, K, epi);
    QUAMBA_LAUNCH_CHECK();
    return QUAMBA_OK;
  }
  const int kind = c.kind, splits = c.splits;
  KSplit ks{c.slices_per_split, splits > 1 ? static_cast<int32_t *>(ws) : nullptr};

  int rc;
  switch (kind) {
    case 0: rc = run_reg<64, 64, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 2: rc = run_dma<128, 160, 4, 1, 2, 128, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 3: rc = run_dma<64, 64, 2, 2, 4, 64, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 5: rc = run_dma<64, 64, 2, 2, 3, 128, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 4: rc = run_dma<256, 320, 4, 2, 2, 128, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 6: rc = run_dma<128, 160, 4, 1, 3, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 7:
      rc = conv ? run_dma<64, 32, 2, 1, 4, 128, 2, 2, false, true>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st)
                : run_dma<64, 32, 2, 1, 4, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st);
      break;
    case 11:
      rc = conv ? run_dma<64, 64, 2, 2, 3, 256, 2, 2, false, true>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st)
                : run_dma<64, 64, 2, 2, 3, 256, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st);
      break;
    case 8: rc = run_dma<128, 160, 4, 1, 2, 256, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 9: rc = run_dma<64, 64, 2, 2, 2, 256, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 10: rc = run_dma<256, 256, 4, 2, 2, 128, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 12: rc = run_dma<64, 32, 2, 1, 3, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
    case 13:
      rc = conv ? run_dma<32, 32, 1, 1, 3, 256, 2, 4, false, true>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st)
                : run_dma<32, 32, 1, 1, 3, 256, 2, 4>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st);
      break;
    default: rc = run_reg<128, 128, 2, 2>(A, lda, Wt, ldw, M, N, K, epi, splits, ks, st); break;
  }
  if (rc != QUAMBA_OK || splits == 1 || epi.defer_reduce) return rc;
  const size_t groups = (size_t)M * (N / 4);
  if (conv)
    hipLaunchKernelGGL(splitk_reduce_kernel<true>, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, ks.partial,
                       splits, M, N, epi);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<false>, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, st, ks.partial,
                       splits, M, N, epi);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace quamba

extern "C" void quamba_debug_set_gemm_variant(int v) { quamba::g_gemm_variant.store(v); }
extern "C" void quamba_debug_set_gemm_split(int v) { quamba::g_gemm_split.store(v); }
extern "C" void quamba_debug_set_gemv_max_rows(int v) { quamba::g_gemv_max_rows.store(v < 0 ? 2 : (v < 4 ? v : 4)); }
