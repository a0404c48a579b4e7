// Quantized selective scan with SiLU(z) gate (Section 3.1 Eq. 1; Section 4.2 "Quantization
// for Selective SSM"): int8 x, dt, B, C, z (and int8 A, D) are dequantized inside the kernel
// with their static scales, the recurrence runs on an fp32 state, the output is fp16.
//
//   x = s_x x_q,  dt = softplus(s_dt dt_q + dt_bias),  z = s_z z_q
//   h[n] <- exp(dt * s_A A_q[d,n]) * h[n] + dt * x * s_B B_q[t,n]
//   y = sum_n s_C C_q[t,n] * h[n] + s_D D_q[d] * x,   g = y * z / (1 + exp(-z))
//
// Layout: activations are token-major [t, d] int8, so one wavefront = 64 adjacent channels
// reads 64 contiguous bytes per token and tensor; every lane keeps the 16 states of its channel
// in registers.  B_t and C_t are shared by all channels: each workgroup dequantizes them once
// per block of tokens into LDS and the lanes read them back as broadcasts.
//
// Prefill parallelises over L with a three-pass chunked scan (the recurrence is linear in h):
//   pass 1  per (chunk, channel): end state of the chunk started from h = 0, and sum of dt
//   pass 2  per (channel, n): walk the chunks in order, h_start[c+1] = P_c h_start[c] + h_loc[c]
//           with P_c = exp(A * sum_c dt); emits the start state of every chunk and h_L
//   pass 3  per (chunk, channel): rerun the chunk from its true start state and emit g
// Where sequences x channels alone fill the SIMDs (batches, and any sequence short enough that the three
// launches dominate) prefill instead walks each sequence once, two states per lane: scan_sweep_kernel below.
// Decode is a single recurrence step with 4 lanes per channel (float4 state access).
//
// Pass 1 can also produce dt_q itself (Section 4.3 fuses operators to save memory traffic and
// launches): dt_q = q(W_dt dt_low) is a K = dt_rank contraction, a handful of MFMAs per
// (32-token, 64-channel) tile, which each wave runs for its own channels before it walks the
// tokens.  The codes go through a wave-private LDS tile to the lanes and to dt_q for pass 3.
#include <atomic>
#include <cmath>

#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

constexpr float LOG2E = 1.44269504088896340736f;
constexpr float LN2 = 0.69314718055994530942f;
constexpr int NS = 16;       // d_state
constexpr int TB = 64;       // tokens of B/C staged in LDS at a time
constexpr int SCAN_THREADS = 256;
constexpr int DT_LD = 68;    // row pitch (bytes) of the LDS tile of dt codes: 17 words, odd
constexpr int W_PITCH_MAX = 176;  // the fused dt_proj stages its operand rows in LDS when dt_rank + 16 fits this pitch

__device__ __forceinline__ float exp2_fast(float v) { return __builtin_amdgcn_exp2f(v); }

// softplus(v) = log(1 + exp(v)) = max(v, 0) + log1p(exp(-|v|)).  With e = exp(-|v|) <= 1 the sum
// w = 1 + e lies in [1, 2], so (w - 1) - e is exactly the rounding error of w, and log(w) minus that
// error is log1p(e) to fp32 accuracy even where 1 + e loses the low bits of e (the hardware log2 is
// accurate relative to its result next to 1).  No overflow, and above 20 the result is v itself in
// fp32, which is the written definition.  Measured against fp64 over [-30, 100]: <= 1.1e-6 relative
// down to v = -20 (the same as a series for small e), 7 instructions + 2 transcendentals.
__device__ __forceinline__ float softplus_f(float v) {
  const float e = exp2_fast(-fabsf(v) * LOG2E);
  const float w = 1.f + e;
  const float c = (w - 1.f) - e;
  return fmaxf(v, 0.f) + __builtin_fmaf(__builtin_amdgcn_logf(w), LN2, -c);
}

__device__ __forceinline__ float silu_gate(float y, float z) {
  return y * z * __builtin_amdgcn_rcpf(1.f + exp2_fast(-z * LOG2E));
}

struct Dev {
  const int8_t *x_q, *dt_q, *z_q, *B_q, *C_q, *A_q, *D_q;
  const float *dt_bias;
  int ldz, ldbc;
  float s_x, s_dt, s_z, s_B, s_C, s_A, s_D;
  int L, Di, T, nchunks;
  __half *g16;
  float *y_f32;
  float *hloc;  // [Bt, nchunks, Di, 16]
  float *ssum;  // [Bt, nchunks, Di]
  // fused dt_proj (pass 1): dt_low codes [Bt*L, lddl], W_dt [Di, R], multiplier, dt_q to write
  const int8_t *dtlow_q, *W_dt;
  int lddl, R;
  float m_dt;
  int8_t *dt_out;
  const __half *x_f16;  // scan input in half precision instead of s_x * x_q (comparison variant)
  float x_off;          // -s_x * zero point of an asymmetric x grid: x = s_x x_q + x_off (0 = symmetric)
  const unsigned *s_x_slot;  // bits of the call's max|x| when the scale of x is dynamic
  const int32_t *dbc_part;   // generation: x_proj's sums as dbc_splits partial results [dbc_splits][Bt][R + 2 NS]
  int dbc_splits;
  float m_x_dt, m_x_B, m_x_C;
  WarmRanges warm;  // ranges that extra workgroups along grid.x read into the cache beside the scan
};

// How the scan reads x: int8 codes on a uniform grid (s_x x_q + x_off), half precision values (the
// Appendix H comparison variant), or one-byte codes of a non-uniform format (Appendix K).
// X_I8DYN: the uniform grid with a scale derived in the kernel from the call's max|x| (Appendix K, dynamic row).
enum XMode { X_I8 = 0, X_F16 = 1, X_E4M3 = 2, X_LOG2 = 3, X_I8DYN = 4 };
template <int XM>
__device__ __forceinline__ float x_scale(const Dev &p) {
  if constexpr (XM == X_I8DYN) return dyn_scale(p.s_x_slot);
  else return p.s_x;
}
// raw: the sign-extended code byte, or the 16 bits of the half; sx: x_scale<XM>(p)
template <int XM>
__device__ __forceinline__ float x_value(const Dev &p, int raw, float sx) {
  if constexpr (XM == X_F16) return __half2float(__ushort_as_half(static_cast<unsigned short>(raw)));
  else if constexpr (XM == X_E4M3) return sx * decode_e4m3(static_cast<unsigned>(raw) & 0xffu);
  else if constexpr (XM == X_LOG2) return sx * decode_log2(static_cast<unsigned>(raw) & 0xffu);
  else if constexpr (XM == X_I8DYN) return sx * static_cast<float>(raw);
  else return __builtin_fmaf(sx, static_cast<float>(raw), p.x_off);
}

// B (and C) codes of tokens [row0, row0+cnt) -> fp32 [TB][16] in LDS, in two steps so that the loads can be
// requested ahead of other work: bc_load asks for this thread's TB * 16 / 256 codes, bc_park dequantizes and stores.
constexpr int BC_PER = TB * NS / SCAN_THREADS;
struct BCRegs {
  int b[BC_PER], c[BC_PER];
};
template <bool WITH_C>
__device__ __forceinline__ void bc_load(const Dev &p, size_t row0, int cnt, BCRegs &r) {
#pragma unroll
  for (int k = 0; k < BC_PER; ++k) {
    const int i = threadIdx.x + k * SCAN_THREADS;
    const int tt = min(i >> 4, cnt - 1), n = i & 15;  // past the block: loaded again, parked as zero
    r.b[k] = p.B_q[(row0 + tt) * p.ldbc + n];
    r.c[k] = WITH_C ? p.C_q[(row0 + tt) * p.ldbc + n] : 0;
  }
}
template <bool WITH_C>
__device__ __forceinline__ void bc_park(const Dev &p, int cnt, const BCRegs &r, float (*sB)[NS], float (*sC)[NS]) {
#pragma unroll
  for (int k = 0; k < BC_PER; ++k) {
    const int i = threadIdx.x + k * SCAN_THREADS;
    const int tt = i >> 4, n = i & 15;
    const bool on = tt < cnt;
    sB[tt][n] = on ? p.s_B * static_cast<float>(r.b[k]) : 0.f;
    if (WITH_C) sC[tt][n] = on ? p.s_C * static_cast<float>(r.c[k]) : 0.f;
  }
}

// One (chunk, 256-channel) tile of the scan.  OUTPUT = false: pass 1 (state from zero, sum of
// dt).  OUTPUT = true: pass 3 (state from the carried start, gated output).
// The int8 x / dt / z bytes of the next TS tokens are fetched into registers while the
// current TS tokens are computed, so no load latency sits on the recurrence.
// FUSE_DT (pass 1 only): dt_q is not read but computed from dt_low and W_dt, and written out.
template <bool OUTPUT, bool FUSE_DT, int XM = X_I8>
__global__ __launch_bounds__(SCAN_THREADS) void scan_chunk_kernel(Dev p) {
  static_assert(!(OUTPUT && FUSE_DT), "dt_q is produced by pass 1");
  __shared__ __attribute__((aligned(16))) float sB[TB][NS];
  __shared__ __attribute__((aligned(16))) float sC[OUTPUT ? TB : 1][NS];
  __shared__ __attribute__((aligned(16))) int8_t sDT[FUSE_DT ? SCAN_THREADS / 64 : 1][FUSE_DT ? TB : 1][DT_LD];
  __shared__ __attribute__((aligned(16))) int8_t sW[FUSE_DT ? SCAN_THREADS / 64 : 1][FUSE_DT ? 32 * W_PITCH_MAX : 16];
  __shared__ __attribute__((aligned(16))) int8_t sA[FUSE_DT ? 32 * W_PITCH_MAX : 16];
  if constexpr (OUTPUT) {  // the last workgroups along x only read ahead (whole workgroups: no barrier is skipped)
    const int real = gridDim.x - p.warm.blocks;
    if ((int)blockIdx.x >= real) {
      const int per = gridDim.y * gridDim.z;
      warm_read(p.warm, (blockIdx.x - real) * per + blockIdx.z * gridDim.y + blockIdx.y, p.warm.blocks * per);
      return;
    }
  }
  const int d = blockIdx.x * SCAN_THREADS + threadIdx.x;
  const int c = blockIdx.y, b = blockIdx.z;
  const bool live = d < p.Di;
  const int dd = live ? d : p.Di - 1;
  const int t0 = c * p.T, t1 = min(t0 + p.T, p.L);

  float a2[NS], h[NS];
  {
    const uint4 av = *reinterpret_cast<const uint4 *>(p.A_q + (size_t)dd * NS);
    const unsigned aw[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
    for (int n = 0; n < NS; ++n) {
      a2[n] = static_cast<float>(static_cast<int8_t>(aw[n >> 2] >> (8 * (n & 3)))) * (p.s_A * LOG2E);
      h[n] = 0.f;
    }
    if (OUTPUT) {
      const float *src = p.hloc + (((size_t)b * p.nchunks + c) * p.Di + dd) * NS;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = reinterpret_cast<const float4 *>(src)[q];
        h[4 * q] = v.x;
        h[4 * q + 1] = v.y;
        h[4 * q + 2] = v.z;
        h[4 * q + 3] = v.w;
      }
    }
  }
  const float bias = p.dt_bias[dd];
  const float Dv = OUTPUT ? p.s_D * static_cast<float>(p.D_q[dd]) : 0.f;
  const float sx = x_scale<XM>(p);
  float sdt = 0.f;
  const size_t seq0 = (size_t)b * p.L;
  // x / dt / z / g of this chunk behind buffer descriptors: row offsets are scalar, the lane adds
  // its channel (the launcher checks that a chunk's rows span less than 2^31 bytes)
  const unsigned ud = static_cast<unsigned>(dd);
  const size_t tok0 = seq0 + t0;
  const int nt = t1 - t0;
  const auto rx = XM == X_F16 ? buffer_over(p.x_f16 + tok0 * p.Di, nt * p.Di * 2) : buffer_over(p.x_q + tok0 * p.Di, nt * p.Di);
  const auto rdt = FUSE_DT ? rx : buffer_over(p.dt_q + tok0 * p.Di, nt * p.Di);
  const auto rz = OUTPUT ? buffer_over(p.z_q + tok0 * p.ldz, (nt - 1) * p.ldz + p.Di) : rx;
  const auto rg = OUTPUT ? buffer_over(p.g16 + tok0 * p.Di, nt * p.Di * 2) : rx;
  // the optional fp32 copy of the output: an empty descriptor drops every store when it is not asked for
  const auto ry = (OUTPUT && p.y_f32) ? buffer_over(p.y_f32 + tok0 * p.Di, nt * p.Di * 4) : buffer_over(p.x_q, 0);
  const unsigned ud_out = live ? ud : 0x0fffffffu;  // lanes past the last channel store nothing

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // dt codes of tokens [tok0, tok0 + 32) for this wave's 64 channels -> rows [row0, row0 + 32) of
  // its LDS tile.  MFMA operands come straight from global memory (every fragment is used once):
  // lane l supplies 16 bytes of k at offset 32 s + 16 (l / 32) of weight row / token row l % 32;
  // register r of tile i then holds channel 32 i + 8 (r / 4) + 4 (l / 32) + r % 4 of token l % 32.
  // Operand rows: a lane of the MFMA layout wants 16 bytes of one row, so a wave-level load straight from global memory
  // touches 32 rows = 32 cache lines for 1 KB (measured at 2.8B width: 2.7 us of the pass).  Where the rows fit
  // (R + 16 <= W_PITCH_MAX, whole workgroups of channels) they are read as whole rows instead - the 32 weight rows of a
  // tile are 32 R contiguous bytes, 64 / (R / 16) rows per wave-level load, parked in the wave's own LDS region; the
  // 32 token rows once per workgroup, shared by its four waves - and read back from LDS as fragments.
  const int cpr = p.R >> 4;  // 16-byte pieces per row
  const bool w_staged = FUSE_DT && p.R + 16 <= W_PITCH_MAX && (p.Di % SCAN_THREADS) == 0;
  const int w_r0 = w_staged ? lane / cpr : 0, w_col = lane - w_r0 * cpr, w_rows = w_staged ? 64 / cpr : 1;
  constexpr int W_LOADS = 6;  // 32 rows at 6 or more rows per load (R <= 160: 64 lanes hold 6 rows of 10 pieces)
  constexpr int A_LOADS = 2;  // 32 rows of at most 10 pieces over 256 threads
  auto dt_tile = [&](int tok0, int row0) {
    const int dw0 = blockIdx.x * SCAN_THREADS + wave * 64;
    const int koff = 16 * (lane >> 5);
    // codes of tile i: register r of lane l is channel 32 i + 8 (r / 4) + 4 (l / 32) + r % 4 of token l % 32
    auto emit = [&](const v16i &acc, int i) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int a[4] = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
        *reinterpret_cast<unsigned *>(&sDT[wave][row0 + (lane & 31)][32 * i + 8 * g + 4 * (lane >> 5)]) =
            requant_pack4(a, p.m_dt);
      }
    };
    if (w_staged) {
      const int pitch = p.R + 16;
      int8_t *lw = sW[wave];
      v4i wv[W_LOADS], av[A_LOADS];
      int a_at[A_LOADS];  // LDS offset of this thread's piece of the token rows, -1: none
      auto w_load = [&](int i) {
#pragma unroll
        for (int g = 0; g < W_LOADS; ++g) {
          const int row = g * w_rows + w_r0;
          wv[g] = v4i{0, 0, 0, 0};
          if (w_r0 < w_rows && row < 32)
            wv[g] = *reinterpret_cast<const v4i *>(p.W_dt + (size_t)(dw0 + 32 * i + row) * p.R + 16 * w_col);
        }
      };
      auto w_park = [&]() {
#pragma unroll
        for (int g = 0; g < W_LOADS; ++g) {
          const int row = g * w_rows + w_r0;
          if (w_r0 < w_rows && row < 32) *reinterpret_cast<v4i *>(lw + row * pitch + 16 * w_col) = wv[g];
        }
      };
#pragma unroll
      for (int k = 0; k < A_LOADS; ++k) {
        const int c = static_cast<int>(threadIdx.x) + SCAN_THREADS * k;
        const int row = c / cpr, col = c - row * cpr;
        a_at[k] = -1;
        av[k] = v4i{0, 0, 0, 0};
        if (row < 32) {
          a_at[k] = row * pitch + 16 * col;
          av[k] = *reinterpret_cast<const v4i *>(p.dtlow_q + (seq0 + min(tok0 + row, t1 - 1)) * p.lddl + 16 * col);
        }
      }
      w_load(0);
      __syncthreads();  // the token rows of the previous tile have been read by every wave
#pragma unroll
      for (int k = 0; k < A_LOADS; ++k)
        if (a_at[k] >= 0) *reinterpret_cast<v4i *>(sA + a_at[k]) = av[k];
      w_park();
      __builtin_amdgcn_sched_barrier(0);  // keeps the loads below from being hoisted over the stores: one set of registers
      w_load(1);  // the second tile's rows travel under the first tile's products
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if (i == 1) w_park();  // the wave's own region, its LDS accesses execute in order: no barrier
        v16i acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0;
        for (int k0 = 0; k0 < p.R; k0 += 32) {
          // a lane whose half lies past R (R an odd multiple of 16) multiplies zeros
          v4i fw = v4i{0, 0, 0, 0}, fa = v4i{0, 0, 0, 0};
          if (k0 + koff < p.R) {
            fw = *reinterpret_cast<const v4i *>(lw + (lane & 31) * pitch + k0 + koff);
            fa = *reinterpret_cast<const v4i *>(sA + (lane & 31) * pitch + k0 + koff);
          }
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw, fa, acc, 0, 0, 0);
        }
        emit(acc, i);
        __builtin_amdgcn_sched_barrier(0);  // one accumulator tile at a time
      }
      return;
    }
    {  // operands straight from global memory, the two 32-channel tiles one after the other
      const int8_t *arow = p.dtlow_q + (seq0 + min(tok0 + (lane & 31), t1 - 1)) * p.lddl;
#pragma nounroll
      for (int i = 0; i < 2; ++i) {
        const int8_t *wrow = p.W_dt + (size_t)min(dw0 + 32 * i + (lane & 31), p.Di - 1) * p.R;
        v16i acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0;
        constexpr int PH = 3;  // k steps whose operands are in flight together
        for (int s0 = 0; s0 * 32 < p.R; s0 += PH) {
          v4i fa[PH], fw[PH];
#pragma unroll
          for (int j = 0; j < PH; ++j) {
            const int kc = 32 * (s0 + j) + koff;
            fa[j] = fw[j] = v4i{0, 0, 0, 0};
            if (kc < p.R) {  // R is a multiple of 16: a 16-byte piece is all in or all out
              fa[j] = *reinterpret_cast<const v4i *>(arow + kc);
              fw[j] = *reinterpret_cast<const v4i *>(wrow + kc);
            }
          }
#pragma unroll
          for (int j = 0; j < PH; ++j) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fa[j], acc, 0, 0, 0);
        }
        emit(acc, i);
      }
    }
  };
  // rows [0, cnt) of the wave's tile -> dt_q (64 contiguous bytes per token)
  auto dt_store = [&](int tb, int cnt) {
    const int ch = blockIdx.x * SCAN_THREADS + wave * 64 + 4 * (lane & 15);
    for (int tt = lane >> 4; tt < cnt; tt += 4)
      if (ch < p.Di)  // Di is a multiple of 4
        *reinterpret_cast<unsigned *>(p.dt_out + (seq0 + tb + tt) * p.Di + ch) =
            *reinterpret_cast<const unsigned *>(&sDT[wave][tt][4 * (lane & 15)]);
  };

  constexpr int TS = 8;
  struct Regs {
    int x[TS], dt[TS], z[TS];
  };
  auto fetch = [&](Regs &r, int t) {
#pragma unroll
    for (int i = 0; i < TS; ++i) {
      // clamp: tokens past the chunk are loaded but never used
      const int row = min(t + i, t1 - 1) - t0;
      r.x[i] = XM == X_F16 ? static_cast<int>(buffer_load_u16(rx, 2 * ud, row * p.Di * 2)) : buffer_load_i8(rx, ud, row * p.Di);
      if (!FUSE_DT) r.dt[i] = buffer_load_i8(rdt, ud, row * p.Di);  // fused: read from the LDS tile
      if (OUTPUT) r.z[i] = buffer_load_i8(rz, ud, row * p.ldz);
    }
  };
  auto token = [&](const Regs &r, int i, int t, int tl) {  // t: token index, tl: index inside the LDS block
      {
        const float xv = x_value<XM>(p, r.x[i], sx);
        const int dtq = FUSE_DT ? static_cast<int>(sDT[wave][tl + i][lane]) : r.dt[i];
        const float dt = softplus_f(p.s_dt * static_cast<float>(dtq) + bias);
        const float u = dt * xv;
        if (!OUTPUT) sdt += dt;
        float y = 0.f;
#pragma unroll
        for (int n = 0; n < NS; ++n) {
          h[n] = exp2_fast(dt * a2[n]) * h[n] + u * sB[tl + i][n];
          if (OUTPUT) y += sC[tl + i][n] * h[n];
        }
        if (OUTPUT) {
          y += Dv * xv;
          const float g = silu_gate(y, p.s_z * static_cast<float>(r.z[i]));
          buffer_store_f16(rg, 2 * ud_out, (t + i - t0) * p.Di * 2, g);
          buffer_store_f32(ry, 4 * ud_out, (t + i - t0) * p.Di * 4, g);
        }
      }
  };
  // Whole groups of TS tokens run without per-token range tests, as one straight block the
  // scheduler can interleave; only the ragged end of a sequence takes the tested form.
  auto compute = [&](const Regs &r, int t, int tl) {
    if (t + TS <= t1) {
#pragma unroll
      for (int i = 0; i < TS; ++i) token(r, i, t, tl);
    } else {
#pragma unroll
      for (int i = 0; i < TS; ++i)
        if (t + i < t1) token(r, i, t, tl);
    }
  };

  for (int tb = t0; tb < t1; tb += TB) {
    const int cnt = min(TB, t1 - tb);
    Regs ra, rb;
    // the loads of the block's start are requested together: B / C codes and the first TS tokens
    BCRegs bc;
    if (!FUSE_DT) {
      bc_load<OUTPUT>(p, seq0 + tb, cnt, bc);
      fetch(ra, tb);
    }
    if (FUSE_DT) {  // the tile is private to the wave: its LDS accesses execute in order
      dt_tile(tb, 0);
      if (cnt > 32) dt_tile(tb + 32, 32);
      dt_store(tb, cnt);
      bc_load<OUTPUT>(p, seq0 + tb, cnt, bc);  // (behind the tile: in front of it they cost it a wave per SIMD in registers)
      fetch(ra, tb);
    }
    __syncthreads();
    bc_park<OUTPUT>(p, cnt, bc, sB, sC);
    __syncthreads();
    for (int ts = 0; ts < cnt; ts += 2 * TS) {
      if (ts + TS < cnt) fetch(rb, tb + ts + TS);
      compute(ra, tb + ts, ts);
      if (ts + 2 * TS < cnt) fetch(ra, tb + ts + 2 * TS);
      if (ts + TS < cnt) compute(rb, tb + ts + TS, ts + TS);
    }
  }
  if (!OUTPUT && live) {
    float *dst = p.hloc + (((size_t)b * p.nchunks + c) * p.Di + d) * NS;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      reinterpret_cast<float4 *>(dst)[q] = make_float4(h[4 * q], h[4 * q + 1], h[4 * q + 2], h[4 * q + 3]);
    p.ssum[((size_t)b * p.nchunks + c) * p.Di + d] = sdt;
  }
}

// ---------------------------------------------------------------- pass 2: carry across chunks
// One thread per (b, d, n).  In place: hloc[c] is replaced by the start state of chunk c.
// All loads of a block of up to 64 chunks are issued before the walk starts, so the memory
// latency is paid once per block instead of once per chunk.  The kernel moves the chunk states
// once in and once out and is bound by that traffic.
__global__ __launch_bounds__(256) void scan_carry_kernel(Dev p, float *__restrict__ ssm_state, int Bt) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t per_b = (size_t)p.Di * NS;
  if (idx >= per_b * Bt) return;
  const int b = static_cast<int>(idx / per_b);
  const size_t dn = idx % per_b;
  const int d = static_cast<int>(dn / NS);
  const float a2 = static_cast<float>(p.A_q[dn]) * (p.s_A * LOG2E);
  float h = ssm_state ? ssm_state[idx] : 0.f;
  float *hl = p.hloc + (size_t)b * p.nchunks * per_b + dn;
  const float *ss = p.ssum + (size_t)b * p.nchunks * p.Di + d;
  constexpr int G = 64;
  for (int c0 = 0; c0 < p.nchunks; c0 += G) {
    float loc[G], s[G];
#pragma unroll
    for (int i = 0; i < G; ++i) {
      loc[i] = 0.f;
      s[i] = 0.f;
      if (c0 + i < p.nchunks) {
        loc[i] = hl[(size_t)(c0 + i) * per_b];
        s[i] = ss[(size_t)(c0 + i) * p.Di];
      }
    }
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const float start = h;
      if (c0 + i < p.nchunks) h = exp2_fast(a2 * s[i]) * h + loc[i];
      loc[i] = start;
    }
#pragma unroll
    for (int i = 0; i < G; ++i)
      if (c0 + i < p.nchunks) hl[(size_t)(c0 + i) * per_b] = loc[i];
  }
  if (ssm_state) ssm_state[idx] = h;
}

// ---------------------------------------------------------------- prefill: one sweep per sequence
// The chunked form pays for its parallelism over L with every exponential twice (pass 1 and pass 3).
// When sequences x channels alone give several waves per SIMD, one sweep over each whole sequence is
// cheaper.  A lane owns two of the 16 states of one channel (8 lanes per channel, 8 channels per wave,
// 32 per workgroup), so the recurrence of a (channel, state pair) is serial in a lane and everything
// else is spread over lanes:
//   * the work per (token, channel) - dt code (MFMA tile of the fused dt_proj), softplus, x, z - is done
//     once, a 16-token x 32-channel tile per wave and superblock of 64 tokens, and handed to the lanes of
//     the recurrence through LDS as (dt, dt x), D x and the z code; B and C go there as (B0, B1, C0, C1)
//     per state pair.  The global loads of superblock k + 1 are issued before the recurrence over
//     superblock k and consumed after it.
//   * the partial sums C h of 8 tokens are added across the 8 lanes of a channel with a transposing
//     butterfly (3 DPP steps, 21 instructions for 8 tokens), which leaves lane j with token j's sum:
//     it gates, rounds and stores that one value.
// Tokens past the end of the sequence enter as dt = 0, dt x = 0: they leave the state as it is.
constexpr int SW_CH = 32;      // channels per workgroup
constexpr int SW_SB = 64;      // tokens per superblock: one 16-token tile per wave
constexpr int SW_THREADS = 256;

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// NK: k steps of 64 the dt_proj contraction may take (dt_rank <= 64 NK); 0: dt_q is read, not computed.
// LAT: the form for one or two workgroups per CU, where a wave has its SIMD (almost) to itself and nothing but
// its own instruction order hides latencies: the LDS reads of group g + 1 are in flight under group g, the 16
// exponentials of a group are issued ahead of the two recurrence chains that consume them, and the gate of
// group g - 1 (a serial chain with two transcendentals) is spread between them.
template <int NK, int XM, bool LAT>
__global__ __launch_bounds__(SW_THREADS, LAT ? 1 : 3) void scan_sweep_kernel(Dev p, float *__restrict__ ssm_state) {
  constexpr bool FUSE_DT = NK > 0;
  constexpr int NKR = FUSE_DT ? NK : 1;
  __shared__ __attribute__((aligned(16))) float2 sDU[SW_SB][SW_CH + 1];  // (dt, dt x); odd pitch: a tile's token rows on different banks
  __shared__ __attribute__((aligned(16))) float4 sBC[SW_SB][NS / 2];     // (B[2g], B[2g+1], C[2g], C[2g+1])
  __shared__ float sDX[SW_SB][SW_CH + 1];                                 // D x
  __shared__ __attribute__((aligned(4))) int8_t sZ[SW_SB][SW_CH + 4];    // z code
  // Workgroups go to the 8 XCDs round-robin by index: give one XCD consecutive channel blocks, so the
  // blocks that share 128-byte lines of x, z and g share an L2.
  const int nblk = p.Di / SW_CH;
  const int bx = blockIdx.x;
  if (bx >= nblk) {  // appended workgroups only read ahead
    warm_read(p.warm, (bx - nblk) * gridDim.y + blockIdx.y, p.warm.blocks * gridDim.y);
    return;
  }
  const int cb = (nblk % 8 == 0) ? (bx & 7) * (nblk >> 3) + (bx >> 3) : bx;
  const int b = blockIdx.y;
  const int ch0 = cb * SW_CH;
  const size_t seq0 = (size_t)b * p.L;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- recurrence role: channel chl of the workgroup, states 2 ng and 2 ng + 1
  const int ng = lane & 7, chl = 8 * wave + (lane >> 3), chg = ch0 + chl;
  float a20, a21, h0 = 0.f, h1 = 0.f;
  {
    const unsigned short aw = *reinterpret_cast<const unsigned short *>(p.A_q + (size_t)chg * NS + 2 * ng);
    a20 = static_cast<float>(static_cast<int8_t>(aw & 0xff)) * (p.s_A * LOG2E);
    a21 = static_cast<float>(static_cast<int8_t>(aw >> 8)) * (p.s_A * LOG2E);
    if (ssm_state) {
      const float2 hv = *reinterpret_cast<const float2 *>(ssm_state + ((size_t)b * p.Di + chg) * NS + 2 * ng);
      h0 = hv.x;
      h1 = hv.y;
    }
  }
  const bool up4 = (ng & 4) != 0, up2 = (ng & 2) != 0, up1 = (ng & 1) != 0;

  // ---- tile role (v_mfma_i32_16x16x64_i8, weights as the A operand): token row lane % 16 of the wave's
  // 16-token tile; register r of result m is channel 16 m + 4 (lane / 16) + r of the workgroup.  Both
  // operands take the 16 bytes at k = 64 s + 16 (lane / 16) of their row.
  const int tokl = lane & 15, kq = lane >> 4;
  float bias_r[8], Dv_r[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int c = ch0 + 16 * (r >> 2) + 4 * kq + (r & 3);
    bias_r[r] = p.dt_bias[c];
    Dv_r[r] = p.s_D * static_cast<float>(p.D_q[c]);
  }
  v4i wfrag[2][NKR];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int s = 0; s < NKR; ++s) {
      wfrag[m][s] = v4i{0, 0, 0, 0};
      if constexpr (FUSE_DT) {
        const int kc = 64 * s + 16 * kq;
        if (kc < p.R) wfrag[m][s] = *reinterpret_cast<const v4i *>(p.W_dt + (size_t)(ch0 + 16 * m + tokl) * p.R + kc);
      }
    }
  const float sx = x_scale<XM>(p);

  struct Pre {
    v4i a[NKR];
    unsigned x[2], z[2], dtc[2];
    unsigned bq, cq;
  };
  auto issue = [&](Pre &r, int sb) {
    const size_t row = seq0 + min(sb * SW_SB + 16 * wave + tokl, p.L - 1);  // clamped rows are zeroed in produce
#pragma unroll
    for (int s = 0; s < NKR; ++s) {
      r.a[s] = v4i{0, 0, 0, 0};
      if constexpr (FUSE_DT) {
        const int kc = 64 * s + 16 * kq;
        if (kc < p.R) r.a[s] = *reinterpret_cast<const v4i *>(p.dtlow_q + row * p.lddl + kc);
      }
    }
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const int c = ch0 + 16 * m + 4 * kq;
      r.x[m] = *reinterpret_cast<const unsigned *>(p.x_q + row * p.Di + c);
      r.z[m] = *reinterpret_cast<const unsigned *>(p.z_q + row * p.ldz + c);
      r.dtc[m] = FUSE_DT ? 0u : *reinterpret_cast<const unsigned *>(p.dt_q + row * p.Di + c);
    }
    // B and C of token tid / 4, states 4 (tid % 4) .. + 4
    const size_t rowb = seq0 + min(sb * SW_SB + (tid >> 2), p.L - 1);
    r.bq = *reinterpret_cast<const unsigned *>(p.B_q + rowb * p.ldbc + 4 * (tid & 3));
    r.cq = *reinterpret_cast<const unsigned *>(p.C_q + rowb * p.ldbc + 4 * (tid & 3));
  };
  auto produce = [&](const Pre &r, int sb) {
    const int tl = 16 * wave + tokl;
    const int tok = sb * SW_SB + tl;
    const bool valid = tok < p.L;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      unsigned pk;
      if constexpr (FUSE_DT) {
        v4i acc = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < NKR; ++s) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wfrag[m][s], r.a[s], acc, 0, 0, 0);
        const int a4[4] = {acc[0], acc[1], acc[2], acc[3]};
        pk = requant_pack4(a4, p.m_dt);
        if (valid) *reinterpret_cast<unsigned *>(p.dt_out + (seq0 + tok) * p.Di + ch0 + 16 * m + 4 * kq) = pk;
      } else {
        pk = r.dtc[m];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = 16 * m + 4 * kq + i, idx = 4 * m + i;
        const int dtq = static_cast<int>(static_cast<int8_t>(pk >> (8 * i)));
        const int xr = static_cast<int>(static_cast<int8_t>(r.x[m] >> (8 * i)));
        float dt = softplus_f(p.s_dt * static_cast<float>(dtq) + bias_r[idx]);
        const float xv = x_value<XM>(p, xr, sx);
        float u = dt * xv, dx = Dv_r[idx] * xv;
        if (!valid) dt = u = dx = 0.f;
        sDU[tl][c] = make_float2(dt, u);
        sDX[tl][c] = dx;
      }
      *reinterpret_cast<unsigned *>(&sZ[tl][16 * m + 4 * kq]) = valid ? r.z[m] : 0u;
    }
    const int quarter = tid & 3, tb = tid >> 2;
    const bool validb = sb * SW_SB + tb < p.L;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      float4 v;
      v.x = p.s_B * static_cast<float>(static_cast<int8_t>(r.bq >> (16 * q)));
      v.y = p.s_B * static_cast<float>(static_cast<int8_t>(r.bq >> (16 * q + 8)));
      v.z = p.s_C * static_cast<float>(static_cast<int8_t>(r.cq >> (16 * q)));
      v.w = p.s_C * static_cast<float>(static_cast<int8_t>(r.cq >> (16 * q + 8)));
      if (!validb) v = make_float4(0.f, 0.f, 0.f, 0.f);
      sBC[tb][2 * quarter + q] = v;
    }
  };

  // outputs of this sequence behind buffer descriptors: a lane stores at 32-bit offset (token * Di + channel) and a
  // token past the end becomes an offset past the end, which the range test drops (no branch around the store);
  // the optional fp32 copy is an empty descriptor when it is not asked for
  const auto rg = buffer_over(p.g16 + seq0 * p.Di, p.L * p.Di * 2);
  const auto ry = p.y_f32 ? buffer_over(p.y_f32 + seq0 * p.Di, p.L * p.Di * 4) : buffer_over(p.x_q, 0);
  auto store_g = [&](int tok, float gv) {
    const unsigned e = tok >= 0 && tok < p.L ? static_cast<unsigned>(tok * p.Di + chg) : 0x1fffffffu;
    buffer_store_f16(rg, 2 * e, 0, gv);
    buffer_store_f32(ry, 4 * e, 0, gv);
  };
  auto group = [&](int g, int tok0) {  // tok0: index in the sequence of the group's first token
    float yp[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float2 du = sDU[8 * g + j][chl];
      const float4 bc = sBC[8 * g + j][ng];
      const float e0 = exp2_fast(du.x * a20), e1 = exp2_fast(du.x * a21);
      h0 = __builtin_fmaf(e0, h0, du.y * bc.x);
      h1 = __builtin_fmaf(e1, h1, du.y * bc.y);
      yp[j] = __builtin_fmaf(bc.w, h1, bc.z * h0);
    }
    const float dx = sDX[8 * g + ng][chl];
    const float zv = p.s_z * static_cast<float>(sZ[8 * g + ng][chl]);
    // lanes 0-3 of a channel keep tokens 0-3 and take their partner's (lane 7 - i) sums for them, lanes 4-7
    // the same for tokens 4-7; then pairs of tokens inside quads, then single tokens
    float q4[4], q2[2];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float keep = up4 ? yp[4 + k] : yp[k], send = up4 ? yp[k] : yp[4 + k];
      q4[k] = keep + dpp_f<0x141>(send);  // row_half_mirror
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const float keep = up2 ? q4[2 + k] : q4[k], send = up2 ? q4[k] : q4[2 + k];
      q2[k] = keep + dpp_f<0x4E>(send);  // quad_perm [2, 3, 0, 1]
    }
    const float keep = up1 ? q2[1] : q2[0], send = up1 ? q2[0] : q2[1];
    const float y = keep + dpp_f<0xB1>(send) + dx;  // quad_perm [1, 0, 3, 2]
    store_g(tok0 + ng, silu_gate(y, zv));
  };

  // ---- the latency-ordered form of the same group
  struct Rec {
    float2 du[8];
    float4 bc[8];
    float dx;
    int z;
  };
  auto load = [&](Rec &r, int g) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      r.du[j] = sDU[8 * g + j][chl];
      r.bc[j] = sBC[8 * g + j][ng];
    }
    r.dx = sDX[8 * g + ng][chl];
    r.z = static_cast<int>(sZ[8 * g + ng][chl]);
  };
  struct Pending {  // a group whose sums are complete and whose gate is still to be applied
    float y, zs;
    int tok;
  };
  auto group_lat = [&](const Rec &r, int tok0, Pending &pend) {
    float e0[8], e1[8], ub0[8], ub1[8];
    float gt = 0.f, gy = pend.y, gz = pend.zs;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float m0 = r.du[j].x * a20, m1 = r.du[j].x * a21;
      e0[j] = exp2_fast(m0);
      ub0[j] = r.du[j].y * r.bc[j].x;
      e1[j] = exp2_fast(m1);
      ub1[j] = r.du[j].y * r.bc[j].y;
      // the previous group's gate, one step per token of this one
      if (j == 0) gt = exp2_fast(-gz * LOG2E);
      if (j == 2) gt = 1.f + gt;
      if (j == 4) gt = __builtin_amdgcn_rcpf(gt);
      if (j == 6) gy = gy * gz * gt;
    }
    store_g(pend.tok, gy);
    __builtin_amdgcn_sched_barrier(0);
    float yp[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      h0 = __builtin_fmaf(e0[j], h0, ub0[j]);
      h1 = __builtin_fmaf(e1[j], h1, ub1[j]);
      yp[j] = __builtin_fmaf(r.bc[j].w, h1, r.bc[j].z * h0);
    }
    __builtin_amdgcn_sched_barrier(0);
    float q4[4], q2[2];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float keep = up4 ? yp[4 + k] : yp[k], send = up4 ? yp[k] : yp[4 + k];
      q4[k] = keep + dpp_f<0x141>(send);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const float keep = up2 ? q4[2 + k] : q4[k], send = up2 ? q4[k] : q4[2 + k];
      q2[k] = keep + dpp_f<0x4E>(send);
    }
    const float keep = up1 ? q2[1] : q2[0], send = up1 ? q2[0] : q2[1];
    pend.y = keep + dpp_f<0xB1>(send) + r.dx;
    pend.zs = p.s_z * static_cast<float>(r.z);
    pend.tok = tok0 + ng;
  };
  auto flush = [&](Pending &pend) {  // the gate of the last group of a superblock
    store_g(pend.tok, silu_gate(pend.y, pend.zs));
    pend.tok = -1;
  };

  const int nsb = (p.L + SW_SB - 1) / SW_SB;
  Pre pre;
  issue(pre, 0);
  produce(pre, 0);
  __syncthreads();
  for (int sb = 0; sb < nsb; ++sb) {
    const bool more = sb + 1 < nsb;
    if (more) issue(pre, sb + 1);
    const int ngroups = (min(SW_SB, p.L - sb * SW_SB) + 7) >> 3;
    if constexpr (LAT) {
      Rec ra, rb;
      Pending pend{0.f, 0.f, -1};
      load(ra, 0);
      for (int g = 0; g < ngroups; g += 2) {
        if (g + 1 < ngroups) load(rb, g + 1);
        group_lat(ra, sb * SW_SB + 8 * g, pend);
        if (g + 2 < ngroups) load(ra, g + 2);
        if (g + 1 < ngroups) group_lat(rb, sb * SW_SB + 8 * g + 8, pend);
      }
      flush(pend);
    } else {
      for (int g = 0; g < ngroups; ++g) group(g, sb * SW_SB + 8 * g);
    }
    __syncthreads();  // every wave is done reading this superblock
    if (more) produce(pre, sb + 1);
    __syncthreads();
  }
  if (ssm_state)
    *reinterpret_cast<float2 *>(ssm_state + ((size_t)b * p.Di + chg) * NS + 2 * ng) = make_float2(h0, h1);
}

// ---------------------------------------------------------------- decode: one step
// 4 lanes per channel, each owning 4 of the 16 states as one float4.  FUSE_DT: the step also forms
// its own dt code, dt_q = q(W_dt[d, :] . dt_low[b, :], m_dt) (dt_proj, K = dt_rank): the four lanes of
// a channel share the 16-byte pieces of the two rows and add their parts with two shuffles.
template <bool FUSE_DT, int XM = X_I8>
__global__ __launch_bounds__(256) void scan_step_kernel(Dev p, float *__restrict__ ssm_state, int Bt) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // (b, d, quad)
  const size_t total = (size_t)Bt * p.Di * 4;
  const bool live = idx < total;
  const size_t id = live ? idx : total - 1;
  const int q = static_cast<int>(id & 3);
  const size_t bd = id >> 2;
  const int b = static_cast<int>(bd / p.Di), d = static_cast<int>(bd % p.Di);

  float4 hv = reinterpret_cast<const float4 *>(ssm_state)[id];
  float h[4] = {hv.x, hv.y, hv.z, hv.w};
  const unsigned aw = *reinterpret_cast<const unsigned *>(p.A_q + (size_t)d * NS + 4 * q);
  const unsigned bw = *reinterpret_cast<const unsigned *>(p.B_q + (size_t)b * p.ldbc + 4 * q);
  const unsigned cw = *reinterpret_cast<const unsigned *>(p.C_q + (size_t)b * p.ldbc + 4 * q);
  // (a compile-time choice: a run-time test of the pointer would put this load behind a branch and
  // cost the step one more memory round trip)
  const float xv = x_value<XM>(p, XM == X_F16 ? static_cast<int>(__half_as_ushort(p.x_f16[(size_t)b * p.Di + d]))
                                               : static_cast<int>(p.x_q[(size_t)b * p.Di + d]), x_scale<XM>(p));
  int dtq;
  if (FUSE_DT) {
    const int8_t *wrow = p.W_dt + (size_t)d * p.R;
    const int8_t *arow = p.dtlow_q + (size_t)b * p.lddl;
    int acc = 0;
    for (int kc = 16 * q; kc < p.R; kc += 64) {
      const v4i w = *reinterpret_cast<const v4i *>(wrow + kc);
      const v4i a = *reinterpret_cast<const v4i *>(arow + kc);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_sdot4(a[e], w[e], acc, false);
    }
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    const float v = __builtin_amdgcn_fmed3f(static_cast<float>(acc) * p.m_dt, -128.f, 127.f);
    dtq = static_cast<int>(__builtin_rintf(v));
    if (live && q == 0 && p.dt_out) p.dt_out[(size_t)b * p.Di + d] = static_cast<int8_t>(dtq);
  } else {
    dtq = p.dt_q[(size_t)b * p.Di + d];
  }
  const float dt = softplus_f(p.s_dt * static_cast<float>(dtq) + p.dt_bias[d]);
  const float zv = p.s_z * static_cast<float>(p.z_q[(size_t)b * p.ldz + d]);
  const float u = dt * xv;
  float y = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float a2 = static_cast<float>(static_cast<int8_t>(aw >> (8 * j))) * (p.s_A * LOG2E);
    const float Bv = p.s_B * static_cast<float>(static_cast<int8_t>(bw >> (8 * j)));
    const float Cv = p.s_C * static_cast<float>(static_cast<int8_t>(cw >> (8 * j)));
    // (explicit fused multiply-adds: both step kernels must round alike whatever the compiler contracts)
    h[j] = __builtin_fmaf(exp2_fast(dt * a2), h[j], u * Bv);
    y = __builtin_fmaf(Cv, h[j], y);
  }
  y += __shfl_xor(y, 1);
  y += __shfl_xor(y, 2);
  y = __builtin_fmaf(p.s_D * static_cast<float>(p.D_q[d]), xv, y);
  const float g = silu_gate(y, zv);
  if (live) {
    reinterpret_cast<float4 *>(ssm_state)[id] = make_float4(h[0], h[1], h[2], h[3]);
    if (q == 0) {
      p.g16[(size_t)b * p.Di + d] = __float2half_rn(g);
      if (p.y_f32) p.y_f32[(size_t)b * p.Di + d] = g;
    }
  }
}

// The same step with dt_proj inside for many sequences: a workgroup owns 64 channels and walks BB
// sequences, so the lanes keep their pieces of the W_dt rows (NP pieces of 16 bytes per lane:
// dt_rank <= 64 NP) in registers and W_dt is read Bt / BB times instead of Bt times.  All state and
// code loads of the BB sequences are requested before the first dot product.  BB = 4 (measured at
// 2.8B, batch 64: step 47.5 us with the separate dt_proj GEMM, 44.6 us with BB = 4 or 2, 47.4 us
// with BB = 8, whose 183 registers leave two waves per SIMD and nothing to overlap the loads with).
// PART: x_proj's K was split over the grid and its reduce kernel left out; the workgroup adds up the
// partial sums of its BB sequences (R + 32 columns each) and requantizes them into LDS first, after
// its weight pieces are requested.  Integer sums: the codes are the reduce kernel's bit for bit.
template <int XM, int BB, int NP, bool PART>
__global__ __launch_bounds__(256) void scan_step_batch_kernel(Dev p, float *__restrict__ ssm_state, int Bt) {
  constexpr int LDP = NP * 64 + 2 * NS;  // R <= 64 NP
  __shared__ __attribute__((aligned(16))) int8_t dbc[PART ? BB : 1][LDP];
  const int q = threadIdx.x & 3;
  const int d = blockIdx.x * 64 + (threadIdx.x >> 2);
  const bool live = d < p.Di;
  const int dd = live ? d : p.Di - 1;
  const int b0 = blockIdx.y * BB;

  v4i w[NP];
#pragma unroll
  for (int j = 0; j < NP; ++j) {
    const int kc = 16 * q + 64 * j;
    w[j] = v4i{0, 0, 0, 0};
    if (kc < p.R) w[j] = *reinterpret_cast<const v4i *>(p.W_dt + (size_t)dd * p.R + kc);
  }
  const unsigned aw = *reinterpret_cast<const unsigned *>(p.A_q + (size_t)dd * NS + 4 * q);
  const float bias = p.dt_bias[dd];
  const float Dv = p.s_D * static_cast<float>(p.D_q[dd]);
  const float sx = x_scale<XM>(p);
  float a2[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) a2[j] = static_cast<float>(static_cast<int8_t>(aw >> (8 * j))) * (p.s_A * LOG2E);

  float4 hv[BB];
  unsigned bw[BB], cw[BB];
  float xv[BB], zv[BB];
  v4i a[BB][NP];
#pragma unroll
  for (int i = 0; i < BB; ++i) {
    const size_t b = static_cast<size_t>(min(b0 + i, Bt - 1));  // past the batch: loaded again, never stored
    hv[i] = reinterpret_cast<const float4 *>(ssm_state)[(b * p.Di + dd) * 4 + q];
    xv[i] = x_value<XM>(p, XM == X_F16 ? static_cast<int>(__half_as_ushort(p.x_f16[b * p.Di + dd]))
                                       : static_cast<int>(p.x_q[b * p.Di + dd]), sx);
    zv[i] = p.s_z * static_cast<float>(p.z_q[b * p.ldz + dd]);
  }
  if constexpr (PART) {
    const int NX = p.R + 2 * NS, per_row = NX / 4;
    for (int g = threadIdx.x; g < BB * per_row; g += 256) {
      const int i = g / per_row, gn = (g % per_row) * 4;
      const size_t b = static_cast<size_t>(min(b0 + i, Bt - 1));
      v4i v[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        v[s] = v4i{0, 0, 0, 0};
        if (s < p.dbc_splits) v[s] = *reinterpret_cast<const v4i *>(p.dbc_part + ((size_t)s * Bt + b) * NX + gn);
      }
      int sum[4] = {0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) sum[e] += v[s][e];
      const float m = gn < p.R ? p.m_x_dt : (gn < p.R + NS ? p.m_x_B : p.m_x_C);
      *reinterpret_cast<unsigned *>(&dbc[i][gn]) = requant_pack4(sum, m);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < BB; ++i) {
    const size_t b = static_cast<size_t>(min(b0 + i, Bt - 1));
    if constexpr (PART) {
      bw[i] = *reinterpret_cast<const unsigned *>(&dbc[i][p.R + 4 * q]);
      cw[i] = *reinterpret_cast<const unsigned *>(&dbc[i][p.R + NS + 4 * q]);
    } else {
      bw[i] = *reinterpret_cast<const unsigned *>(p.B_q + b * p.ldbc + 4 * q);
      cw[i] = *reinterpret_cast<const unsigned *>(p.C_q + b * p.ldbc + 4 * q);
    }
    if constexpr (!PART) {
#pragma unroll
      for (int j = 0; j < NP; ++j) {
        const int kc = 16 * q + 64 * j;
        a[i][j] = v4i{0, 0, 0, 0};
        if (kc < p.R) a[i][j] = *reinterpret_cast<const v4i *>(p.dtlow_q + b * p.lddl + kc);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < BB; ++i) {
    const size_t b = static_cast<size_t>(b0 + i);
    const bool on = live && b0 + i < Bt;
    if constexpr (PART) {  // out of LDS just before use: held for all BB sequences at once they cost a wave per SIMD
#pragma unroll
      for (int j = 0; j < NP; ++j) {
        const int kc = 16 * q + 64 * j;
        a[i][j] = v4i{0, 0, 0, 0};
        if (kc < p.R) a[i][j] = *reinterpret_cast<const v4i *>(&dbc[i][kc]);
      }
    }
    int acc = 0;
#pragma unroll
    for (int j = 0; j < NP; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_sdot4(a[i][j][e], w[j][e], acc, false);
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    const int dtq = static_cast<int>(__builtin_rintf(__builtin_amdgcn_fmed3f(static_cast<float>(acc) * p.m_dt, -128.f, 127.f)));
    if (on && q == 0 && p.dt_out) p.dt_out[b * p.Di + d] = static_cast<int8_t>(dtq);
    const float dt = softplus_f(p.s_dt * static_cast<float>(dtq) + bias);
    const float u = dt * xv[i];
    float h[4] = {hv[i].x, hv[i].y, hv[i].z, hv[i].w};
    float y = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float Bv = p.s_B * static_cast<float>(static_cast<int8_t>(bw[i] >> (8 * j)));
      const float Cv = p.s_C * static_cast<float>(static_cast<int8_t>(cw[i] >> (8 * j)));
      h[j] = __builtin_fmaf(exp2_fast(dt * a2[j]), h[j], u * Bv);
      y = __builtin_fmaf(Cv, h[j], y);
    }
    y += __shfl_xor(y, 1);
    y += __shfl_xor(y, 2);
    y = __builtin_fmaf(Dv, xv[i], y);
    const float g = silu_gate(y, zv[i]);
    if (on) {
      reinterpret_cast<float4 *>(ssm_state)[(b * p.Di + d) * 4 + q] = make_float4(h[0], h[1], h[2], h[3]);
      if (q == 0) {
        p.g16[b * p.Di + d] = __float2half_rn(g);
        if (p.y_f32) p.y_f32[b * p.Di + d] = g;
      }
    }
  }
}

Dev make_dev(const ScanArgs &a) {
  Dev p{};
  p.x_q = a.x_q; p.dt_q = a.dt_q; p.z_q = a.z_q; p.B_q = a.B_q; p.C_q = a.C_q; p.A_q = a.A_q; p.D_q = a.D_q;
  p.dt_bias = a.dt_bias; p.ldz = a.ldz; p.ldbc = a.ldbc;
  p.s_x = a.s_x; p.s_dt = a.s_dt; p.s_z = a.s_z; p.s_B = a.s_B; p.s_C = a.s_C; p.s_A = a.s_A; p.s_D = a.s_D;
  p.L = a.L; p.Di = a.Di; p.g16 = a.g16; p.y_f32 = a.y_f32;
  p.dtlow_q = a.dtlow_q; p.W_dt = a.W_dt; p.lddl = a.lddl; p.R = a.R; p.m_dt = a.m_dt; p.dt_out = a.dt_out;
  if (a.dtlow_q && a.dt_out) p.dt_q = a.dt_out;
  p.x_f16 = a.x_f16;
  p.s_x_slot = a.s_x_slot;
  p.dbc_part = a.dbc_part; p.dbc_splits = a.dbc_splits; p.m_x_dt = a.m_x_dt; p.m_x_B = a.m_x_B; p.m_x_C = a.m_x_C;
  p.x_off = -a.s_x * static_cast<float>(a.x_zero_point);  // -0.f for the symmetric grid: adds nothing
  for (int r = 0; r < 3; ++r) {
    const bool on = a.warm_ptr[r] && aligned(a.warm_ptr[r], 16);
    p.warm.ptr[r] = on ? static_cast<const uint4 *>(a.warm_ptr[r]) : nullptr;
    p.warm.n16[r] = on ? static_cast<unsigned>(std::min<size_t>(a.warm_bytes[r] / 16, 0xffffffffu)) : 0u;
  }
  p.warm.blocks = 0;
  return p;
}

// Chunk length.  A (chunk, 256-channel) tile is one workgroup, i.e. one wave on each SIMD of
// a CU.  Take the fewest chunks (least per-chunk state traffic: 128 B per channel and chunk, read
// and written twice) that give at least 4 workgroups per CU (the recurrence needs several waves
// per SIMD to hide its own latencies) and fill the last round of 256 CUs to 90 %; chunks are
// never shorter than 16 tokens.
void choose_chunks(int Bt, int L, int Di, int *T, int *nchunks) {
  const long per_chunk = (long)Bt * ((Di + SCAN_THREADS - 1) / SCAN_THREADS);
  // Plenty of workgroups even at one staging block of B / C per chunk: 64-token chunks measure 4-6 % faster
  // than the longer ones the rule below would take (three workgroups are resident per CU, so many short
  // ones fill the tail better, and a chunk of exactly one staging block has no ragged second block).
  if (per_chunk * ((L + TB - 1) / TB) >= 1280) {
    *T = TB;
    *nchunks = (L + TB - 1) / TB;
    return;
  }
  const int max_chunks = (L + 15) / 16;
  int best_n = max_chunks > 0 ? max_chunks : 1;
  for (int n = 1; n <= max_chunks; ++n) {
    int t = (L + n - 1) / n;
    t = (t + 7) / 8 * 8;
    const int real_n = (L + t - 1) / t;
    const long wgs = per_chunk * real_n;
    const long rounds = (wgs + 255) / 256;
    // equal chunks when L allows (a ragged last chunk leaves SIMDs idle), unless there are many
    const bool full = wgs >= 1024 && (double)wgs / (double)(rounds * 256) >= 0.9 && (L % t == 0 || real_n >= 16);
    if (full) {
      best_n = real_n;
      break;
    }
  }
  int t = (L + best_n - 1) / best_n;
  t = (t + 7) / 8 * 8;
  *T = t;
  *nchunks = (L + t - 1) / t;
}

}  // namespace

size_t scan_workspace_bytes(int Bt, int L, int Di) {
  int T, nc;
  choose_chunks(Bt, L, Di, &T, &nc);
  const size_t hloc = align_up((size_t)Bt * nc * Di * NS * sizeof(float), 256);
  const size_t ssum = align_up((size_t)Bt * nc * Di * sizeof(float), 256);
  return hloc + ssum;
}

// 0: the cheaper form by the estimate below, 1: always chunked, 2: one sweep wherever its layout rules hold
std::atomic<int> g_scan_variant_hook{0};

namespace {

int scan_x_mode(const ScanArgs &a) {
  return a.x_f16 ? X_F16 : (a.s_x_slot ? X_I8DYN : (a.x_format == QUAMBA_XFMT_E4M3 ? X_E4M3 : (a.x_format == QUAMBA_XFMT_LOG2 ? X_LOG2 : X_I8)));
}

// The sweep reads x, z and dt four channels at a time, B and C four states at a time and the state as pairs.
bool sweep_layout_ok(const ScanArgs &a) {
  if (a.x_f16 || a.L < 1 || a.Bt < 1 || a.Bt > 65535 || a.Di % SW_CH) return false;
  if ((long long)a.L * a.Di * 4 >= 0x7fffffffLL) return false;  // 32-bit byte offsets inside one sequence's outputs
  if (!aligned(a.x_q, 4) || !aligned(a.z_q, 4) || a.ldz % 4 || !aligned(a.B_q, 4) || !aligned(a.C_q, 4) || a.ldbc % 4 ||
      !aligned(a.A_q, 2) || (a.ssm_state && !aligned(a.ssm_state, 8)))
    return false;
  if (a.dtlow_q)
    return a.W_dt && a.dt_out && a.R >= 16 && a.R <= 256 && a.R % 16 == 0 && a.lddl % 16 == 0 && a.lddl >= a.R &&
           aligned(a.dtlow_q, 16) && aligned(a.W_dt, 16) && aligned(a.dt_out, 4);
  return aligned(a.dt_q, 4);
}

// Which form is faster, from fits to measured times (microseconds; W = workgroups of the sweep = Bt * Di / 32,
// k = workgroups per CU):
//   sweep    3.6 + L * s(k): a wave alone on its SIMD walks a token in 65 ns (a lone wave issues one instruction
//            of any kind per 5.4 clocks, and a token costs it about 27); two per SIMD 98 ns; from three on the
//            SIMD is busy, 40 ns per token and wave
//   chunked  30 + L * (W / 256) * 52 ns: three launches and the carry, every exponential taken twice
// so the sweep takes the short sequences and the batches, the chunked form a long single sequence.
bool sweep_is_cheaper(const ScanArgs &a) {
  const double W = (double)a.Bt * (a.Di / SW_CH);
  const int k = (int)std::ceil(W / 256.0);
  const double s = k <= 1 ? 0.0645 : (k == 2 ? 0.098 : 0.040 * k);
  const double sweep = 3.6 + a.L * s;
  const double chunked = 30.0 + (double)a.L * (W / 256.0) * 0.052;
  return sweep < chunked;
}

template <int NK, int XM, bool LAT>
int run_sweep(const Dev &p, const ScanArgs &a, hipStream_t st) {
  Dev q = p;
  if (q.warm.n16[0] || q.warm.n16[1] || q.warm.n16[2]) q.warm.blocks = std::max(1, 96 / a.Bt);  // about 96 workgroups in all
  hipLaunchKernelGGL((scan_sweep_kernel<NK, XM, LAT>), dim3(a.Di / SW_CH + q.warm.blocks, a.Bt), dim3(SW_THREADS), 0, st, q,
                     a.ssm_state);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

// lat: at most one workgroup per CU, where the latency-ordered form pays: 10-15 % (with two per CU it
// measures the same as the plain form); compiled for int8 x on the calibrated grid only
template <int XM>
int dispatch_sweep(const Dev &p, const ScanArgs &a, hipStream_t st) {
  const bool lat = XM == X_I8 && (long)a.Bt * (a.Di / SW_CH) <= 256;
  if constexpr (XM == X_I8) {
    if (lat) {
      if (!a.dtlow_q) return run_sweep<0, XM, true>(p, a, st);
      if (a.R <= 192) return run_sweep<3, XM, true>(p, a, st);
      return run_sweep<4, XM, true>(p, a, st);
    }
  }
  if (!a.dtlow_q) return run_sweep<0, XM, false>(p, a, st);
  if (a.R <= 192) return run_sweep<3, XM, false>(p, a, st);
  return run_sweep<4, XM, false>(p, a, st);
}

}  // namespace

int launch_scan_prefill(const ScanArgs &a, void *ws, size_t ws_bytes, hipStream_t st) {
  if (ws_bytes < scan_workspace_bytes(a.Bt, a.L, a.Di))
    return fail(QUAMBA_EWORKSPACE, "scan: workspace %zu < %zu", ws_bytes, scan_workspace_bytes(a.Bt, a.L, a.Di));
  Dev p = make_dev(a);
  const int variant = g_scan_variant_hook.load(std::memory_order_relaxed);
  if (variant != 1 && sweep_layout_ok(a) && (variant == 2 || sweep_is_cheaper(a))) {
    switch (scan_x_mode(a)) {
      case X_E4M3: return dispatch_sweep<X_E4M3>(p, a, st);
      case X_LOG2: return dispatch_sweep<X_LOG2>(p, a, st);
      case X_I8DYN: return dispatch_sweep<X_I8DYN>(p, a, st);
      default: return dispatch_sweep<X_I8>(p, a, st);
    }
  }
  choose_chunks(a.Bt, a.L, a.Di, &p.T, &p.nchunks);
  if ((long long)p.T * std::max(a.ldz, (a.y_f32 ? 4 : 2) * a.Di) > 0x7fffffffLL)  // 32-bit offsets inside a chunk
    return fail(QUAMBA_EUNSUPPORTED, "scan: a chunk of %d tokens x %d channels exceeds 2^31 bytes", p.T, a.Di);
  p.hloc = static_cast<float *>(ws);
  p.ssum = reinterpret_cast<float *>(static_cast<char *>(ws) +
                                     align_up((size_t)a.Bt * p.nchunks * a.Di * NS * sizeof(float), 256));
  dim3 grid((a.Di + SCAN_THREADS - 1) / SCAN_THREADS, p.nchunks, a.Bt);
  const int xm = scan_x_mode(a);
#define QUAMBA_XM_SWITCH(CALL) \
  switch (xm) {                \
    case X_F16: CALL(X_F16); break;   \
    case X_E4M3: CALL(X_E4M3); break; \
    case X_LOG2: CALL(X_LOG2); break; \
    case X_I8DYN: CALL(X_I8DYN); break; \
    default: CALL(X_I8); break;       \
  }
  if (a.dtlow_q) {
    if (!a.W_dt || !a.dt_out || a.R < 16 || a.R % 16 || a.lddl % 16 || a.lddl < a.R || a.Di % 4 ||
        !aligned(a.dtlow_q, 16) || !aligned(a.W_dt, 16) || !aligned(a.dt_out, 4))
      return fail(QUAMBA_EUNSUPPORTED, "scan: fused dt_proj needs dt_rank and lddl multiples of 16, Di a multiple "
                                       "of 4, 16-byte aligned dt_low and W_dt");
#define QUAMBA_PASS1F(XMV) hipLaunchKernelGGL((scan_chunk_kernel<false, true, XMV>), grid, dim3(SCAN_THREADS), 0, st, p)
    QUAMBA_XM_SWITCH(QUAMBA_PASS1F)
#undef QUAMBA_PASS1F
  } else {
#define QUAMBA_PASS1(XMV) hipLaunchKernelGGL((scan_chunk_kernel<false, false, XMV>), grid, dim3(SCAN_THREADS), 0, st, p)
    QUAMBA_XM_SWITCH(QUAMBA_PASS1)
#undef QUAMBA_PASS1
  }
  QUAMBA_LAUNCH_CHECK();
  const size_t n2 = (size_t)a.Bt * a.Di * NS;
  hipLaunchKernelGGL(scan_carry_kernel, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, st, p, a.ssm_state,
                     a.Bt);
  QUAMBA_LAUNCH_CHECK();
  dim3 grid3 = grid;
  if (p.warm.n16[0] || p.warm.n16[1] || p.warm.n16[2]) {  // about 128 workgroups that read ahead
    p.warm.blocks = std::max(1, (int)(128 / ((long)p.nchunks * a.Bt)));
    grid3.x += p.warm.blocks;
  }
#define QUAMBA_PASS3(XMV) hipLaunchKernelGGL((scan_chunk_kernel<true, false, XMV>), grid3, dim3(SCAN_THREADS), 0, st, p)
  QUAMBA_XM_SWITCH(QUAMBA_PASS3)
#undef QUAMBA_PASS3
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int launch_scan_step(const ScanArgs &a, hipStream_t st) {
  if (a.dbc_part && (!a.dtlow_q || a.R > 256 || a.dbc_splits < 1 || a.dbc_splits > 8 || !aligned(a.dbc_part, 16)))
    return fail(QUAMBA_EUNSUPPORTED, "scan_step: partial x_proj sums need the fused dt_proj, dt_rank <= 256 and at most 8 "
                                     "partial results");
  Dev p = make_dev(a);
  p.L = 1;
  const int xm = scan_x_mode(a);
  const size_t n = (size_t)a.Bt * a.Di * 4;
  if (a.dtlow_q) {
    if (!a.W_dt || a.R < 16 || a.R % 16 || a.lddl % 16 || a.lddl < a.R || !aligned(a.dtlow_q, 16) || !aligned(a.W_dt, 16))
      return fail(QUAMBA_EUNSUPPORTED, "scan_step: fused dt_proj needs dt_rank and lddl multiples of 16 and 16-byte "
                                       "aligned dt_low and W_dt");
    constexpr int BB = 4;
    const int np = (a.R + 63) / 64;
    if (a.dbc_part && a.Bt <= 16) {  // a workgroup per sequence and 64 channels, as the kernel below, plus the sums
      const dim3 grid((unsigned)((a.Di + 63) / 64), (unsigned)a.Bt);
#define QUAMBA_STEP_ONE(XMV)                                                                                                 \
  do {                                                                                                                       \
    if (np == 1) hipLaunchKernelGGL((scan_step_batch_kernel<XMV, 1, 1, true>), grid, dim3(256), 0, st, p, a.ssm_state, a.Bt);      \
    else if (np == 2) hipLaunchKernelGGL((scan_step_batch_kernel<XMV, 1, 2, true>), grid, dim3(256), 0, st, p, a.ssm_state, a.Bt); \
    else if (np == 3) hipLaunchKernelGGL((scan_step_batch_kernel<XMV, 1, 3, true>), grid, dim3(256), 0, st, p, a.ssm_state, a.Bt); \
    else hipLaunchKernelGGL((scan_step_batch_kernel<XMV, 1, 4, true>), grid, dim3(256), 0, st, p, a.ssm_state, a.Bt);              \
  } while (0)
      QUAMBA_XM_SWITCH(QUAMBA_STEP_ONE)
#undef QUAMBA_STEP_ONE
    } else if (a.Bt > 16 && np <= 4) {  // many sequences: keep the W_dt rows in registers over BB of them
      const dim3 grid((unsigned)((a.Di + 63) / 64), (unsigned)((a.Bt + BB - 1) / BB));
#define QUAMBA_STEP_BATCH_NP(XMV, NPV)                                                                                  \
  do {                                                                                                                \
    if (a.dbc_part) hipLaunchKernelGGL((scan_step_batch_kernel<XMV, BB, NPV, true>), grid, dim3(256), 0, st, p, a.ssm_state, a.Bt); \
    else hipLaunchKernelGGL((scan_step_batch_kernel<XMV, BB, NPV, false>), grid, dim3(256), 0, st, p, a.ssm_state, a.Bt);          \
  } while (0)
#define QUAMBA_STEP_BATCH(XMV)                      \
  do {                                              \
    if (np == 1) QUAMBA_STEP_BATCH_NP(XMV, 1);      \
    else if (np == 2) QUAMBA_STEP_BATCH_NP(XMV, 2); \
    else if (np == 3) QUAMBA_STEP_BATCH_NP(XMV, 3); \
    else QUAMBA_STEP_BATCH_NP(XMV, 4);              \
  } while (0)
      QUAMBA_XM_SWITCH(QUAMBA_STEP_BATCH)
#undef QUAMBA_STEP_BATCH
#undef QUAMBA_STEP_BATCH_NP
    } else {
#define QUAMBA_STEPF(XMV) \
  hipLaunchKernelGGL((scan_step_kernel<true, XMV>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, a.ssm_state, a.Bt)
      QUAMBA_XM_SWITCH(QUAMBA_STEPF)
#undef QUAMBA_STEPF
    }
  } else {
#define QUAMBA_STEP(XMV) \
  hipLaunchKernelGGL((scan_step_kernel<false, XMV>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, a.ssm_state, a.Bt)
    QUAMBA_XM_SWITCH(QUAMBA_STEP)
#undef QUAMBA_STEP
  }
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

#undef QUAMBA_XM_SWITCH

}  // namespace quamba

extern "C" void quamba_debug_set_scan_variant(int v) { quamba::g_scan_variant_hook.store(v); }
