// Instruction-rate probes behind the roofline statements of this library (diagnostics; nothing on the
// hot path calls them).  Each probe is a loop over registers only, so what it times is the issue rate
// of one instruction class on every SIMD of the chip at once:
//   QUAMBA_PROBE_FMA_F32   v_fma_f32 on 8 independent registers
//   QUAMBA_PROBE_EXP_F32   v_exp_f32 on 8 independent registers (the decay factor of the scan, Eq. 1)
//   QUAMBA_PROBE_SCAN_MIX  the scan's state update per (token, channel, state): 1 exp, 2 mul, 2 fma
//   QUAMBA_PROBE_MFMA_I8   v_mfma_i32_32x32x32_i8 on 4 independent accumulators, operands all zero
//   QUAMBA_PROBE_MFMA_I8_RANDOM  the same with seeded random int8 operands (the rate of the matrix
//                          cores depends on the data: the part is power-limited)
// The result is instructions per second and per SIMD; the caller turns it into cycles with the clock.
#include "common.h"
#include "device_util.h"

namespace quamba {

namespace {

constexpr int REGS = 8;

template <int MODE>
__global__ __launch_bounds__(256) void valu_probe_kernel(float *out, int iters, float seed, unsigned long long *clk) {
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  float a[REGS], A[REGS], Bv[REGS], Cv[REGS];
#pragma unroll
  for (int r = 0; r < REGS; ++r) {
    a[r] = seed + 0.001f * (float)(threadIdx.x + r);
    A[r] = -(float)(r + 1) * (1.f + seed * 1e-3f);
    Bv[r] = 0.01f * (float)(r + 1) + seed * 1e-4f;
    Cv[r] = 0.02f * (float)(r + 1) - seed * 1e-4f;
  }
  const float m = 0.5f + seed * 1e-6f, c = 0.01f + seed * 1e-6f;
  float dt = 0.05f + seed * 1e-5f, y = 0.f;
#pragma unroll 4
  for (int it = 0; it < iters; ++it) {
    if constexpr (MODE == QUAMBA_PROBE_SCAN_MIX) {
      dt = __builtin_fmaf(dt, m, c);  // a fresh step size per token (converges to about 0.02)
      const float dtx = dt * seed;
#pragma unroll
      for (int r = 0; r < REGS; ++r) {  // h = exp2(dt A) h + (dt x) B;  y += C h
        const float e = __builtin_amdgcn_exp2f(dt * A[r]);
        a[r] = __builtin_fmaf(e, a[r], dtx * Bv[r]);
        y = __builtin_fmaf(Cv[r], a[r], y);
      }
    } else if constexpr (MODE == QUAMBA_PROBE_MIX_NOEXP) {  // the same update without the exponential
      dt = __builtin_fmaf(dt, m, c);
      const float dtx = dt * seed;
#pragma unroll
      for (int r = 0; r < REGS; ++r) {
        const float e = dt * A[r] + 1.0f;  // one instruction in the exponential's place
        a[r] = __builtin_fmaf(e, a[r], dtx * Bv[r]);
        y = __builtin_fmaf(Cv[r], a[r], y);
      }
    } else if constexpr (MODE == QUAMBA_PROBE_MIX_GROUPED) {  // the same update, the 8 exponentials issued as one run
      dt = __builtin_fmaf(dt, m, c);
      const float dtx = dt * seed;
      float e[REGS];
#pragma unroll
      for (int r = 0; r < REGS; ++r) e[r] = dt * A[r];
#pragma unroll
      for (int r = 0; r < REGS; ++r) e[r] = __builtin_amdgcn_exp2f(e[r]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int r = 0; r < REGS; ++r) {
        a[r] = __builtin_fmaf(e[r], a[r], dtx * Bv[r]);
        y = __builtin_fmaf(Cv[r], a[r], y);
      }
      __builtin_amdgcn_sched_barrier(0);
    } else if constexpr (MODE == QUAMBA_PROBE_FMA_EXP_INDEP) {  // 4 multiply-adds and 4 exponentials, all independent
#pragma unroll
      for (int r = 0; r < REGS; r += 2) {
        a[r] = __builtin_fmaf(a[r], m, c);
        a[r + 1] = __builtin_amdgcn_exp2f(-a[r + 1]);
      }
    } else {
#pragma unroll
      for (int r = 0; r < REGS; ++r) {
        if constexpr (MODE == QUAMBA_PROBE_FMA_F32) a[r] = __builtin_fmaf(a[r], m, c);
        else if constexpr (MODE == QUAMBA_PROBE_MUL_F32) a[r] = a[r] * m + 0.f * c;
        else a[r] = __builtin_amdgcn_exp2f(-a[r]);  // x -> 2^-x stays in (0.5, 1): no denormals, no overflow
      }
    }
  }
  float s = y;
#pragma unroll
  for (int r = 0; r < REGS; ++r) s += a[r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {  // shader-clock and constant-rate-clock ticks this wave lived
    clk[0] = clock64() - c0;
    clk[1] = wall_clock64() - w0;
  }
}

template <bool RANDOM>
__global__ __launch_bounds__(256) void mfma_probe_kernel(const v4i *operands, int *out, int iters,
                                                        unsigned long long *clk) {
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  v4i a[2], b[2];
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    a[i] = RANDOM ? operands[(i * 2 + 0) * 64 + lane] : v4i{0, 0, 0, 0};
    b[i] = RANDOM ? operands[(i * 2 + 1) * 64 + lane] : v4i{0, 0, 0, 0};
  }
  v16i acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0;
#pragma unroll 4
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t & 1], b[t >> 1], acc[t], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[t][r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clk[0] = clock64() - c0;
    clk[1] = wall_clock64() - w0;
  }
}

}  // namespace

}  // namespace quamba

using namespace quamba;

extern "C" size_t quamba_probe_workspace_bytes(int waves_per_simd) {
  if (waves_per_simd < 1 || waves_per_simd > 8) return 0;
  // 4 KiB of MFMA operands, 256 bytes for the two clock deltas, one word per thread of 256 CUs x 4 SIMDs x waves
  return 4096 + 256 + (size_t)1024 * waves_per_simd * 64 * 4;
}

extern "C" int quamba_probe_rate(int probe, int waves_per_simd, int iters, double *instr_per_call /* host */,
                                 void *ws, size_t ws_bytes, void *stream) {
  if (!ws || !instr_per_call) return fail(QUAMBA_EINVAL, "probe: NULL pointer");
  if (waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) return fail(QUAMBA_EINVAL, "probe: waves_per_simd=%d iters=%d", waves_per_simd, iters);
  if (!aligned(ws, 256) || ws_bytes < quamba_probe_workspace_bytes(waves_per_simd))
    return fail(QUAMBA_EWORKSPACE, "probe: workspace too small or not 256-byte aligned");
  hipStream_t st = as_stream(stream);
  const int blocks = 256 * waves_per_simd;  // 4 waves per block: one per SIMD of a CU
  unsigned long long *clk = reinterpret_cast<unsigned long long *>(static_cast<char *>(ws) + 4096);
  float *outf = reinterpret_cast<float *>(static_cast<char *>(ws) + 4096 + 256);
  const double waves = (double)blocks * 4;
  switch (probe) {
    case QUAMBA_PROBE_FMA_F32:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_FMA_F32>, dim3(blocks), dim3(256), 0, st, outf, iters, 1.25f, clk);
      *instr_per_call = waves * iters * REGS;
      break;
    case QUAMBA_PROBE_EXP_F32:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_EXP_F32>, dim3(blocks), dim3(256), 0, st, outf, iters, 0.5f, clk);
      *instr_per_call = waves * iters * REGS;
      break;
    case QUAMBA_PROBE_SCAN_MIX:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_SCAN_MIX>, dim3(blocks), dim3(256), 0, st, outf, iters, -0.5f, clk);
      *instr_per_call = waves * iters * REGS;  // state updates (5 instructions each)
      break;
    case QUAMBA_PROBE_MUL_F32:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_MUL_F32>, dim3(blocks), dim3(256), 0, st, outf, iters, 1.25f, clk);
      *instr_per_call = waves * iters * REGS;
      break;
    case QUAMBA_PROBE_FMA_EXP_INDEP:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_FMA_EXP_INDEP>, dim3(blocks), dim3(256), 0, st, outf, iters, 0.5f, clk);
      *instr_per_call = waves * iters * REGS;
      break;
    case QUAMBA_PROBE_MIX_NOEXP:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_MIX_NOEXP>, dim3(blocks), dim3(256), 0, st, outf, iters, -0.5f, clk);
      *instr_per_call = waves * iters * REGS;
      break;
    case QUAMBA_PROBE_MIX_GROUPED:
      hipLaunchKernelGGL(valu_probe_kernel<QUAMBA_PROBE_MIX_GROUPED>, dim3(blocks), dim3(256), 0, st, outf, iters, -0.5f, clk);
      *instr_per_call = waves * iters * REGS;
      break;
    case QUAMBA_PROBE_MFMA_I8:
      hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(blocks), dim3(256), 0, st, static_cast<const v4i *>(ws),
                         reinterpret_cast<int *>(outf), iters, clk);
      *instr_per_call = waves * iters * 4;
      break;
    case QUAMBA_PROBE_MFMA_I8_RANDOM:
      hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(blocks), dim3(256), 0, st, static_cast<const v4i *>(ws),
                         reinterpret_cast<int *>(outf), iters, clk);
      *instr_per_call = waves * iters * 4;
      break;
    default:
      return fail(QUAMBA_EINVAL, "probe: unknown probe %d", probe);
  }
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}
