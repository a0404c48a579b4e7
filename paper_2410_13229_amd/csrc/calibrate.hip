// Offline calibration (Section 5.1 "Quantization setup"; Section 4.2): an fp32 forward of the
// unquantized mixer over the calibration batch with absmax observers, the percentile maximum
// for the scan input x, the Hadamard-space scale of the scan output and the folding of H_n
// into W_out, followed by the per-tensor symmetric quantization of every weight (Eq. 2).
// This runs once per layer, so the kernels here are plain tiled fp32 code, not tuned.
#include <cmath>
#include <cstring>
#include <vector>

#include "common.h"

namespace quamba {

// defined in hadamard.hip: fp32 rows in, fp32 rows out (no quantization)
int launch_hadamard_f32(const float *x, int M, int n, float *y, hipStream_t st);

namespace {

constexpr float LOG2E = 1.44269504088896340736f;

// ---------------------------------------------------------------- fp32 GEMM, C = A W^T
constexpr int GT = 64, GK = 16;
__global__ __launch_bounds__(256) void sgemm_tn_kernel(const float *__restrict__ A, int lda,
                                                       const float *__restrict__ W, int ldw,
                                                       float *__restrict__ C, int ldc, int M, int N, int K) {
  __shared__ float sa[GK][GT + 4], sw[GK][GT + 4];
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += GK) {
    for (int i = threadIdx.x; i < GT * GK; i += 256) {
      const int r = i / GK, k = i % GK;
      sa[k][r] = (m0 + r < M && k0 + k < K) ? A[(size_t)(m0 + r) * lda + k0 + k] : 0.f;
      sw[k][r] = (n0 + r < N && k0 + k < K) ? W[(size_t)(n0 + r) * ldw + k0 + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < GK; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = sa[k][ty * 4 + i];
        w[i] = sw[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * w[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) C[(size_t)m * ldc + n] = acc[i][j];
    }
}

int sgemm(const float *A, int lda, const float *W, int ldw, float *C, int ldc, int M, int N, int K,
          hipStream_t st) {
  dim3 grid((N + GT - 1) / GT, (M + GT - 1) / GT);
  hipLaunchKernelGGL(sgemm_tn_kernel, grid, dim3(256), 0, st, A, lda, W, ldw, C, ldc, M, N, K);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

// ---------------------------------------------------------------- small elementwise kernels
__global__ void half_to_float_kernel(const __half *x, float *y, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) y[i] = __half2float(x[i]);
}

__global__ void neg_exp_kernel(const float *a_log, float *a, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) a[i] = static_cast<float>(-exp(static_cast<double>(a_log[i])));  // once, offline: fp64
}

__global__ void fill_u32_kernel(unsigned *p, size_t n, unsigned v) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// max |x| over the column range [c0, c1) of a [rows, ld] matrix, as the bit pattern of a
// non-negative float (which orders like an unsigned integer) combined with atomicMax.
__global__ __launch_bounds__(256) void absmax_kernel(const float *__restrict__ x, size_t rows, int ld, int c0,
                                                     int c1, unsigned *slot) {
  const int w = c1 - c0;
  const size_t total = rows * (size_t)w;
  float m = 0.f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const size_t r = i / w;
    const int c = static_cast<int>(i % w);
    m = fmaxf(m, fabsf(x[r * ld + c0 + c]));
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((threadIdx.x & 63) == 0) atomicMax(slot, __float_as_uint(m));
}

int absmax(const float *x, size_t rows, int ld, int c0, int c1, unsigned *slot, hipStream_t st) {
  const size_t total = rows * (size_t)(c1 - c0);
  const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 2048);
  hipLaunchKernelGGL(absmax_kernel, dim3(blocks ? blocks : 1), dim3(256), 0, st, x, rows, ld, c0, c1, slot);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

// causal conv (width 4, zero history) + bias + SiLU in fp32; xz has row stride ld
__global__ void conv_silu_f32_kernel(const float *__restrict__ xz, int ld, const float *__restrict__ w,
                                     const float *__restrict__ b, int L, int Di, float *__restrict__ x,
                                     size_t total) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int d = static_cast<int>(i % Di);
  const size_t row = i / Di;
  const int t = static_cast<int>(row % L);
  float v = b[d];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tj = t - 3 + j;
    if (tj >= 0) v += w[d * 4 + j] * xz[(row - 3 + j) * ld + d];
  }
  x[i] = v / (1.f + expf(-v));
}

// sequential fp32 selective scan + gate, one thread per (sequence, channel)
__global__ void scan_f32_kernel(const float *__restrict__ x, const float *__restrict__ dt_raw,
                                const float *__restrict__ dt_bias, const float *__restrict__ A,
                                const float *__restrict__ dbc, int nx, int R, const float *__restrict__ D,
                                const float *__restrict__ xz, int Bt, int L, int Di, float *__restrict__ g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)Bt * Di) return;
  const int d = static_cast<int>(i % Di), b = static_cast<int>(i / Di);
  float a2[16], h[16];
#pragma unroll
  for (int n = 0; n < 16; ++n) {
    a2[n] = A[(size_t)d * 16 + n] * LOG2E;
    h[n] = 0.f;
  }
  const float bias = dt_bias[d], Dv = D[d];
  for (int t = 0; t < L; ++t) {
    const size_t row = (size_t)b * L + t;
    const float xv = x[row * Di + d];
    const float pre = dt_raw[row * Di + d] + bias;
    const float dt = pre > 20.f ? pre : log1pf(expf(pre));
    const float zv = xz[row * (2 * (size_t)Di) + Di + d];
    const float *B = dbc + row * nx + R, *C = B + 16;
    float y = 0.f;
#pragma unroll
    for (int n = 0; n < 16; ++n) {
      h[n] = exp2f(dt * a2[n]) * h[n] + dt * xv * B[n];
      y += C[n] * h[n];
    }
    y += Dv * xv;
    g[row * Di + d] = y * zv / (1.f + expf(-zv));
  }
}

// radix-select histogram: count byte `shift/8` of |x| bit patterns whose higher bits equal prefix
__global__ void select_hist_kernel(const float *__restrict__ x, size_t n, unsigned prefix, unsigned mask,
                                   int shift, unsigned long long *hist) {
  __shared__ unsigned local[256];
  local[threadIdx.x] = 0;
  __syncthreads();
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const unsigned bits = __float_as_uint(fabsf(x[i]));
    if ((bits & mask) == prefix) atomicAdd(&local[(bits >> shift) & 255u], 1u);
  }
  __syncthreads();
  if (local[threadIdx.x]) atomicAdd(&hist[threadIdx.x], (unsigned long long)local[threadIdx.x]);
}

// ---------------------------------------------------------------- model-optimal clipping scalar
// Section 5.1 names a clipping optimisation as the enhanced variant; the rule is the stationary
// point of (4^-bits / 3) s^2 #{0 < |x| <= s} + sum_{|x| > s} (|x| - s)^2, iterated as
//   s <- sum(|x| : |x| > s) / (4^-bits / 3 * #{0 < |x| <= s} + #{|x| > s}).
// One pass gathers the three sums per workgroup, a one-workgroup pass adds them in a fixed order
// (same result on every run) and moves s.  state[0] = s, state[1] = updates made, state[2] = done.
struct ClipPart {
  double sum_out;
  unsigned long long n_out, n_in;
};
constexpr int CLIP_BLOCKS = 1024;

__global__ __launch_bounds__(256) void clip_stats_kernel(const float *__restrict__ x, size_t n,
                                                         const double *__restrict__ state, ClipPart *parts) {
  const double s = state[0];
  double sum = 0.0;
  unsigned long long n_out = 0, n_in = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const double a = static_cast<double>(fabsf(x[i]));
    if (a > s) {
      sum += a;
      ++n_out;
    } else if (a > 0.0) {
      ++n_in;
    }
  }
  __shared__ ClipPart part[256];
  part[threadIdx.x] = ClipPart{sum, n_out, n_in};
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      part[threadIdx.x].sum_out += part[threadIdx.x + off].sum_out;
      part[threadIdx.x].n_out += part[threadIdx.x + off].n_out;
      part[threadIdx.x].n_in += part[threadIdx.x + off].n_in;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) parts[blockIdx.x] = part[0];
}

__global__ __launch_bounds__(256) void clip_update_kernel(const ClipPart *__restrict__ parts, int nparts, double c,
                                                          int first, double *state) {
  __shared__ ClipPart part[256];
  ClipPart acc{0.0, 0, 0};
  for (int i = threadIdx.x; i < nparts; i += 256) {
    acc.sum_out += parts[i].sum_out;
    acc.n_out += parts[i].n_out;
    acc.n_in += parts[i].n_in;
  }
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      part[threadIdx.x].sum_out += part[threadIdx.x + off].sum_out;
      part[threadIdx.x].n_out += part[threadIdx.x + off].n_out;
      part[threadIdx.x].n_in += part[threadIdx.x + off].n_in;
    }
    __syncthreads();
  }
  if (threadIdx.x != 0 || state[2] != 0.0) return;
  const ClipPart t = part[0];
  if (first) {  // the start value: every element counts as outside, which makes the quotient mean |x|
    state[0] = t.n_out ? t.sum_out / static_cast<double>(t.n_out) : 0.0;
    return;
  }
  if (t.n_out == 0) {
    state[2] = 1.0;
    return;
  }
  const double nxt = t.sum_out / (c * static_cast<double>(t.n_in) + static_cast<double>(t.n_out));
  if (nxt == state[0]) {
    state[2] = 1.0;
    return;
  }
  state[0] = nxt;
  state[1] += 1.0;
}

__global__ void clip_init_kernel(double *state) {
  if (threadIdx.x == 0) {
    state[0] = -1.0;  // below every |x|
    state[1] = 0.0;
    state[2] = 0.0;
  }
}

constexpr size_t CLIP_WS_BYTES = 256 + CLIP_BLOCKS * sizeof(ClipPart);

__global__ void quantize_f32_kernel(const float *__restrict__ x, int8_t *__restrict__ q, size_t n, float inv_s) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float v = __builtin_rintf(x[i] * inv_s);
  v = fminf(fmaxf(v, -128.f), 127.f);
  q[i] = static_cast<int8_t>(static_cast<int>(v));
}

__global__ void copy_f32_kernel(const float *x, float *y, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) y[i] = x[i];
}

// max(0, -min x) over x[0, n), as the bit pattern of a non-negative float
__global__ __launch_bounds__(256) void negmax_kernel(const float *__restrict__ x, size_t n, unsigned *slot) {
  float m = 0.f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) m = fmaxf(m, -x[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((threadIdx.x & 63) == 0) atomicMax(slot, __float_as_uint(m));
}

// out[r] = factor * sum_k w[r, k] (int32; |sum| <= 128 K): one workgroup per row
__global__ __launch_bounds__(256) void scaled_rowsum_i8_kernel(const int8_t *__restrict__ w, int K, int factor,
                                                               int32_t *__restrict__ out) {
  int acc = 0;
  for (int k = threadIdx.x; k < K; k += 256) acc += w[(size_t)blockIdx.x * K + k];
  __shared__ int part[4];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) out[blockIdx.x] = factor * (part[0] + part[1] + part[2] + part[3]);
}

inline unsigned nblk(size_t n) { return (unsigned)((n + 255) / 256); }

struct CalPlan {
  size_t u32, xz, x, dbc, dtr, g, gH, woh, a, slots, hist, clip, total;
};

CalPlan cal_plan(const quamba_dims *d, int nb, int Lc) {
  const size_t M = (size_t)nb * Lc, Di = d->d_inner, Dm = d->d_model, NX = d->dt_rank + 2 * d->d_state;
  CalPlan p{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += align_up(bytes, 256);
    return at;
  };
  p.u32 = take(M * Dm * 4);
  p.xz = take(M * 2 * Di * 4);
  p.x = take(M * Di * 4);
  p.dbc = take(M * NX * 4);
  p.dtr = take(M * Di * 4);
  p.g = take(M * Di * 4);
  p.gH = take(M * Di * 4);
  p.woh = take(Dm * Di * 4);
  p.a = take(Di * d->d_state * 4);
  p.slots = take(32 * 4);
  p.hist = take(256 * 8);
  p.clip = take(CLIP_WS_BYTES);
  p.total = off;
  return p;
}

enum Slot { S_U, S_XPRE, S_Z, S_DTL, S_B, S_C, S_DT, S_Y, S_WIN, S_CW, S_WX, S_WDT, S_A, S_D, S_WOH, S_COUNT };

struct CalBufs {
  float *u32, *xz, *x, *dbc, *dtr, *g, *gH, *woh, *A;
  unsigned *slots;
  unsigned long long *hist;
};

CalBufs carve(const CalPlan &p, void *ws) {
  char *base = static_cast<char *>(ws);
  auto f = [&](size_t off) { return reinterpret_cast<float *>(base + off); };
  return CalBufs{f(p.u32), f(p.xz), f(p.x), f(p.dbc), f(p.dtr), f(p.g), f(p.gH), f(p.woh), f(p.a),
                 reinterpret_cast<unsigned *>(base + p.slots), reinterpret_cast<unsigned long long *>(base + p.hist)};
}

// The unquantized mixer up to the gated scan output (Section 3.1), fp32: leaves x_pre | z, x,
// dt_low | B | C, dt_raw and g in the workspace.  calib_u == nullptr: the input is already in b.u32.
int fp_forward(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
               const CalBufs &b, hipStream_t st) {
  const int Dm = d->d_model, Di = d->d_inner, N = d->d_state, R = d->dt_rank, NX = R + 2 * N;
  const size_t M = (size_t)nb * Lc;
  if (calib_u) hipLaunchKernelGGL(half_to_float_kernel, dim3(nblk(M * Dm)), dim3(256), 0, st, calib_u, b.u32, M * Dm);
  hipLaunchKernelGGL(neg_exp_kernel, dim3(nblk((size_t)Di * N)), dim3(256), 0, st, w->A_log, b.A, (size_t)Di * N);
  QUAMBA_LAUNCH_CHECK();
  int rc;
  if ((rc = sgemm(b.u32, Dm, w->W_in, Dm, b.xz, 2 * Di, (int)M, 2 * Di, Dm, st))) return rc;
  hipLaunchKernelGGL(conv_silu_f32_kernel, dim3(nblk(M * Di)), dim3(256), 0, st, b.xz, 2 * Di, w->conv_w,
                     w->conv_b, Lc, Di, b.x, M * Di);
  QUAMBA_LAUNCH_CHECK();
  if ((rc = sgemm(b.x, Di, w->W_x, Di, b.dbc, NX, (int)M, NX, Di, st))) return rc;
  if ((rc = sgemm(b.dbc, NX, w->W_dt, R, b.dtr, Di, (int)M, Di, R, st))) return rc;
  hipLaunchKernelGGL(scan_f32_kernel, dim3(nblk((size_t)nb * Di)), dim3(256), 0, st, b.x, b.dtr, w->dt_bias, b.A,
                     b.dbc, NX, R, w->D, b.xz, nb, Lc, Di, b.g);
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

}  // namespace

size_t calibrate_workspace_bytes(const quamba_dims *d, int nb, int Lc) { return cal_plan(d, nb, Lc).total; }

size_t clip_search_workspace_bytes() { return CLIP_WS_BYTES; }

// Runs the fixed-point iteration above on x[0, n) and returns the scalar and the number of updates
// on the host (synchronises the stream).
int clip_search(const float *x, size_t n, int bits, int max_iters, double *clip_out, int *iters_out, void *ws,
                size_t ws_bytes, hipStream_t st) {
  if (ws_bytes < CLIP_WS_BYTES) return fail(QUAMBA_EWORKSPACE, "clip_search: workspace %zu < %zu", ws_bytes, CLIP_WS_BYTES);
  double *state = static_cast<double *>(ws);
  ClipPart *parts = reinterpret_cast<ClipPart *>(static_cast<char *>(ws) + 256);
  const double c = std::pow(4.0, -static_cast<double>(bits)) / 3.0;
  const int blocks = (int)std::min<size_t>(std::max<size_t>((n + 255) / 256, 1), CLIP_BLOCKS);
  hipLaunchKernelGGL(clip_init_kernel, dim3(1), dim3(64), 0, st, state);
  for (int it = 0; it <= max_iters; ++it) {  // pass 0 produces the start value
    hipLaunchKernelGGL(clip_stats_kernel, dim3(blocks), dim3(256), 0, st, x, n, state, parts);
    hipLaunchKernelGGL(clip_update_kernel, dim3(1), dim3(256), 0, st, parts, blocks, c, it == 0 ? 1 : 0, state);
    QUAMBA_LAUNCH_CHECK();
  }
  double h[3];
  QUAMBA_HIP(hipMemcpyAsync(h, state, sizeof(h), hipMemcpyDeviceToHost, st));
  QUAMBA_HIP(hipStreamSynchronize(st));
  *clip_out = h[0];
  if (iters_out) *iters_out = static_cast<int>(h[1]);
  return QUAMBA_OK;
}

// The unquantized mixer of Section 3.1 in fp32 on u [nb, Lc, Dm] (fp16), each sequence from an
// empty history: out [nb * Lc, Dm] fp32.  The reference the quantized path is compared with.
int fp_mixer(const quamba_dims *d, const quamba_fp_weights *w, const __half *u, int nb, int Lc, float *out,
             void *ws, size_t ws_bytes, hipStream_t st) {
  const CalPlan p = cal_plan(d, nb, Lc);
  if (ws_bytes < p.total) return fail(QUAMBA_EWORKSPACE, "fp mixer: workspace %zu < %zu", ws_bytes, p.total);
  const CalBufs b = carve(p, ws);
  int rc;
  if ((rc = fp_forward(d, w, u, nb, Lc, b, st))) return rc;
  return sgemm(b.g, d->d_inner, w->W_out, d->d_inner, out, d->d_model, nb * Lc, d->d_model, d->d_inner, st);
}

int calibrate(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
              int x_rule, double x_percentile, quamba_qweights *oq, quamba_scales *os, void *ws, size_t ws_bytes,
              hipStream_t st, float *out_f32, float *x_clip_out = nullptr);

namespace {
// res[row] += out[row]; u[row] = res[row] / sqrt(mean(res[row]^2) + eps) * w   (fp32; one workgroup per row)
__global__ __launch_bounds__(256) void add_rmsnorm_f32_kernel(float *__restrict__ res, const float *__restrict__ out,
                                                              const __half *__restrict__ w, float eps, int Dm,
                                                              float *__restrict__ u) {
  const size_t row = blockIdx.x;
  float ss = 0.f;
  for (int i = threadIdx.x; i < Dm; i += 256) {
    const float r = res[row * Dm + i] + out[row * Dm + i];
    res[row * Dm + i] = r;
    ss += r * r;
  }
  __shared__ float part[4];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float rinv = 1.f / sqrtf((part[0] + part[1] + part[2] + part[3]) / static_cast<float>(Dm) + eps);
  for (int i = threadIdx.x; i < Dm; i += 256) u[row * Dm + i] = res[row * Dm + i] * rinv * __half2float(w[i]);
}
}  // namespace

// One block of a stack (Section 5.1: every layer gets its own static scales): the block input is
// the RMSNorm of the unquantized residual stream, which the call advances.
int calibrate_block(const quamba_dims *d, const quamba_fp_weights *w, const __half *norm_w, float eps, float *res,
                    float *out, int nb, int Lc, double x_percentile, quamba_qweights *oq, quamba_scales *os, void *ws,
                    size_t ws_bytes, hipStream_t st) {
  const CalPlan p = cal_plan(d, nb, Lc);
  if (ws_bytes < p.total) return fail(QUAMBA_EWORKSPACE, "calibrate: workspace %zu < %zu", ws_bytes, p.total);
  float *u32 = reinterpret_cast<float *>(static_cast<char *>(ws) + p.u32);
  hipLaunchKernelGGL(add_rmsnorm_f32_kernel, dim3((unsigned)((size_t)nb * Lc)), dim3(256), 0, st, res, out, norm_w, eps,
                     d->d_model, u32);
  QUAMBA_LAUNCH_CHECK();
  return calibrate(d, w, nullptr, nb, Lc, QUAMBA_X_PERCENTILE, x_percentile, oq, os, ws, ws_bytes, st, out);
}

// calib_u == nullptr: the fp32 block input is already in the workspace's own input buffer
// (calibrate_block puts it there).  out_f32 != nullptr: also receives the unquantized block output
// g W_out^T, which feeds the next block of a stack.
int calibrate(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
              int x_rule, double x_percentile, quamba_qweights *oq, quamba_scales *os, void *ws, size_t ws_bytes,
              hipStream_t st, float *out_f32, float *x_clip_out) {
  const CalPlan p = cal_plan(d, nb, Lc);
  if (ws_bytes < p.total) return fail(QUAMBA_EWORKSPACE, "calibrate: workspace %zu < %zu", ws_bytes, p.total);
  const int Dm = d->d_model, Di = d->d_inner, N = d->d_state, R = d->dt_rank, NX = R + 2 * N;
  const size_t M = (size_t)nb * Lc;
  char *base = static_cast<char *>(ws);
  const CalBufs b = carve(p, ws);
  float *u32 = b.u32, *xz = b.xz, *x = b.x, *dbc = b.dbc, *dtr = b.dtr, *g = b.g, *gH = b.gH, *woh = b.woh, *A = b.A;
  unsigned *slots = b.slots;
  unsigned long long *hist = b.hist;

  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, slots, (size_t)32, 0u);
  QUAMBA_LAUNCH_CHECK();
  int rc;
  if ((rc = fp_forward(d, w, calib_u, nb, Lc, b, st))) return rc;
  if ((rc = launch_hadamard_f32(g, (int)M, Di, gH, st))) return rc;      // y^H = H_n g
  if ((rc = launch_hadamard_f32(w->W_out, Dm, Di, woh, st))) return rc;  // rows of W_out^H
  if (out_f32 && (rc = sgemm(g, Di, w->W_out, Di, out_f32, Dm, (int)M, Dm, Di, st))) return rc;

  // observers
  struct Obs { const float *p; size_t rows; int ld, c0, c1, slot; };
  const Obs obs[] = {
      {u32, M, Dm, 0, Dm, S_U},         {xz, M, 2 * Di, 0, Di, S_XPRE},    {xz, M, 2 * Di, Di, 2 * Di, S_Z},
      {dbc, M, NX, 0, R, S_DTL},        {dbc, M, NX, R, R + N, S_B},       {dbc, M, NX, R + N, NX, S_C},
      {dtr, M, Di, 0, Di, S_DT},        {gH, M, Di, 0, Di, S_Y},           {w->W_in, (size_t)2 * Di, Dm, 0, Dm, S_WIN},
      {w->conv_w, (size_t)Di, 4, 0, 4, S_CW}, {w->W_x, (size_t)NX, Di, 0, Di, S_WX},
      {w->W_dt, (size_t)Di, R, 0, R, S_WDT},  {A, (size_t)Di, N, 0, N, S_A},   {w->D, 1, Di, 0, Di, S_D},
      {woh, (size_t)Dm, Di, 0, Di, S_WOH}};
  for (const Obs &o : obs)
    if ((rc = absmax(o.p, o.rows, o.ld, o.c0, o.c1, slots + o.slot, st))) return rc;

  float mx[S_COUNT];
  QUAMBA_HIP(hipMemcpyAsync(mx, slots, sizeof(mx), hipMemcpyDeviceToHost, st));
  QUAMBA_HIP(hipStreamSynchronize(st));

  const size_t nx = M * Di;
  float xp;
  if (x_rule == QUAMBA_X_MSE_CLIP) {
    double clip;
    if ((rc = clip_search(x, nx, 8, 32, &clip, nullptr, base + p.clip, CLIP_WS_BYTES, st))) return rc;
    xp = static_cast<float>(clip);
  } else {
  // percentile maximum of |x| (Section 4.2): value of 1-based rank ceil(p/100 * n), found by a
  // most-significant-byte-first radix select on the bit patterns
  size_t rank = (size_t)std::ceil(x_percentile * (double)nx / 100.0);
  if (rank < 1) rank = 1;
  if (rank > nx) rank = nx;
  unsigned prefix = 0, mask = 0;
  size_t below = 0;  // elements known to be smaller than every candidate
  for (int shift = 24; shift >= 0; shift -= 8) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(2), dim3(256), 0, st, reinterpret_cast<unsigned *>(hist),
                       (size_t)512, 0u);
    hipLaunchKernelGGL(select_hist_kernel, dim3(1024), dim3(256), 0, st, x, nx, prefix, mask, shift, hist);
    QUAMBA_LAUNCH_CHECK();
    unsigned long long h[256];
    QUAMBA_HIP(hipMemcpyAsync(h, hist, sizeof(h), hipMemcpyDeviceToHost, st));
    QUAMBA_HIP(hipStreamSynchronize(st));
    int byte = 255;
    for (int v = 0; v < 256; ++v) {
      if (below + h[v] >= rank) {
        byte = v;
        break;
      }
      below += h[v];
    }
    prefix |= (unsigned)byte << shift;
    mask |= 0xffu << shift;
  }
  std::memcpy(&xp, &prefix, 4);
  }

  if (x_clip_out) *x_clip_out = xp;  // the clipping value of x before it becomes a scale
  auto sc_of = [](float m) { return m > 0.f ? (float)((double)m / 127.0) : 1.0f; };
  quamba_scales s{};
  s.s_u = sc_of(mx[S_U]); s.s_xpre = sc_of(mx[S_XPRE]); s.s_z = sc_of(mx[S_Z]); s.s_x = sc_of(xp);
  s.s_dtl = sc_of(mx[S_DTL]); s.s_B = sc_of(mx[S_B]); s.s_C = sc_of(mx[S_C]); s.s_dt = sc_of(mx[S_DT]);
  s.s_y = sc_of(mx[S_Y]); s.s_Win = sc_of(mx[S_WIN]); s.s_cw = sc_of(mx[S_CW]); s.s_Wx = sc_of(mx[S_WX]);
  s.s_Wdt = sc_of(mx[S_WDT]); s.s_A = sc_of(mx[S_A]); s.s_D = sc_of(mx[S_D]); s.s_WoutH = sc_of(mx[S_WOH]);
  const double du = s.s_u, dxp = s.s_xpre, dz = s.s_z, dx = s.s_x, ddtl = s.s_dtl, dB = s.s_B, dC = s.s_C,
               ddt = s.s_dt, dy = s.s_y, dWin = s.s_Win, dcw = s.s_cw, dWx = s.s_Wx, dWdt = s.s_Wdt,
               dWoh = s.s_WoutH;
  s.inv_s_u = (float)(1.0 / du);
  s.m_in_x = (float)(du * dWin / dxp);
  s.m_in_z = (float)(du * dWin / dz);
  s.m_conv = (float)(dcw * dxp);
  s.inv_s_x = (float)(1.0 / dx);
  s.m_x_dt = (float)(dx * dWx / ddtl);
  s.m_x_B = (float)(dx * dWx / dB);
  s.m_x_C = (float)(dx * dWx / dC);
  s.m_dt = (float)(ddtl * dWdt / ddt);
  s.inv_s_y = (float)(1.0 / dy);
  s.m_out = (float)(dy * dWoh / (double)Di);
  *os = s;

  // quantize the weights (Eq. 2) and copy the two fp32 bias vectors
  struct QW { const float *src; int8_t *dst; size_t n; float sc; };
  const QW qws[] = {{w->W_in, oq->W_in, (size_t)2 * Di * Dm, s.s_Win}, {w->conv_w, oq->conv_w, (size_t)Di * 4, s.s_cw},
                    {w->W_x, oq->W_x, (size_t)NX * Di, s.s_Wx},        {w->W_dt, oq->W_dt, (size_t)Di * R, s.s_Wdt},
                    {A, oq->A, (size_t)Di * N, s.s_A},                 {w->D, oq->D, (size_t)Di, s.s_D},
                    {woh, oq->W_outH, (size_t)Dm * Di, s.s_WoutH}};
  for (const QW &q : qws) {
    hipLaunchKernelGGL(quantize_f32_kernel, dim3(nblk(q.n)), dim3(256), 0, st, q.src, q.dst, q.n,
                       (float)(1.0 / (double)q.sc));
    QUAMBA_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(copy_f32_kernel, dim3(nblk(Di)), dim3(256), 0, st, w->conv_b, oq->conv_b, (size_t)Di);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(nblk(Di)), dim3(256), 0, st, w->dt_bias, oq->dt_bias, (size_t)Di);
  QUAMBA_LAUNCH_CHECK();
  QUAMBA_HIP(hipStreamSynchronize(st));
  return QUAMBA_OK;
}

// Calibration of the Appendix H comparison variant: Quamba's calibration, then the scale of H_n x
// (absmax over the calibration batch) and the x_proj weight with every row transformed by the same
// H_n, quantized per tensor; (H w) . (H x) = n (w . x) puts 1/n into the multipliers.
int calibrate_hadx(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
                   double x_percentile, quamba_qweights *oq, quamba_scales *os, quamba_hadx *oh, void *ws,
                   size_t ws_bytes, hipStream_t st) {
  int rc;
  if ((rc = calibrate(d, w, calib_u, nb, Lc, QUAMBA_X_PERCENTILE, x_percentile, oq, os, ws, ws_bytes, st, nullptr)))
    return rc;
  const CalPlan p = cal_plan(d, nb, Lc);
  const CalBufs b = carve(p, ws);
  const int Di = d->d_inner, Dm = d->d_model, NX = d->dt_rank + 2 * d->d_state;
  const size_t M = (size_t)nb * Lc;
  if (NX > Dm) return fail(QUAMBA_EUNSUPPORTED, "calibrate: dt_rank + 2 d_state = %d exceeds d_model = %d", NX, Dm);
  // the forward pass left x in the workspace; gH and woh are free again
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, b.slots, (size_t)32, 0u);
  QUAMBA_LAUNCH_CHECK();
  if ((rc = launch_hadamard_f32(b.x, (int)M, Di, b.gH, st))) return rc;
  if ((rc = launch_hadamard_f32(w->W_x, NX, Di, b.woh, st))) return rc;
  if ((rc = absmax(b.gH, M, Di, 0, Di, b.slots + 0, st))) return rc;
  if ((rc = absmax(b.woh, (size_t)NX, Di, 0, Di, b.slots + 1, st))) return rc;
  float mx[2];
  QUAMBA_HIP(hipMemcpyAsync(mx, b.slots, sizeof(mx), hipMemcpyDeviceToHost, st));
  QUAMBA_HIP(hipStreamSynchronize(st));
  auto sc_of = [](float m) { return m > 0.f ? (float)((double)m / 127.0) : 1.0f; };
  oh->s_xH = sc_of(mx[0]);
  oh->s_WxH = sc_of(mx[1]);
  const double a = oh->s_xH, c = oh->s_WxH;
  oh->inv_s_xH = (float)(1.0 / a);
  oh->m_xh_dt = (float)(a * c / ((double)Di * (double)os->s_dtl));
  oh->m_xh_B = (float)(a * c / ((double)Di * (double)os->s_B));
  oh->m_xh_C = (float)(a * c / ((double)Di * (double)os->s_C));
  oh->xhat_scale = (float)(a / (double)Di);
  const size_t nw = (size_t)NX * Di;
  hipLaunchKernelGGL(quantize_f32_kernel, dim3(nblk(nw)), dim3(256), 0, st, b.woh, oh->W_xH, nw, (float)(1.0 / c));
  QUAMBA_LAUNCH_CHECK();
  QUAMBA_HIP(hipStreamSynchronize(st));
  return QUAMBA_OK;
}

// Calibration with an asymmetric grid for the scan input (Appendix K): Quamba's calibration, then
// lo = min(min x, 0), hi = the percentile maximum, s = (hi - lo) / 255, zero point
// clamp(rne(-128 - lo / s)), and the x_proj column term -zp * rowsum(W_x_q).
int calibrate_xasym(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
                    double x_percentile, quamba_qweights *oq, quamba_scales *os, quamba_xasym *oa, void *ws,
                    size_t ws_bytes, hipStream_t st) {
  int rc;
  float hi = 0.f;
  if ((rc = calibrate(d, w, calib_u, nb, Lc, QUAMBA_X_PERCENTILE, x_percentile, oq, os, ws, ws_bytes, st, nullptr, &hi)))
    return rc;
  const CalPlan p = cal_plan(d, nb, Lc);
  const CalBufs b = carve(p, ws);
  const int Di = d->d_inner, NX = d->dt_rank + 2 * d->d_state;
  const size_t nx = (size_t)nb * Lc * Di;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, b.slots, (size_t)32, 0u);
  hipLaunchKernelGGL(negmax_kernel, dim3((unsigned)std::min<size_t>((nx + 255) / 256, 2048)), dim3(256), 0, st, b.x, nx,
                     b.slots);
  QUAMBA_LAUNCH_CHECK();
  float neg;
  QUAMBA_HIP(hipMemcpyAsync(&neg, b.slots, sizeof(neg), hipMemcpyDeviceToHost, st));
  QUAMBA_HIP(hipStreamSynchronize(st));
  const double lo = -(double)neg, span = (double)hi - lo;
  const float s = span > 0.0 ? (float)(span / 255.0) : 1.0f;
  int zp = (int)std::nearbyint(-128.0 - lo / (double)s);
  zp = std::min(127, std::max(-128, zp));
  oa->s_x = s;
  oa->inv_s_x = (float)(1.0 / (double)s);
  oa->zero_point = zp;
  oa->m_x_dt = (float)((double)s * (double)os->s_Wx / (double)os->s_dtl);
  oa->m_x_B = (float)((double)s * (double)os->s_Wx / (double)os->s_B);
  oa->m_x_C = (float)((double)s * (double)os->s_Wx / (double)os->s_C);
  hipLaunchKernelGGL(scaled_rowsum_i8_kernel, dim3(NX), dim3(256), 0, st, oq->W_x, Di, -zp, oa->col_bias);
  QUAMBA_LAUNCH_CHECK();
  QUAMBA_HIP(hipStreamSynchronize(st));
  return QUAMBA_OK;
}

// Calibration with a non-uniform 8-bit format for the scan input (Appendix K): Quamba's calibration,
// then the format's scale (log2: the maximum of |x| over the batch; E4M3: the percentile maximum
// over 448), the multipliers with it, and the int8 codes of W_x as bfloat16 for the matrix units.
int calibrate_xfmt(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc, int format,
                   double x_percentile, quamba_qweights *oq, quamba_scales *os, quamba_xfmt *of, void *ws,
                   size_t ws_bytes, hipStream_t st) {
  int rc;
  float hi = 0.f;
  if ((rc = calibrate(d, w, calib_u, nb, Lc, QUAMBA_X_PERCENTILE, x_percentile, oq, os, ws, ws_bytes, st, nullptr, &hi)))
    return rc;
  const CalPlan p = cal_plan(d, nb, Lc);
  const CalBufs b = carve(p, ws);
  const int Di = d->d_inner, NX = d->dt_rank + 2 * d->d_state;
  float s;
  if (format == QUAMBA_XFMT_E4M3) {
    s = hi > 0.f ? (float)((double)hi / 448.0) : 1.0f;
  } else {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, b.slots, (size_t)32, 0u);
    QUAMBA_LAUNCH_CHECK();
    if ((rc = absmax(b.x, (size_t)nb * Lc, Di, 0, Di, b.slots + 0, st))) return rc;
    float mx;
    QUAMBA_HIP(hipMemcpyAsync(&mx, b.slots, sizeof(mx), hipMemcpyDeviceToHost, st));
    QUAMBA_HIP(hipStreamSynchronize(st));
    s = mx > 0.f ? mx : 1.0f;
  }
  of->format = format;
  of->s_x = s;
  of->inv_s_x = (float)(1.0 / (double)s);
  of->m_x_dt = (float)((double)s * (double)os->s_Wx / (double)os->s_dtl);
  of->m_x_B = (float)((double)s * (double)os->s_Wx / (double)os->s_B);
  of->m_x_C = (float)((double)s * (double)os->s_Wx / (double)os->s_C);
  if ((rc = launch_i8_to_bf16(oq->W_x, NX, Di, of->W_x_bf16, st))) return rc;
  QUAMBA_HIP(hipStreamSynchronize(st));
  return QUAMBA_OK;
}

}  // namespace quamba
