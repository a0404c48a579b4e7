// Whole-model shell around the stack of quantized blocks: what Section 5.2 times as time to first
// token, time per output token and time to last token is this loop.
//
//   res = E[token] (fp16), out = 0
//   block l: (u_q, res) = add_rmsnorm_quant(out, res; w_l, 1/s_u,l)   (Section 4.3 "Fused RMSNorm")
//            out = mixer_l(u_q)                                        (Sections 4.2, 4.3)
//   y = fp16(RMSNorm(out + res) * w_f),  logits = y E^T (fp32),  next = argmax logits
//
// The embedding and the head are one fp16 matrix (tied) and stay in half precision: the recipe
// quantizes the blocks.  Only the last position of every sequence reaches the head, so the head
// is a skinny product that streams E once: an fp16 MFMA kernel with fp32 accumulation.
// Generation keeps the current token, the step counter and the token log on the device, so one
// step is a fixed sequence of launches that can be replayed from a HIP graph.
#include "common.h"
#include "device_util.h"

namespace quamba {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------------ embedding
// res[m, :] = E[clamp(token[m]), :], out[m, :] = 0; 16 bytes per lane.
__global__ __launch_bounds__(256) void embed_kernel(const __half *__restrict__ E, const int32_t *__restrict__ tokens,
                                                    int M, int Dm, int vocab, __half *__restrict__ res,
                                                    __half *__restrict__ out) {
  const int per_row = Dm / 8;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)M * per_row) return;
  const int m = static_cast<int>(idx / per_row), g = static_cast<int>(idx % per_row);
  const int tok = min(max(tokens[m], 0), vocab - 1);
  reinterpret_cast<uint4 *>(res + (size_t)m * Dm)[g] = reinterpret_cast<const uint4 *>(E + (size_t)tok * Dm)[g];
  reinterpret_cast<uint4 *>(out + (size_t)m * Dm)[g] = make_uint4(0u, 0u, 0u, 0u);
}

// ------------------------------------------------------------------ final norm of the last positions
// y[b, :] = fp16(RMSNorm(fp16(out[row] + res[row])) * w) with row = b * L + L - 1.  One workgroup
// per sequence; the row stays in registers between the reduction and the scaling.
constexpr int FN_MAX_PER_THREAD = 4;  // groups of 8 halves per thread: Dm <= 8192

__global__ __launch_bounds__(256) void final_norm_kernel(const __half *__restrict__ out, const __half *__restrict__ res,
                                                         const __half *__restrict__ weight, float eps, int L, int Dm,
                                                         __half *__restrict__ y) {
  const size_t row = (size_t)blockIdx.x * L + (L - 1);
  const int ngroups = Dm / 8;
  float vals[FN_MAX_PER_THREAD][8];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < FN_MAX_PER_THREAD; ++i) {
    const int g = threadIdx.x + i * 256;
    if (g < ngroups) {
      union {
        uint4 u;
        __half h[8];
      } a, r;
      a.u = *reinterpret_cast<const uint4 *>(out + row * Dm + (size_t)g * 8);
      r.u = *reinterpret_cast<const uint4 *>(res + row * Dm + (size_t)g * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float f = __half2float(__float2half_rn(__half2float(a.h[e]) + __half2float(r.h[e])));
        vals[i][e] = f;
        ss += f * f;
      }
    }
  }
  __shared__ float part[4];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = part[0] + part[1] + part[2] + part[3];
  const float rinv = 1.f / sqrtf(tot / static_cast<float>(Dm) + eps);
#pragma unroll
  for (int i = 0; i < FN_MAX_PER_THREAD; ++i) {
    const int g = threadIdx.x + i * 256;
    if (g < ngroups) {
      union {
        uint4 u;
        __half h[8];
      } wv, o;
      wv.u = *reinterpret_cast<const uint4 *>(weight + (size_t)g * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) o.h[e] = __float2half_rn(vals[i][e] * rinv * __half2float(wv.h[e]));
      *reinterpret_cast<uint4 *>(y + (size_t)blockIdx.x * Dm + (size_t)g * 8) = o.u;
    }
  }
}

// ------------------------------------------------------------------ head: logits = y E^T
// 64 vocabulary rows x 64 tokens per workgroup (2 x 2 waves of 32 x 32), fp16 MFMA with fp32
// accumulation.  The vocabulary rows are the MFMA A operand, so a lane ends with four consecutive
// vocabulary entries of one token.  Slices of 64 halves go global -> registers -> a
// double-buffered, XOR-swizzled LDS tile; pieces past K, past the vocabulary or past the batch
// are zero.
__device__ __forceinline__ int swz128(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

// With `pmax` / `pidx` ([gridDim.x, Bt]) every workgroup also leaves, per token, the largest of its 64
// logits and that entry's index (lowest index among equals), so that the selection does not have to
// read the logits again.
__global__ __launch_bounds__(256) void head_kernel(const __half *__restrict__ y, const __half *__restrict__ E, int Bt,
                                                   int V, int K, float *__restrict__ logits,
                                                   float *__restrict__ pmax, int32_t *__restrict__ pidx) {
  constexpr int BKB = 128;  // bytes of K per slice
  __shared__ __attribute__((aligned(16))) int8_t lds[2][128 * BKB];  // rows 0..63 tokens, 64..127 vocabulary
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int v0 = blockIdx.x * 64, b0 = blockIdx.y * 64;
  const int Kb = K * 2;

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;

  v4i reg[4];
  auto fetch = [&](int k0) {  // k0 in bytes
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + i * 256;  // 1024 pieces of 16 bytes: 128 rows x 8
      const int row = c >> 3, gk = k0 + (c & 7) * 16;
      v4i v = {0, 0, 0, 0};
      if (gk < Kb) {
        if (row < 64) {
          if (b0 + row < Bt) v = *reinterpret_cast<const v4i *>(reinterpret_cast<const int8_t *>(y + (size_t)(b0 + row) * K) + gk);
        } else if (v0 + row - 64 < V) {
          v = *reinterpret_cast<const v4i *>(reinterpret_cast<const int8_t *>(E + (size_t)(v0 + row - 64) * K) + gk);
        }
      }
      reg[i] = v;
    }
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = tid + i * 256;
      const int row = c >> 3;
      // the swizzle phase follows the row inside its operand
      *reinterpret_cast<v4i *>(lds[buf] + (row < 64 ? 0 : 64 * BKB) + swz128(row & 63, c & 7)) = reg[i];
    }
  };
  const int nk = (Kb + BKB - 1) / BKB;
  fetch(0);
  park(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * BKB);
    const int8_t *la = lds[buf];            // tokens
    const int8_t *lw = lds[buf] + 64 * BKB;  // vocabulary rows
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int chunk = s * 2 + (lane >> 5);
      const h8 fa = *reinterpret_cast<const h8 *>(la + swz128(wm * 32 + (lane & 31), chunk));
      const h8 fw = *reinterpret_cast<const h8 *>(lw + swz128(wn * 32 + (lane & 31), chunk));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw, fa, acc, 0, 0, 0);
    }
    if (kt + 1 < nk) park(buf ^ 1);
    __syncthreads();
  }
  // register r: vocabulary entry v0 + wn*32 + 8 (r/4) + 4 (lane/32) + r%4, token b0 + wm*32 + lane%32
  const int b = b0 + wm * 32 + (lane & 31);
  if (logits && b < Bt) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int v = v0 + wn * 32 + 8 * g + 4 * (lane >> 5);
      float *dst = logits + (size_t)b * V + v;
      if ((V & 3) == 0) {
        if (v < V) *reinterpret_cast<float4 *>(dst) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (v + e < V) dst[e] = acc[4 * g + e];
      }
    }
  }
  if (pmax) {
    // per lane over its 16 entries (ascending index), then the other half-wave, then the other wn wave
    float best = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int v = v0 + wn * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (v < V && (acc[r] > best || (acc[r] == best && v < bi))) {
        best = acc[r];
        bi = v;
      }
    }
    const float ob = __shfl_xor(best, 32);
    const int oi = __shfl_xor(bi, 32);
    if (ob > best || (ob == best && oi < bi)) {
      best = ob;
      bi = oi;
    }
    __shared__ float sbest[2][64];
    __shared__ int sidx[2][64];
    if (lane < 32) {
      sbest[wn][wm * 32 + lane] = best;
      sidx[wn][wm * 32 + lane] = bi;
    }
    __syncthreads();
    if (tid < 64 && b0 + tid < Bt) {
      float x = sbest[0][tid];
      int xi = sidx[0][tid];
      if (sbest[1][tid] > x || (sbest[1][tid] == x && sidx[1][tid] < xi)) {
        x = sbest[1][tid];
        xi = sidx[1][tid];
      }
      pmax[(size_t)blockIdx.x * Bt + b0 + tid] = x;
      pidx[(size_t)blockIdx.x * Bt + b0 + tid] = xi;
    }
  }
}

// Selection from the head's per-workgroup partials [P, Bt]: one workgroup per token.
__global__ __launch_bounds__(256) void argmax_partials_kernel(const float *__restrict__ pmax,
                                                              const int32_t *__restrict__ pidx, int P, int Bt,
                                                              int32_t *__restrict__ next, int32_t *__restrict__ log,
                                                              const int32_t *__restrict__ step) {
  const int b = blockIdx.x;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int p = threadIdx.x; p < P; p += 256) {
    const float x = pmax[(size_t)p * Bt + b];
    const int xi = pidx[(size_t)p * Bt + b];
    if (x > best || (x == best && xi < bi)) {
      best = x;
      bi = xi;
    }
  }
  __shared__ float sb[256];
  __shared__ int si[256];
  sb[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      const float ob = sb[threadIdx.x + off];
      const int oi = si[threadIdx.x + off];
      if (ob > sb[threadIdx.x] || (ob == sb[threadIdx.x] && oi < si[threadIdx.x])) {
        sb[threadIdx.x] = ob;
        si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const int r = si[0] == 0x7fffffff ? 0 : si[0];  // a row of NaNs selects token 0
    next[b] = r;
    if (log) log[(size_t)(*step) * Bt + b] = r;
  }
}

// ------------------------------------------------------------------ greedy selection
// next[b] = index of the largest logit of row b, the lowest index among equal maxima.  With a
// log: also log[step * Bt + b], where step is read from device memory (bump_kernel advances it).
__global__ __launch_bounds__(256) void argmax_kernel(const float *__restrict__ logits, int V, int Bt,
                                                     int32_t *__restrict__ next, int32_t *__restrict__ log,
                                                     const int32_t *__restrict__ step) {
  const int b = blockIdx.x;
  const float *row = logits + (size_t)b * V;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int v = threadIdx.x; v < V; v += 256) {
    const float x = row[v];
    if (x > best || (x == best && v < bi)) {
      best = x;
      bi = v;
    }
  }
  __shared__ float sb[256];
  __shared__ int si[256];
  sb[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      const float ob = sb[threadIdx.x + off];
      const int oi = si[threadIdx.x + off];
      if (ob > sb[threadIdx.x] || (ob == sb[threadIdx.x] && oi < si[threadIdx.x])) {
        sb[threadIdx.x] = ob;
        si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const int r = si[0] == 0x7fffffff ? 0 : si[0];  // a row of NaNs selects token 0
    next[b] = r;
    if (log) log[(size_t)(*step) * Bt + b] = r;
  }
}

__global__ __launch_bounds__(256) void zero_kernel(uint4 *p, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void set_step_kernel(int32_t *step, int v) { *step = v; }
__global__ void bump_kernel(int32_t *step) { *step += 1; }

// ------------------------------------------------------------------ host side
struct Carve {
  size_t res, res2, out, u_q, y, pmax, pidx, cur, step, mixer, mixer_bytes, total;
};

Carve carve(const quamba_model *m, int Bt, int L) {
  const size_t M = (size_t)Bt * L, Dm = m->dims.d_model;
  Carve c{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += align_up(bytes, 256);
    return at;
  };
  c.res = take(M * Dm * sizeof(__half));
  c.res2 = take(L == 1 ? M * Dm * sizeof(__half) : 0);  // second residual buffer of the fused generation path
  c.out = take(M * Dm * sizeof(__half));
  c.u_q = take(M * Dm);
  c.y = take((size_t)Bt * Dm * sizeof(__half));
  c.pmax = take((size_t)((m->vocab + 63) / 64) * Bt * sizeof(float));
  c.pidx = take((size_t)((m->vocab + 63) / 64) * Bt * sizeof(int32_t));
  c.cur = take((size_t)Bt * sizeof(int32_t));
  c.step = take(sizeof(int32_t));
  c.mixer_bytes = mixer_workspace_bytes(&m->dims, Bt, L);
  c.mixer = take(c.mixer_bytes);
  c.total = off;
  return c;
}

int check_model(const quamba_model *m) {
  if (!m) return fail(QUAMBA_EINVAL, "model is NULL");
  int rc = check_model_dims(&m->dims);
  if (rc != QUAMBA_OK) return rc;
  if (m->n_layers < 1 || m->vocab < 1) return fail(QUAMBA_EINVAL, "model: n_layers=%d vocab=%d", m->n_layers, m->vocab);
  if (!m->embedding || !m->norm_f || !m->layers) return fail(QUAMBA_EINVAL, "model: NULL pointer");
  if (m->dims.d_model > 8 * 256 * FN_MAX_PER_THREAD)
    return fail(QUAMBA_EUNSUPPORTED, "model: d_model=%d > %d", m->dims.d_model, 8 * 256 * FN_MAX_PER_THREAD);
  if (!aligned(m->embedding, 16) || !aligned(m->norm_f, 16))
    return fail(QUAMBA_EINVAL, "model: embedding and norm_f must be 16-byte aligned");
  for (int l = 0; l < m->n_layers; ++l)
    if (!m->layers[l].norm_w || !aligned(m->layers[l].norm_w, 16))
      return fail(QUAMBA_EINVAL, "model: layer %d norm_w is NULL or not 16-byte aligned", l);
  return QUAMBA_OK;
}

// One pass of the whole model over tokens [Bt, L] (decode: L == 1 on carried states).
int run_model(const quamba_model *m, const int32_t *tokens, int Bt, int L, bool decode, float *logits_out,
              int32_t *next, int32_t *log, float *ssm_states, __half *conv_states, char *base, const Carve &c,
              hipStream_t st) {
  const int Dm = m->dims.d_model, Di = m->dims.d_inner, N = m->dims.d_state, M = Bt * L;
  __half *res = reinterpret_cast<__half *>(base + c.res);
  __half *out = reinterpret_cast<__half *>(base + c.out);
  int8_t *u_q = reinterpret_cast<int8_t *>(base + c.u_q);
  __half *y = reinterpret_cast<__half *>(base + c.y);
  float *logits = logits_out;  // the logits are written only when the caller wants them
  float *pmax = next ? reinterpret_cast<float *>(base + c.pmax) : nullptr;
  int32_t *pidx = next ? reinterpret_cast<int32_t *>(base + c.pidx) : nullptr;
  int32_t *step = reinterpret_cast<int32_t *>(base + c.step);

  const size_t pieces = (size_t)M * (Dm / 8);
  hipLaunchKernelGGL(embed_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<const __half *>(m->embedding), tokens, M,
                     Dm, m->vocab, res, out);
  QUAMBA_LAUNCH_CHECK();
  // generation with at most 4 sequences: the add + norm + quantization runs inside each block's first
  // kernel, which reads one residual buffer and writes the other
  const bool fused = decode && mixer_decode_norm_available(&m->dims, Bt);
  __half *res_other = reinterpret_cast<__half *>(base + c.res2);
  // generation with more sequences: where out_proj splits K over the grid, the next block's add + norm +
  // quantization adds up the partial sums (the last block's output is stored as usual for the final norm)
  OutPartial prev{false, 1, nullptr, 0.f};
  for (int l = 0; l < m->n_layers; ++l) {
    const quamba_layer &ly = m->layers[l];
    float *ssm = ssm_states + (size_t)l * Bt * Di * N;
    __half *cs = conv_states + (size_t)l * Bt * Di * 3;
    int rc;
    if (fused) {
      const NormIn norm{out, res, res_other, reinterpret_cast<const __half *>(ly.norm_w), m->eps};
      rc = mixer_decode_norm(&m->dims, &ly.q, &ly.s, norm, Bt, out, ssm, cs, base + c.mixer, c.mixer_bytes, st);
      __half *tmp = res;
      res = res_other;
      res_other = tmp;
    } else {
      if (prev.splits > 1)
        rc = launch_add_rmsnorm_quant_partial(prev.partial, prev.splits, prev.m_out, res,
                                              reinterpret_cast<const __half *>(ly.norm_w), m->eps, ly.s.inv_s_u, u_q, M,
                                              Dm, st);
      else
        rc = launch_add_rmsnorm_quant(out, res, reinterpret_cast<const __half *>(ly.norm_w), m->eps, ly.s.inv_s_u,
                                      u_q, M, Dm, st);
      if (rc != QUAMBA_OK) return rc;
      prev = OutPartial{decode && l + 1 < m->n_layers, 1, nullptr, 0.f};
      rc = mixer_run_q(&m->dims, &ly.q, &ly.s, u_q, Bt, L, decode, out, ssm, cs, base + c.mixer, c.mixer_bytes, st,
                       &prev, (!decode && l + 1 < m->n_layers) ? &m->layers[l + 1].q : nullptr);
    }
    if (rc != QUAMBA_OK) return rc;
  }
  hipLaunchKernelGGL(final_norm_kernel, dim3(Bt), dim3(256), 0, st, out, res,
                     reinterpret_cast<const __half *>(m->norm_f), m->eps, L, Dm, y);
  QUAMBA_LAUNCH_CHECK();
  if (!logits && !next) return QUAMBA_OK;
  const int P = (m->vocab + 63) / 64;
  hipLaunchKernelGGL(head_kernel, dim3(P, (Bt + 63) / 64), dim3(256), 0, st, y,
                     reinterpret_cast<const __half *>(m->embedding), Bt, m->vocab, Dm, logits, pmax, pidx);
  QUAMBA_LAUNCH_CHECK();
  if (next) {
    hipLaunchKernelGGL(argmax_partials_kernel, dim3(Bt), dim3(256), 0, st, pmax, pidx, P, Bt, next, log, step);
    QUAMBA_LAUNCH_CHECK();
  }
  return QUAMBA_OK;
}

int check_run(const quamba_model *m, const void *tokens, int Bt, int L, const void *ssm, const void *conv,
              const void *ws, size_t ws_bytes, Carve *c) {
  int rc = check_model(m);
  if (rc != QUAMBA_OK) return rc;
  if (!tokens || !ssm || !conv) return fail(QUAMBA_EINVAL, "model: tokens or state pointer is NULL");
  if (Bt < 1 || L < 1) return fail(QUAMBA_EINVAL, "model: batch=%d, L=%d must be >= 1", Bt, L);
  *c = carve(m, Bt, L);
  if (!ws || ws_bytes < c->total) return fail(QUAMBA_EWORKSPACE, "model: workspace %zu < %zu", ws_bytes, c->total);
  if (!aligned(ws, 256) || !aligned(ssm, 16) || !aligned(conv, 8))
    return fail(QUAMBA_EINVAL, "model: workspace must be 256-byte aligned, ssm states 16-byte, conv states 8-byte");
  return QUAMBA_OK;
}

}  // namespace
}  // namespace quamba

using namespace quamba;

extern "C" {

size_t quamba_model_workspace_bytes(const quamba_model *model, int batch, int L) {
  if (check_model(model) != QUAMBA_OK || batch < 1 || L < 1) return 0;
  return carve(model, batch, L).total;
}

int quamba_embed(const quamba_half *embedding, const int32_t *tokens, int M, int Dm, int vocab, quamba_half *res,
                 quamba_half *out, void *stream) {
  if (!embedding || !tokens || !res || !out) return fail(QUAMBA_EINVAL, "embed: NULL pointer");
  if (M < 0 || Dm < 8 || Dm % 8 || vocab < 1) return fail(QUAMBA_EINVAL, "embed: M=%d Dm=%d vocab=%d", M, Dm, vocab);
  if (!aligned(embedding, 16) || !aligned(res, 16) || !aligned(out, 16))
    return fail(QUAMBA_EINVAL, "embed: buffers must be 16-byte aligned");
  if (M == 0) return QUAMBA_OK;
  const size_t pieces = (size_t)M * (Dm / 8);
  hipLaunchKernelGGL(embed_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, as_stream(stream),
                     reinterpret_cast<const __half *>(embedding), tokens, M, Dm, vocab,
                     reinterpret_cast<__half *>(res), reinterpret_cast<__half *>(out));
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int quamba_final_norm(const quamba_half *out, const quamba_half *res, const quamba_half *weight, float eps, int Bt,
                      int L, int Dm, quamba_half *y, void *stream) {
  if (!out || !res || !weight || !y) return fail(QUAMBA_EINVAL, "final_norm: NULL pointer");
  if (Bt < 1 || L < 1) return fail(QUAMBA_EINVAL, "final_norm: Bt=%d L=%d", Bt, L);
  if (Dm < 8 || Dm % 8 || Dm > 8 * 256 * FN_MAX_PER_THREAD)
    return fail(QUAMBA_EUNSUPPORTED, "final_norm: d_model=%d must be a multiple of 8 and <= %d", Dm,
                8 * 256 * FN_MAX_PER_THREAD);
  if (!aligned(out, 16) || !aligned(res, 16) || !aligned(weight, 16) || !aligned(y, 16))
    return fail(QUAMBA_EINVAL, "final_norm: buffers must be 16-byte aligned");
  hipLaunchKernelGGL(final_norm_kernel, dim3(Bt), dim3(256), 0, as_stream(stream),
                     reinterpret_cast<const __half *>(out), reinterpret_cast<const __half *>(res),
                     reinterpret_cast<const __half *>(weight), eps, L, Dm, reinterpret_cast<__half *>(y));
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int quamba_lm_head(const quamba_half *y, const quamba_half *embedding, int Bt, int vocab, int Dm, float *logits,
                   void *stream) {
  if (!y || !embedding || !logits) return fail(QUAMBA_EINVAL, "lm_head: NULL pointer");
  if (Bt < 1 || vocab < 1 || Dm < 8 || Dm % 8) return fail(QUAMBA_EINVAL, "lm_head: Bt=%d vocab=%d Dm=%d", Bt, vocab, Dm);
  if (!aligned(y, 16) || !aligned(embedding, 16) || !aligned(logits, 16))
    return fail(QUAMBA_EINVAL, "lm_head: buffers must be 16-byte aligned");
  hipLaunchKernelGGL(head_kernel, dim3((vocab + 63) / 64, (Bt + 63) / 64), dim3(256), 0, as_stream(stream),
                     reinterpret_cast<const __half *>(y), reinterpret_cast<const __half *>(embedding), Bt, vocab, Dm,
                     logits, static_cast<float *>(nullptr), static_cast<int32_t *>(nullptr));
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int quamba_argmax(const float *logits, int Bt, int vocab, int32_t *next_token, void *stream) {
  if (!logits || !next_token) return fail(QUAMBA_EINVAL, "argmax: NULL pointer");
  if (Bt < 1 || vocab < 1) return fail(QUAMBA_EINVAL, "argmax: Bt=%d vocab=%d", Bt, vocab);
  hipLaunchKernelGGL(argmax_kernel, dim3(Bt), dim3(256), 0, as_stream(stream), logits, vocab, Bt, next_token,
                     static_cast<int32_t *>(nullptr), static_cast<const int32_t *>(nullptr));
  QUAMBA_LAUNCH_CHECK();
  return QUAMBA_OK;
}

int quamba_model_prefill(const quamba_model *model, const int32_t *tokens, int Bt, int L, float *logits,
                         int32_t *next_token, float *ssm_states, quamba_half *conv_states, void *ws, size_t ws_bytes,
                         void *stream) {
  Carve c;
  int rc = check_run(model, tokens, Bt, L, ssm_states, conv_states, ws, ws_bytes, &c);
  if (rc != QUAMBA_OK) return rc;
  if (logits && !aligned(logits, 16)) return fail(QUAMBA_EINVAL, "model: logits must be 16-byte aligned");
  {  // fresh sequences start from a zero recurrent state (a fill kernel: safe under stream capture)
    const size_t n16 = (size_t)model->n_layers * Bt * model->dims.d_inner * model->dims.d_state * sizeof(float) / 16;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, as_stream(stream),
                       reinterpret_cast<uint4 *>(ssm_states), n16);
    QUAMBA_LAUNCH_CHECK();
  }
  return run_model(model, tokens, Bt, L, false, logits, next_token, nullptr, ssm_states,
                   reinterpret_cast<__half *>(conv_states), static_cast<char *>(ws), c, as_stream(stream));
}

int quamba_model_decode(const quamba_model *model, const int32_t *tokens, int Bt, float *logits, int32_t *next_token,
                        float *ssm_states, quamba_half *conv_states, void *ws, size_t ws_bytes, void *stream) {
  Carve c;
  int rc = check_run(model, tokens, Bt, 1, ssm_states, conv_states, ws, ws_bytes, &c);
  if (rc != QUAMBA_OK) return rc;
  if (logits && !aligned(logits, 16)) return fail(QUAMBA_EINVAL, "model: logits must be 16-byte aligned");
  return run_model(model, tokens, Bt, 1, true, logits, next_token, nullptr, ssm_states,
                   reinterpret_cast<__half *>(conv_states), static_cast<char *>(ws), c, as_stream(stream));
}

int quamba_model_generate(const quamba_model *model, const int32_t *first_tokens, int Bt, int n_new,
                          int32_t *tokens_out, float *ssm_states, quamba_half *conv_states, void *ws, size_t ws_bytes,
                          int use_graph, void *stream) {
  Carve c;
  int rc = check_run(model, first_tokens, Bt, 1, ssm_states, conv_states, ws, ws_bytes, &c);
  if (rc != QUAMBA_OK) return rc;
  if (!tokens_out || n_new < 1) return fail(QUAMBA_EINVAL, "generate: tokens_out is NULL or n_new < 1");
  hipStream_t st = as_stream(stream);
  if (use_graph && st == nullptr)
    return fail(QUAMBA_EUNSUPPORTED, "generate: graph replay needs a stream other than the default stream");
  char *base = static_cast<char *>(ws);
  int32_t *cur = reinterpret_cast<int32_t *>(base + c.cur);
  int32_t *step = reinterpret_cast<int32_t *>(base + c.step);
  __half *cs = reinterpret_cast<__half *>(conv_states);
  QUAMBA_HIP(hipMemcpyAsync(cur, first_tokens, (size_t)Bt * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
  hipLaunchKernelGGL(set_step_kernel, dim3(1), dim3(1), 0, st, step, 0);
  QUAMBA_LAUNCH_CHECK();
  // one step: reads cur, writes the selected tokens to cur and to row *step of the log, advances step
  auto one_step = [&]() -> int {
    int r = run_model(model, cur, Bt, 1, true, nullptr, cur, tokens_out, ssm_states, cs, base, c, st);
    if (r != QUAMBA_OK) return r;
    hipLaunchKernelGGL(bump_kernel, dim3(1), dim3(1), 0, st, step);
    QUAMBA_LAUNCH_CHECK();
    return QUAMBA_OK;
  };
  rc = one_step();  // eager: also settles every kernel attribute before anything is captured
  if (rc != QUAMBA_OK || n_new == 1) return rc;
  if (!use_graph) {
    for (int i = 1; i < n_new; ++i) {
      rc = one_step();
      if (rc != QUAMBA_OK) return rc;
    }
    return QUAMBA_OK;
  }
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  QUAMBA_HIP(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
  rc = one_step();
  hipError_t e = hipStreamEndCapture(st, &graph);
  if (rc != QUAMBA_OK) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
  }
  if (e != hipSuccess) return fail(QUAMBA_EHIP, "generate: stream capture failed: %s", hipGetErrorString(e));
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    (void)hipGraphDestroy(graph);
    return fail(QUAMBA_EHIP, "generate: graph instantiation failed: %s", hipGetErrorString(e));
  }
  for (int i = 1; i < n_new && e == hipSuccess; ++i) e = hipGraphLaunch(exec, st);
  // the replays must have run before the executable graph is released
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  (void)hipGraphExecDestroy(exec);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) return fail(QUAMBA_EHIP, "generate: graph launch failed: %s", hipGetErrorString(e));
  return QUAMBA_OK;
}

}  // extern "C"
