// C-ABI entry points: argument checks, workspace carving and the order of kernel launches of
// the quantized mixer (Sections 4.2 and 4.3).  No arithmetic of the method lives here.
#include <atomic>
#include <cstring>
#include <mutex>

#include "common.h"

// Scratch of quamba_mixer_decode_noalloc: the workspace of one generation step, held by every GPU the
// library runs on until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and copies get the per-device address kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[QUAMBA_NOALLOC_SCRATCH_BYTES];

namespace quamba {

// calibrate.hip
size_t calibrate_workspace_bytes(const quamba_dims *d, int nb, int Lc);
int calibrate(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
              int x_rule, double x_percentile, quamba_qweights *oq, quamba_scales *os, void *ws, size_t ws_bytes,
              hipStream_t st, float *out_f32, float *x_clip_out = nullptr);
int fp_mixer(const quamba_dims *d, const quamba_fp_weights *w, const __half *u, int nb, int Lc, float *out,
             void *ws, size_t ws_bytes, hipStream_t st);
int calibrate_hadx(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
                   double x_percentile, quamba_qweights *oq, quamba_scales *os, quamba_hadx *oh, void *ws,
                   size_t ws_bytes, hipStream_t st);
int calibrate_xasym(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc,
                    double x_percentile, quamba_qweights *oq, quamba_scales *os, quamba_xasym *oa, void *ws,
                    size_t ws_bytes, hipStream_t st);
int calibrate_xfmt(const quamba_dims *d, const quamba_fp_weights *w, const __half *calib_u, int nb, int Lc, int format,
                   double x_percentile, quamba_qweights *oq, quamba_scales *os, quamba_xfmt *of, void *ws,
                   size_t ws_bytes, hipStream_t st);
size_t clip_search_workspace_bytes();
int clip_search(const float *x, size_t n, int bits, int max_iters, double *clip_out, int *iters_out, void *ws,
                size_t ws_bytes, hipStream_t st);
int calibrate_block(const quamba_dims *d, const quamba_fp_weights *w, const __half *norm_w, float eps, float *res,
                    float *out, int nb, int Lc, double x_percentile, quamba_qweights *oq, quamba_scales *os, void *ws,
                    size_t ws_bytes, hipStream_t st);

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

namespace {

int check_dims(const quamba_dims *d) {
  if (!d) return fail(QUAMBA_EINVAL, "dims is NULL");
  if (d->d_model <= 0 || d->d_inner <= 0 || d->dt_rank <= 0)
    return fail(QUAMBA_EINVAL, "non-positive dimension");
  if (d->d_state != 16) return fail(QUAMBA_EUNSUPPORTED, "d_state=%d (only 16 is built)", d->d_state);
  if (d->d_conv != 4) return fail(QUAMBA_EUNSUPPORTED, "d_conv=%d (only 4 is built)", d->d_conv);
  if (d->d_model % 16 || d->d_inner % 16 || d->dt_rank % 16)
    return fail(QUAMBA_EUNSUPPORTED, "d_model, d_inner and dt_rank must be multiples of 16");
  int k, m;
  if (!hadamard_factor(d->d_inner, &k, &m) || m < 4)
    return fail(QUAMBA_EUNSUPPORTED, "d_inner=%d is not k*2^m with k in (1,12,20), m >= 4", d->d_inner);
  return QUAMBA_OK;
}

// Workspace carving, shared by the size query and the launches.
struct Plan {
  size_t u_q, xz_q, x_q, dbc_q, dt_q, g16, gH_q, scan, gemm, gemm_bytes, x16, acc_x, slot, total;
};

// hadx: the Appendix H comparison variant also keeps the scan input in half precision
// dyn: the dynamic-scale variant of Appendix K also keeps x in half precision, the raw x_proj sums and one word for max|x|
Plan make_plan(const quamba_dims *d, int Bt, int L, bool hadx = false, bool dyn = false) {
  const size_t M = (size_t)Bt * L;
  const size_t nx = d->dt_rank + 2 * d->d_state;
  Plan p{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += align_up(bytes, 256);
    return at;
  };
  p.u_q = take(M * d->d_model);
  p.xz_q = take(M * 2 * d->d_inner);
  p.x_q = take(M * d->d_inner);
  p.dbc_q = take(M * nx);
  p.dt_q = take(M * d->d_inner);
  p.g16 = take(M * d->d_inner * sizeof(__half));
  p.gH_q = take(M * d->d_inner);
  p.scan = take(scan_workspace_bytes(Bt, L, d->d_inner));  // a one-token prefill still runs the chunked scan
  // split-K partial sums: x_proj always (skinny N), every projection when M is small
  const size_t widest = M <= 64 ? (size_t)2 * d->d_inner : nx;
  p.gemm_bytes = gemm_workspace_bytes((int)M, (int)widest);
  p.gemm = take(p.gemm_bytes);
  p.x16 = take((hadx || dyn) ? M * d->d_inner * sizeof(__half) : 0);
  p.acc_x = take(dyn ? M * nx * sizeof(int32_t) : 0);
  p.slot = take(dyn ? 256 : 0);
  p.total = off;
  return p;
}

// Tuning hooks (process-wide; every call reads each of them once, at its start).
std::atomic<int> g_fuse_dt_hook{1};
std::atomic<int> g_fuse_decode_hook{1};

int check_q(const quamba_qweights *qw, const quamba_scales *sc) {
  if (!qw || !sc) return fail(QUAMBA_EINVAL, "qweights or scales is NULL");
  if (!qw->W_in || !qw->conv_w || !qw->W_x || !qw->W_dt || !qw->A || !qw->D || !qw->W_outH || !qw->conv_b ||
      !qw->dt_bias)
    return fail(QUAMBA_EINVAL, "a quantized weight pointer is NULL");
  // the kernels read weights and biases in 16-byte pieces
  for (const void *p : {(const void *)qw->W_in, (const void *)qw->conv_w, (const void *)qw->W_x, (const void *)qw->W_dt,
                        (const void *)qw->A, (const void *)qw->W_outH, (const void *)qw->conv_b})
    if (!aligned(p, 16)) return fail(QUAMBA_EINVAL, "quantized weights and conv_b must be 16-byte aligned");
  if (!aligned(qw->dt_bias, 4)) return fail(QUAMBA_EINVAL, "dt_bias must be 4-byte aligned");
  return QUAMBA_OK;
}

#define QUAMBA_TRY(expr)            \
  do {                              \
    int rc_ = (expr);               \
    if (rc_ != QUAMBA_OK) return rc_; \
  } while (0)

int tap_copy(void *dst, const void *src, size_t bytes, hipStream_t st) {
  if (dst) QUAMBA_HIP(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, st));
  return QUAMBA_OK;
}

// The dynamic-scale variant of Appendix K: where the caller wants the call's scale and the half-precision x (both optional).
struct DynX {
  float *s_x_out;
  __half *x16_out;
};

// Steps shared by prefill (L >= 1, fresh conv history) and decode (L == 1, carried state).
// `norm` (generation with at most 4 sequences only): the block input is not given but formed inside
// the first kernel from the previous block's output and the residual stream.
int run_mixer(const quamba_dims *d, const quamba_qweights *qw, const quamba_scales *sc, const __half *u,
              const int8_t *u_q_in, int Bt, int L, bool decode, __half *out, float *ssm_state,
              __half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes, hipStream_t st,
              const NormIn *norm = nullptr, const quamba_hadx *hx = nullptr, const quamba_hadx_taps *hx_taps = nullptr,
              const quamba_xasym *xa = nullptr, const quamba_xfmt *xf = nullptr, const DynX *dyn = nullptr,
              OutPartial *defer_out = nullptr, const quamba_qweights *next_qw = nullptr) {
  if (defer_out) defer_out->splits = 1;
  const int g_fuse_dt = g_fuse_dt_hook.load(std::memory_order_relaxed);
  const int g_fuse_decode = g_fuse_decode_hook.load(std::memory_order_relaxed);
  const int g_gemv_max_rows = gemv_max_rows();
  QUAMBA_TRY(check_dims(d));
  QUAMBA_TRY(check_q(qw, sc));
  if ((!u && !u_q_in && !norm) || !out) return fail(QUAMBA_EINVAL, "input or output pointer is NULL");
  if (norm && !(decode && Bt <= 4)) return fail(QUAMBA_EINVAL, "fused block input needs decode with batch <= 4");
  if (Bt < 1 || L < 1) return fail(QUAMBA_EINVAL, "batch=%d, L=%d must be >= 1", Bt, L);
  if (decode && (!ssm_state || !conv_state)) return fail(QUAMBA_EINVAL, "decode needs ssm_state and conv_state");
  if (hx && (!hx->W_xH || !aligned(hx->W_xH, 16))) return fail(QUAMBA_EINVAL, "variant: W_xH is NULL or not 16-byte aligned");
  if ((ssm_state && !aligned(ssm_state, 16)) || (conv_state && !aligned(conv_state, 8)))
    return fail(QUAMBA_EINVAL, "ssm_state must be 16-byte aligned, conv_state 8-byte");
  if (xa && (!xa->col_bias || !aligned(xa->col_bias, 16))) return fail(QUAMBA_EINVAL, "variant: col_bias is NULL or unaligned");
  if ((hx || xa) && norm) return fail(QUAMBA_EINVAL, "variant: the fused block input is not built for it");
  if ((hx != nullptr) + (xa != nullptr) + (xf != nullptr) + (dyn != nullptr) > 1)
    return fail(QUAMBA_EINVAL, "the x variants exclude each other");
  if (dyn && norm) return fail(QUAMBA_EINVAL, "variant: the fused block input is not built for it");
  if (dyn && (d->d_inner % 8 != 0 || (d->dt_rank + 2 * d->d_state) % 4 != 0 || d->dt_rank % 4 != 0 || d->d_state % 4 != 0))
    return fail(QUAMBA_EUNSUPPORTED, "variant: d_inner must be a multiple of 8, dt_rank and d_state multiples of 4");
  if (xf && norm) return fail(QUAMBA_EINVAL, "variant: the fused block input is not built for it");
  if (xf && (xf->format != QUAMBA_XFMT_E4M3 && xf->format != QUAMBA_XFMT_LOG2))
    return fail(QUAMBA_EINVAL, "variant: unknown x format %d", xf->format);
  if (xf && (!xf->W_x_bf16 || !aligned(xf->W_x_bf16, 16))) return fail(QUAMBA_EINVAL, "variant: W_x_bf16 is NULL or unaligned");
  if (xf && (d->d_inner % 32 != 0 || d->dt_rank + 2 * d->d_state > 320 || (d->dt_rank + 2 * d->d_state) % 4 != 0 ||
             d->dt_rank % 4 != 0 || d->d_state % 4 != 0))
    return fail(QUAMBA_EUNSUPPORTED, "variant: d_inner must be a multiple of 32, dt_rank and d_state multiples of 4, "
                                     "dt_rank + 2 d_state at most 320");
  // scale, reciprocal and zero point of the scan input's grid
  const float s_x = xa ? xa->s_x : (xf ? xf->s_x : sc->s_x), inv_s_x = xa ? xa->inv_s_x : (xf ? xf->inv_s_x : sc->inv_s_x);
  const int x_format = xf ? xf->format : 0;
  const int x_zp = xa ? xa->zero_point : 0;
  const Plan p = make_plan(d, Bt, L, hx != nullptr, dyn != nullptr);
  if (!ws || ws_bytes < p.total) return fail(QUAMBA_EWORKSPACE, "workspace %zu < %zu", ws_bytes, p.total);
  if (!aligned(ws, 256) || !aligned(out, 8) || (u && !aligned(u, 16)) || (u_q_in && !aligned(u_q_in, 16)))
    return fail(QUAMBA_EINVAL, "workspace must be 256-byte aligned, u 16-byte, out 8-byte");

  const int Dm = d->d_model, Di = d->d_inner, N = d->d_state, R = d->dt_rank, NX = R + 2 * N;
  const int M = Bt * L;
  char *base = static_cast<char *>(ws);
  int8_t *u_q = reinterpret_cast<int8_t *>(base + p.u_q);
  int8_t *xz_q = reinterpret_cast<int8_t *>(base + p.xz_q);
  int8_t *x_q = reinterpret_cast<int8_t *>(base + p.x_q);
  int8_t *dbc_q = reinterpret_cast<int8_t *>(base + p.dbc_q);
  int8_t *dt_q = reinterpret_cast<int8_t *>(base + p.dt_q);
  __half *g16 = reinterpret_cast<__half *>(base + p.g16);
  int8_t *gH_q = reinterpret_cast<int8_t *>(base + p.gH_q);
  __half *x16 = (hx || dyn) ? reinterpret_cast<__half *>(base + p.x16) : nullptr;
  unsigned *slot = dyn ? reinterpret_cast<unsigned *>(base + p.slot) : nullptr;
  int32_t *acc_x = dyn ? reinterpret_cast<int32_t *>(base + p.acc_x) : nullptr;
  const quamba_hadx_taps hnone{};
  const quamba_hadx_taps &ht = hx_taps ? *hx_taps : hnone;
  const quamba_taps none{};
  const quamba_taps &t = taps ? *taps : none;

  // Generation with one or two sequences: [norm +] in_proj + conv step in one streaming kernel
  // (the kernels serve up to 4; from 3 on the matrix-tile path with its fused epilogues is ahead:
  // 64 blocks at the 2.8B shape, 2.13 against 2.21 ms per step with 3 sequences, 2.30 against 2.45 with 4).
  const bool few = decode && M <= g_gemv_max_rows && Dm <= 8192 && g_fuse_decode && !hx && !xa && !xf && !dyn;
  if (norm && !few) return fail(QUAMBA_EINVAL, "fused block input: the few-sequence kernels do not serve this call");
  // quantize the block input (Eq. 2)
  const int8_t *uq = u_q_in;
  if (!uq && !norm) {
    QUAMBA_TRY(launch_quantize_f16(u, u_q, (size_t)M * Dm, sc->inv_s_u, st));
    uq = u_q;
  }
  if (uq) QUAMBA_TRY(tap_copy(t.u_q, uq, (size_t)M * Dm, st));

  if (few) {
    DecodeInArgs a{};
    if (norm) {
      a.out_prev = norm->out_prev; a.res_in = norm->res_in; a.res_out = norm->res_out; a.norm_w = norm->norm_w;
      a.eps = norm->eps; a.inv_s_u = sc->inv_s_u;
    } else {
      a.u_q = uq;
    }
    a.W_in = qw->W_in; a.Dm = Dm; a.Di = Di; a.M = M; a.m_in_x = sc->m_in_x; a.m_in_z = sc->m_in_z;
    a.conv_w = qw->conv_w; a.conv_b = qw->conv_b; a.s_cw = sc->s_cw; a.s_xpre = sc->s_xpre; a.inv_s_x = sc->inv_s_x;
    a.x_q = x_q; a.xz_q = xz_q; a.acc_in = t.acc_in; a.conv_state = conv_state;
    QUAMBA_TRY(launch_decode_in(a, st));
    QUAMBA_TRY(tap_copy(t.xz_q, xz_q, (size_t)M * 2 * Di, st));
  } else {
    // in_proj: columns [0, Di) -> x_pre, [Di, 2Di) -> z
    // (generation: where the GEMM's epilogue can carry it, the conv step rides along: a kernel less)
    const GemmPlan in_plan = gemm_plan(M, 2 * Di, Dm, base + p.gemm, p.gemm_bytes);
    const bool conv_in_gemm = decode && !hx && !xa && !xf && !dyn && g_fuse_decode && Di % 4 == 0 &&
                              in_plan.fuses_conv_step();
    {
      GemmEpilogue e{xz_q, nullptr, t.acc_in, 2 * Di, Di, 2 * Di, sc->m_in_x, sc->m_in_z, sc->m_in_z};
      if (conv_in_gemm) e.conv = ConvStepEpi{x_q, qw->conv_w, qw->conv_b, conv_state, sc->s_cw, sc->s_xpre, inv_s_x};
      QUAMBA_TRY(launch_gemm_i8(uq, Dm, qw->W_in, Dm, M, 2 * Di, Dm, e, base + p.gemm, p.gemm_bytes, st, &in_plan));
      QUAMBA_TRY(tap_copy(t.xz_q, xz_q, (size_t)M * 2 * Di, st));
    }
    // causal conv + SiLU + requantization with the percentile scale of x
    if (conv_in_gemm) {
    } else if (decode) {
      QUAMBA_TRY(launch_conv_step(xz_q, 2 * Di, qw->conv_w, qw->conv_b, Bt, Di, sc->s_cw, sc->s_xpre,
                                  inv_s_x, x_q, conv_state, st, x16, x_zp, x_format));
    } else {
      QUAMBA_TRY(launch_conv_prefill(xz_q, 2 * Di, qw->conv_w, qw->conv_b, Bt, L, Di, sc->m_conv, inv_s_x,
                                     sc->s_xpre, x_q, conv_state, st, x16, x_zp, x_format));
    }
  }
  if (dyn) {  // the scale of x from this call's own values, then the codes
    QUAMBA_TRY(launch_dyn_absmax_f16(x16, (size_t)M * Di, slot, st));
    QUAMBA_TRY(launch_quantize_f16_dyn(x16, x_q, (size_t)M * Di, slot, st));
    if (dyn->s_x_out) QUAMBA_TRY(launch_dyn_export(slot, dyn->s_x_out, st));
    QUAMBA_TRY(tap_copy(dyn->x16_out, x16, (size_t)M * Di * sizeof(__half), st));
  }
  if (hx) {  // forward Hadamard & quantize: x_q now holds the codes of H_n x
    QUAMBA_TRY(tap_copy(ht.x16, x16, (size_t)M * Di * sizeof(__half), st));
    QUAMBA_TRY(launch_hadamard_quant(x16, M, Di, hx->inv_s_xH, x_q, nullptr, st));
    QUAMBA_TRY(tap_copy(ht.xH_q, x_q, (size_t)M * Di, st));
  }
  QUAMBA_TRY(tap_copy(t.x_q, x_q, (size_t)M * Di, st));
  // dt_proj on the dt_low columns.  In prefill the scan's first pass computes dt_q itself when
  // the shapes allow and the raw dt_proj sums are not asked for; otherwise it is a GEMM.
  // (generation: up to 16 sequences each re-read the W_dt rows; beyond that a workgroup keeps its rows
  // in registers over 8 sequences, which needs dt_rank <= 256; prefill: L > 1)
  const bool fuse_dt = g_fuse_dt && (decode ? (M <= 16 || R <= 256) : L > 1) && !t.acc_dt && R >= 16 && R % 16 == 0 && NX % 16 == 0 && Di % 4 == 0 &&
                       aligned(qw->W_dt, 16);
  // Generation with more than a few sequences: x_proj splits K over the grid; the scan step that follows adds up the
  // partial sums of its own sequences (192 columns each) instead of a reduce kernel in between.
  bool dbc_part = false;
  int x_splits = 1;
  // x_proj: columns dt_low | B | C, each with its own output scale
  if (xf) {  // codes of a non-uniform format: bf16 matrix units on the decoded values, fp32 sums
    QUAMBA_TRY(launch_xfmt_proj(xf->format, reinterpret_cast<const uint8_t *>(x_q), M, NX, Di, xf->W_x_bf16, R, R + N,
                                xf->m_x_dt, xf->m_x_B, xf->m_x_C, dbc_q, reinterpret_cast<float *>(t.acc_x),
                                base + p.gemm, p.gemm_bytes, st));
    QUAMBA_TRY(tap_copy(t.dbc_q, dbc_q, (size_t)M * NX, st));
  } else if (dyn) {  // raw sums, then the requantization with multipliers formed on the device from the call's scale
    GemmEpilogue e{nullptr, nullptr, acc_x, NX, R, R + N, 1.f, 1.f, 1.f};
    QUAMBA_TRY(launch_gemm_i8(x_q, Di, qw->W_x, Di, M, NX, Di, e, base + p.gemm, p.gemm_bytes, st));
    QUAMBA_TRY(launch_requant_dyn(acc_x, dbc_q, M, NX, R, R + N, slot, sc->s_Wx, sc->s_dtl, sc->s_B, sc->s_C, st));
    QUAMBA_TRY(tap_copy(t.acc_x, acc_x, (size_t)M * NX * sizeof(int32_t), st));
    QUAMBA_TRY(tap_copy(t.dbc_q, dbc_q, (size_t)M * NX, st));
  } else {
    GemmEpilogue e{dbc_q, nullptr, t.acc_x, NX, R, R + N, hx ? hx->m_xh_dt : (xa ? xa->m_x_dt : sc->m_x_dt),
                   hx ? hx->m_xh_B : (xa ? xa->m_x_B : sc->m_x_B), hx ? hx->m_xh_C : (xa ? xa->m_x_C : sc->m_x_C),
                   xa ? xa->col_bias : nullptr};
    // the scan step can add up the partial sums of a split K itself: then the split form is the one wanted
    const bool x_can_defer = decode && fuse_dt && g_fuse_decode && R <= 256 && !xa && !t.dbc_q && !t.acc_x;
    const GemmPlan x_plan = gemm_plan(M, NX, Di, base + p.gemm, p.gemm_bytes, x_can_defer);
    x_splits = x_plan.k_splits();
    dbc_part = x_can_defer && x_splits > 1 && x_splits <= 8;
    e.defer_reduce = dbc_part;
    QUAMBA_TRY(launch_gemm_i8(x_q, Di, hx ? hx->W_xH : qw->W_x, Di, M, NX, Di, e, base + p.gemm, p.gemm_bytes, st, &x_plan));
    QUAMBA_TRY(tap_copy(t.dbc_q, dbc_q, (size_t)M * NX, st));
  }
  if (hx) {  // backward Hadamard: the scan's x, half precision, over the conv output that is no longer needed
    QUAMBA_TRY(launch_hadamard_inverse(x_q, M, Di, hx->xhat_scale, x16, st));
    QUAMBA_TRY(tap_copy(ht.xhat16, x16, (size_t)M * Di * sizeof(__half), st));
  }
  if (!fuse_dt) {
    GemmEpilogue e{dt_q, nullptr, t.acc_dt, Di, Di, Di, sc->m_dt, sc->m_dt, sc->m_dt};
    QUAMBA_TRY(launch_gemm_i8(dbc_q, NX, qw->W_dt, R, M, Di, R, e, base + p.gemm, p.gemm_bytes, st));
    QUAMBA_TRY(tap_copy(t.dt_q, dt_q, (size_t)M * Di, st));
  }
  // selective scan + gate
  {
    ScanArgs a{};
    a.x_q = x_q; a.dt_q = dt_q; a.z_q = xz_q + Di; a.ldz = 2 * Di;
    a.B_q = dbc_q + R; a.C_q = dbc_q + R + N; a.ldbc = NX;
    a.A_q = qw->A; a.D_q = qw->D; a.dt_bias = qw->dt_bias;
    a.s_x = s_x; a.x_zero_point = x_zp; a.s_dt = sc->s_dt; a.s_z = sc->s_z; a.s_B = sc->s_B; a.s_C = sc->s_C;
    a.s_A = sc->s_A; a.s_D = sc->s_D;
    a.Bt = Bt; a.L = L; a.Di = Di; a.g16 = g16; a.y_f32 = t.y_f32; a.ssm_state = ssm_state;
    a.x_f16 = dyn ? nullptr : x16;
    a.x_format = x_format;
    a.s_x_slot = slot;
    if (fuse_dt) {  // decode writes the dt codes only when they are asked for as a tap
      a.dtlow_q = dbc_q; a.lddl = NX; a.W_dt = qw->W_dt; a.R = R; a.m_dt = sc->m_dt;
      a.dt_out = (decode && !t.dt_q) ? nullptr : dt_q;
    }
    if (dbc_part) {
      a.dbc_part = reinterpret_cast<const int32_t *>(base + p.gemm); a.dbc_splits = x_splits;
      a.m_x_dt = hx ? hx->m_xh_dt : sc->m_x_dt; a.m_x_B = hx ? hx->m_xh_B : sc->m_x_B; a.m_x_C = hx ? hx->m_xh_C : sc->m_x_C;
    }
    if (decode) {
      QUAMBA_TRY(launch_scan_step(a, st));
    } else {
      if (next_qw) {  // a stack of blocks: warm the cache with the weights that come next
        a.warm_ptr[0] = qw->W_outH; a.warm_bytes[0] = (size_t)Dm * Di;
        a.warm_ptr[1] = next_qw->W_in; a.warm_bytes[1] = (size_t)2 * Di * Dm;
        a.warm_ptr[2] = next_qw->W_x; a.warm_bytes[2] = (size_t)NX * Di;
      }
      QUAMBA_TRY(launch_scan_prefill(a, base + p.scan, p.total - p.scan, st));
    }
    if (fuse_dt) QUAMBA_TRY(tap_copy(t.dt_q, dt_q, (size_t)M * Di, st));
    QUAMBA_TRY(tap_copy(t.g16, g16, (size_t)M * Di * sizeof(__half), st));
  }
  // Hadamard transform + quantization (Eq. 3)
  // (generation with up to three sequences: both ride in the out_proj launch; same codes, same sums)
  if (decode && M <= 3 && g_fuse_decode && !t.gH_f32 && !t.acc_out && hadamard_fuses_out_proj(Di, Dm)) {
    QUAMBA_TRY(launch_hadamard_out_proj(g16, M, Di, sc->inv_s_y, qw->W_outH, Dm, sc->m_out, out, gH_q, st));
    QUAMBA_TRY(tap_copy(t.gH_q, gH_q, (size_t)M * Di, st));
    return QUAMBA_OK;
  }
  QUAMBA_TRY(launch_hadamard_quant(g16, M, Di, sc->inv_s_y, gH_q, t.gH_f32, st));
  QUAMBA_TRY(tap_copy(t.gH_q, gH_q, (size_t)M * Di, st));
  // out_proj with the folded weight, fp16 out; the multiplier carries s_y s_WoutH / n
  {
    GemmEpilogue e{nullptr, out, t.acc_out, Dm, Dm, Dm, sc->m_out, sc->m_out, sc->m_out};
    const bool can_defer = defer_out && defer_out->want && decode && g_fuse_decode && !t.acc_out;
    const GemmPlan out_plan = gemm_plan(M, Dm, Di, base + p.gemm, p.gemm_bytes, can_defer);
    if (can_defer) {
      const int splits = out_plan.k_splits();
      if (splits > 1 && splits <= 8) {
        e.defer_reduce = true;
        *defer_out = OutPartial{true, splits, reinterpret_cast<const int32_t *>(base + p.gemm), sc->m_out};
      }
    }
    QUAMBA_TRY(launch_gemm_i8(gH_q, Di, qw->W_outH, Di, M, Dm, Di, e, base + p.gemm, p.gemm_bytes, st, &out_plan));
  }
  return QUAMBA_OK;
}

int check_calibrate_args(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_qweights *out_q,
                         const quamba_scales *out_s, const void *ws, int nb, int Lc, double x_percentile) {
  QUAMBA_TRY(check_dims(dims));
  if (!w || !out_q || !out_s || !ws) return fail(QUAMBA_EINVAL, "calibrate: NULL pointer");
  if (!w->W_in || !w->conv_w || !w->conv_b || !w->W_x || !w->W_dt || !w->dt_bias || !w->A_log || !w->D ||
      !w->W_out)
    return fail(QUAMBA_EINVAL, "calibrate: a master weight pointer is NULL");
  if (!out_q->W_in || !out_q->conv_w || !out_q->W_x || !out_q->W_dt || !out_q->A || !out_q->D ||
      !out_q->W_outH || !out_q->conv_b || !out_q->dt_bias)
    return fail(QUAMBA_EINVAL, "calibrate: an output weight pointer is NULL");
  if (nb < 1 || Lc < 1) return fail(QUAMBA_EINVAL, "calibrate: nb=%d Lc=%d", nb, Lc);
  if (!(x_percentile > 0.0 && x_percentile <= 100.0))
    return fail(QUAMBA_EINVAL, "calibrate: percentile %g outside (0, 100]", x_percentile);
  if (!aligned(ws, 256) || !aligned(w->W_out, 16))
    return fail(QUAMBA_EINVAL, "calibrate: workspace must be 256-byte aligned, W_out 16-byte");
  return QUAMBA_OK;
}

}  // namespace

size_t mixer_workspace_bytes(const quamba_dims *d, int Bt, int L) { return make_plan(d, Bt, L).total; }

int mixer_run_q(const quamba_dims *d, const quamba_qweights *qw, const quamba_scales *sc, const int8_t *u_q, int Bt,
                int L, bool decode, __half *out, float *ssm_state, __half *conv_state, void *ws, size_t ws_bytes,
                hipStream_t st, OutPartial *defer_out, const quamba_qweights *next_qw) {
  return run_mixer(d, qw, sc, nullptr, u_q, Bt, L, decode, out, ssm_state, conv_state, nullptr, ws, ws_bytes, st,
                   nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, defer_out, next_qw);
}

int mixer_decode_norm(const quamba_dims *d, const quamba_qweights *qw, const quamba_scales *sc, const NormIn &norm,
                      int Bt, __half *out, float *ssm_state, __half *conv_state, void *ws, size_t ws_bytes,
                      hipStream_t st) {
  return run_mixer(d, qw, sc, nullptr, nullptr, Bt, 1, true, out, ssm_state, conv_state, nullptr, ws, ws_bytes, st,
                   &norm);
}

bool mixer_decode_norm_available(const quamba_dims *d, int Bt) {
  return g_fuse_decode_hook.load(std::memory_order_relaxed) && Bt <= gemv_max_rows() && d->d_model <= 8192;
}

int check_model_dims(const quamba_dims *d) { return check_dims(d); }

}  // namespace quamba

using namespace quamba;

extern "C" {

const char *quamba_last_error(void) { return g_err; }

size_t quamba_workspace_bytes(const quamba_dims *dims, int batch, int L) {
  if (check_dims(dims) != QUAMBA_OK || batch < 1 || L < 1) return 0;
  return make_plan(dims, batch, L).total;
}

size_t quamba_calibrate_workspace_bytes(const quamba_dims *dims, int nb, int Lc) {
  if (check_dims(dims) != QUAMBA_OK || nb < 1 || Lc < 1) return 0;
  return calibrate_workspace_bytes(dims, nb, Lc);
}

int quamba_calibrate_x_rule(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u, int nb,
                            int Lc, int x_rule, double x_percentile, quamba_qweights *out_q, quamba_scales *out_s,
                            void *ws, size_t ws_bytes, void *stream) {
  QUAMBA_TRY(check_calibrate_args(dims, w, out_q, out_s, ws, nb, Lc, x_percentile));
  if (!calib_u) return fail(QUAMBA_EINVAL, "calibrate: NULL pointer");
  if (x_rule != QUAMBA_X_PERCENTILE && x_rule != QUAMBA_X_MSE_CLIP)
    return fail(QUAMBA_EINVAL, "calibrate: unknown x_rule %d", x_rule);
  return calibrate(dims, w, reinterpret_cast<const __half *>(calib_u), nb, Lc, x_rule, x_percentile, out_q, out_s, ws,
                   ws_bytes, as_stream(stream), nullptr);
}

int quamba_calibrate(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u, int nb,
                     int Lc, double x_percentile, quamba_qweights *out_q, quamba_scales *out_s, void *ws,
                     size_t ws_bytes, void *stream) {
  return quamba_calibrate_x_rule(dims, w, calib_u, nb, Lc, QUAMBA_X_PERCENTILE, x_percentile, out_q, out_s, ws,
                                 ws_bytes, stream);
}

int quamba_mixer_fp32(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *u, int nb, int L,
                      float *out, void *ws, size_t ws_bytes, void *stream) {
  QUAMBA_TRY(check_dims(dims));
  if (!w || !u || !out || !ws) return fail(QUAMBA_EINVAL, "fp mixer: NULL pointer");
  if (!w->W_in || !w->conv_w || !w->conv_b || !w->W_x || !w->W_dt || !w->dt_bias || !w->A_log || !w->D ||
      !w->W_out)
    return fail(QUAMBA_EINVAL, "fp mixer: a master weight pointer is NULL");
  if (nb < 1 || L < 1) return fail(QUAMBA_EINVAL, "fp mixer: nb=%d L=%d", nb, L);
  if (!aligned(ws, 256)) return fail(QUAMBA_EINVAL, "fp mixer: workspace must be 256-byte aligned");
  return fp_mixer(dims, w, reinterpret_cast<const __half *>(u), nb, L, out, ws, ws_bytes, as_stream(stream));
}

size_t quamba_clip_search_workspace_bytes(void) { return clip_search_workspace_bytes(); }

int quamba_clip_search(const float *x, size_t n, int bits, int max_iters, double *clip_out, int *iters_out, void *ws,
                       size_t ws_bytes, void *stream) {
  if (!x || !clip_out || !ws) return fail(QUAMBA_EINVAL, "clip_search: NULL pointer");
  if (n < 1 || bits < 2 || bits > 16 || max_iters < 1 || max_iters > 1024)
    return fail(QUAMBA_EINVAL, "clip_search: n=%zu bits=%d max_iters=%d", n, bits, max_iters);
  if (!aligned(ws, 256)) return fail(QUAMBA_EINVAL, "clip_search: workspace must be 256-byte aligned");
  return clip_search(x, n, bits, max_iters, clip_out, iters_out, ws, ws_bytes, as_stream(stream));
}

int quamba_calibrate_block(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *norm_w, float eps,
                           float *res, float *out, int nb, int Lc, double x_percentile, quamba_qweights *out_q,
                           quamba_scales *out_s, void *ws, size_t ws_bytes, void *stream) {
  QUAMBA_TRY(check_calibrate_args(dims, w, out_q, out_s, ws, nb, Lc, x_percentile));
  if (!norm_w || !res || !out) return fail(QUAMBA_EINVAL, "calibrate: NULL pointer");
  if (!aligned(res, 16) || !aligned(out, 16)) return fail(QUAMBA_EINVAL, "calibrate: res and out must be 16-byte aligned");
  return calibrate_block(dims, w, reinterpret_cast<const __half *>(norm_w), eps, res, out, nb, Lc, x_percentile, out_q,
                         out_s, ws, ws_bytes, as_stream(stream));
}

int quamba_mixer_prefill(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                         const quamba_half *u, int Bt, int L, quamba_half *out, float *ssm_state,
                         quamba_half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes,
                         void *stream) {
  if (!u) return fail(QUAMBA_EINVAL, "u is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, L, false,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws,
                   ws_bytes, as_stream(stream));
}

int quamba_mixer_prefill_q(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                           const int8_t *u_q, int Bt, int L, quamba_half *out, float *ssm_state,
                           quamba_half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes,
                           void *stream) {
  if (!u_q) return fail(QUAMBA_EINVAL, "u_q is NULL");
  return run_mixer(dims, qw, sc, nullptr, u_q, Bt, L, false, reinterpret_cast<__half *>(out), ssm_state,
                   reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes, as_stream(stream));
}

int quamba_mixer_decode(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                        const quamba_half *u, int Bt, quamba_half *out, float *ssm_state,
                        quamba_half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes,
                        void *stream) {
  if (!u) return fail(QUAMBA_EINVAL, "u is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, 1, true,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws,
                   ws_bytes, as_stream(stream));
}

int quamba_mixer_decode_q(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                          const int8_t *u_q, int Bt, quamba_half *out, float *ssm_state,
                          quamba_half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes,
                          void *stream) {
  if (!u_q) return fail(QUAMBA_EINVAL, "u_q is NULL");
  return run_mixer(dims, qw, sc, nullptr, u_q, Bt, 1, true, reinterpret_cast<__half *>(out), ssm_state,
                   reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes, as_stream(stream));
}

int quamba_add_rmsnorm_quant(const quamba_half *x_out, quamba_half *res, const quamba_half *weight, float eps,
                             float inv_s, int8_t *u_q, int M, int Dm, void *stream) {
  if (!x_out || !res || !weight || !u_q) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (M < 0 || Dm <= 0) return fail(QUAMBA_EINVAL, "M=%d, Dm=%d", M, Dm);
  if (M == 0) return QUAMBA_OK;
  if (!aligned(x_out, 16) || !aligned(res, 16) || !aligned(weight, 16) || !aligned(u_q, 8))
    return fail(QUAMBA_EINVAL, "add_rmsnorm_quant: buffers must be 16-byte aligned");
  return launch_add_rmsnorm_quant(reinterpret_cast<const __half *>(x_out), reinterpret_cast<__half *>(res),
                                  reinterpret_cast<const __half *>(weight), eps, inv_s, u_q, M, Dm,
                                  as_stream(stream));
}

int quamba_quantize_f16(const quamba_half *x, int8_t *q, size_t n, float inv_s, void *stream) {
  if (!x || !q) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (!aligned(x, 16) || !aligned(q, 8)) return fail(QUAMBA_EINVAL, "quantize: x 16-byte, q 8-byte aligned");
  return launch_quantize_f16(reinterpret_cast<const __half *>(x), q, n, inv_s, as_stream(stream));
}

size_t quamba_gemm_workspace_bytes(int M, int N, int K) {
  (void)K;
  if (M < 1 || N < 1) return 0;
  return gemm_workspace_bytes(M, N);
}

int quamba_gemm_i8(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K, int col_end0,
                   int col_end1, const float mult[3], int8_t *out_i8, quamba_half *out_f16, int ldo,
                   int32_t *acc_out, void *ws, size_t ws_bytes, void *stream) {
  if (!A || !Wt || !mult) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (!out_i8 && !out_f16 && !acc_out) return fail(QUAMBA_EINVAL, "gemm: no output requested");
  if (out_i8 && out_f16) return fail(QUAMBA_EINVAL, "gemm: out_i8 and out_f16 are mutually exclusive");
  if (M < 0 || N <= 0 || K <= 0) return fail(QUAMBA_EINVAL, "gemm: M=%d N=%d K=%d", M, N, K);
  if (K % 16 || lda % 16 || ldw % 16 || lda < K || ldw < K)
    return fail(QUAMBA_EUNSUPPORTED, "gemm: K, lda, ldw must be multiples of 16 with lda, ldw >= K");
  if (N % 4 || ((out_i8 || out_f16) && (ldo % 4 || ldo < N)))
    return fail(QUAMBA_EUNSUPPORTED, "gemm: N and ldo must be multiples of 4 with ldo >= N");
  if (col_end0 % 4 || col_end1 % 4 || col_end0 < 0 || col_end1 < col_end0)
    return fail(QUAMBA_EUNSUPPORTED, "gemm: column ranges must end on multiples of 4, in order");
  if (ws && !aligned(ws, 16)) return fail(QUAMBA_EINVAL, "gemm: workspace must be 16-byte aligned");
  if (!aligned(A, 16) || !aligned(Wt, 16) || (out_i8 && !aligned(out_i8, 4)) || (out_f16 && !aligned(out_f16, 8)) ||
      (acc_out && !aligned(acc_out, 16)))
    return fail(QUAMBA_EINVAL, "gemm: misaligned buffer");
  if (M == 0) return QUAMBA_OK;
  GemmEpilogue e{out_i8, reinterpret_cast<__half *>(out_f16), acc_out, ldo, col_end0, col_end1, mult[0], mult[1],
                 mult[2]};
  return launch_gemm_i8(A, lda, Wt, ldw, M, N, K, e, ws, ws ? ws_bytes : 0, as_stream(stream));
}

int quamba_conv_silu_quant(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b, int Bt, int L,
                           int Di, float m_conv, float inv_s_x, float s_xpre, int8_t *x_q,
                           quamba_half *conv_state, void *stream) {
  if (!xpre_q || !w_q || !conv_b || !x_q) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (Bt < 1 || L < 1 || Di < 4) return fail(QUAMBA_EINVAL, "conv: Bt=%d L=%d Di=%d", Bt, L, Di);
  if (Di % 4 || ldx % 4 || ldx < Di) return fail(QUAMBA_EUNSUPPORTED, "conv: Di and ldx must be multiples of 4");
  if (!aligned(xpre_q, 4) || !aligned(w_q, 16) || !aligned(conv_b, 16) || !aligned(x_q, 4))
    return fail(QUAMBA_EINVAL, "conv: misaligned buffer");
  return launch_conv_prefill(xpre_q, ldx, w_q, conv_b, Bt, L, Di, m_conv, inv_s_x, s_xpre, x_q,
                             reinterpret_cast<__half *>(conv_state), as_stream(stream));
}

int quamba_conv_step(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b, int Bt, int Di,
                     float s_cw, float s_xpre, float inv_s_x, int8_t *x_q, quamba_half *conv_state,
                     void *stream) {
  if (!xpre_q || !w_q || !conv_b || !x_q || !conv_state) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (Bt < 1 || Di < 4) return fail(QUAMBA_EINVAL, "conv_step: Bt=%d Di=%d", Bt, Di);
  if (Di % 4 || ldx % 4 || ldx < Di) return fail(QUAMBA_EUNSUPPORTED, "conv_step: Di and ldx multiples of 4");
  if (!aligned(xpre_q, 4) || !aligned(w_q, 16) || !aligned(conv_b, 16) || !aligned(x_q, 4) ||
      !aligned(conv_state, 8))
    return fail(QUAMBA_EINVAL, "conv_step: misaligned buffer");
  return launch_conv_step(xpre_q, ldx, w_q, conv_b, Bt, Di, s_cw, s_xpre, inv_s_x, x_q,
                          reinterpret_cast<__half *>(conv_state), as_stream(stream));
}

size_t quamba_scan_workspace_bytes(int Bt, int L, int Di) {
  if (Bt < 1 || L < 1 || Di < 1) return 0;
  return scan_workspace_bytes(Bt, L, Di);
}

static int fill_scan(ScanArgs &a, const int8_t *x_q, const int8_t *dt_q, const int8_t *z_q, int ldz,
                     const int8_t *B_q, const int8_t *C_q, int ldbc, const int8_t *A_q, const int8_t *D_q,
                     const float *dt_bias, const quamba_scales *sc, int Bt, int L, int Di, quamba_half *g16,
                     float *y_f32, float *ssm_state) {
  if (!x_q || !dt_q || !z_q || !B_q || !C_q || !A_q || !D_q || !dt_bias || !sc || !g16)
    return fail(QUAMBA_EINVAL, "scan: NULL pointer");
  if (Bt < 1 || L < 1 || Di < 1 || ldz < Di || ldbc < 16) return fail(QUAMBA_EINVAL, "scan: bad sizes");
  if (!aligned(A_q, 16) || (ssm_state && !aligned(ssm_state, 16)) || !aligned(B_q, 4) || !aligned(C_q, 4) ||
      ldbc % 4)
    return fail(QUAMBA_EINVAL, "scan: A_q / ssm_state must be 16-byte aligned, B_q / C_q / ldbc 4-byte");
  a.x_q = x_q; a.dt_q = dt_q; a.z_q = z_q; a.ldz = ldz; a.B_q = B_q; a.C_q = C_q; a.ldbc = ldbc;
  a.A_q = A_q; a.D_q = D_q; a.dt_bias = dt_bias;
  a.s_x = sc->s_x; a.s_dt = sc->s_dt; a.s_z = sc->s_z; a.s_B = sc->s_B; a.s_C = sc->s_C; a.s_A = sc->s_A;
  a.s_D = sc->s_D;
  a.Bt = Bt; a.L = L; a.Di = Di; a.g16 = reinterpret_cast<__half *>(g16); a.y_f32 = y_f32;
  a.ssm_state = ssm_state;
  return QUAMBA_OK;
}

int quamba_scan_prefill(const int8_t *x_q, const int8_t *dt_q, const int8_t *z_q, int ldz, const int8_t *B_q,
                        const int8_t *C_q, int ldbc, const int8_t *A_q, const int8_t *D_q, const float *dt_bias,
                        const quamba_scales *sc, int Bt, int L, int Di, quamba_half *g16, float *y_f32,
                        float *ssm_state, void *ws, size_t ws_bytes, void *stream) {
  ScanArgs a{};
  QUAMBA_TRY(fill_scan(a, x_q, dt_q, z_q, ldz, B_q, C_q, ldbc, A_q, D_q, dt_bias, sc, Bt, L, Di, g16, y_f32,
                       ssm_state));
  if (!ws || !aligned(ws, 256)) return fail(QUAMBA_EINVAL, "scan: workspace NULL or not 256-byte aligned");
  return launch_scan_prefill(a, ws, ws_bytes, as_stream(stream));
}

int quamba_scan_prefill_dtproj(const int8_t *x_q, const int8_t *dtlow_q, int lddl, const int8_t *W_dt_q, int R,
                               float m_dt, int8_t *dt_q, const int8_t *z_q, int ldz, const int8_t *B_q,
                               const int8_t *C_q, int ldbc, const int8_t *A_q, const int8_t *D_q,
                               const float *dt_bias, const quamba_scales *sc, int Bt, int L, int Di,
                               quamba_half *g16, float *y_f32, float *ssm_state, void *ws, size_t ws_bytes,
                               void *stream) {
  ScanArgs a{};
  if (!dtlow_q || !W_dt_q || !dt_q) return fail(QUAMBA_EINVAL, "scan: NULL pointer");
  QUAMBA_TRY(fill_scan(a, x_q, dt_q, z_q, ldz, B_q, C_q, ldbc, A_q, D_q, dt_bias, sc, Bt, L, Di, g16, y_f32,
                       ssm_state));
  if (!ws || !aligned(ws, 256)) return fail(QUAMBA_EINVAL, "scan: workspace NULL or not 256-byte aligned");
  a.dtlow_q = dtlow_q; a.lddl = lddl; a.W_dt = W_dt_q; a.R = R; a.m_dt = m_dt; a.dt_out = dt_q;
  return launch_scan_prefill(a, ws, ws_bytes, as_stream(stream));
}

int quamba_scan_step(const int8_t *x_q, const int8_t *dt_q, const int8_t *z_q, int ldz, const int8_t *B_q,
                     const int8_t *C_q, int ldbc, const int8_t *A_q, const int8_t *D_q, const float *dt_bias,
                     const quamba_scales *sc, int Bt, int Di, quamba_half *g16, float *y_f32, float *ssm_state,
                     void *stream) {
  ScanArgs a{};
  QUAMBA_TRY(fill_scan(a, x_q, dt_q, z_q, ldz, B_q, C_q, ldbc, A_q, D_q, dt_bias, sc, Bt, 1, Di, g16, y_f32,
                       ssm_state));
  if (!ssm_state) return fail(QUAMBA_EINVAL, "scan_step: ssm_state is required");
  return launch_scan_step(a, as_stream(stream));
}

int quamba_hadamard_quant(const quamba_half *g, int M, int n, float inv_s_y, int8_t *yH_q, float *yH_f32,
                          void *stream) {
  if (!g || !yH_q) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (M < 0 || n <= 0) return fail(QUAMBA_EINVAL, "hadamard: M=%d n=%d", M, n);
  if (M == 0) return QUAMBA_OK;
  if (!aligned(g, 16) || !aligned(yH_q, 16) || (yH_f32 && !aligned(yH_f32, 16)))
    return fail(QUAMBA_EINVAL, "hadamard: buffers must be 16-byte aligned");
  return launch_hadamard_quant(reinterpret_cast<const __half *>(g), M, n, inv_s_y, yH_q, yH_f32,
                               as_stream(stream));
}

int quamba_hadamard_inverse(const int8_t *xH_q, int M, int n, float scale, quamba_half *x_hat, void *stream) {
  if (!xH_q || !x_hat) return fail(QUAMBA_EINVAL, "NULL pointer");
  if (M < 0 || n <= 0) return fail(QUAMBA_EINVAL, "hadamard: M=%d n=%d", M, n);
  if (M == 0) return QUAMBA_OK;
  if (!aligned(xH_q, 16) || !aligned(x_hat, 16)) return fail(QUAMBA_EINVAL, "hadamard: buffers must be 16-byte aligned");
  return launch_hadamard_inverse(xH_q, M, n, scale, reinterpret_cast<__half *>(x_hat), as_stream(stream));
}

int quamba_calibrate_hadx(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u, int nb,
                          int Lc, double x_percentile, quamba_qweights *out_q, quamba_scales *out_s, quamba_hadx *out_h,
                          void *ws, size_t ws_bytes, void *stream) {
  QUAMBA_TRY(check_calibrate_args(dims, w, out_q, out_s, ws, nb, Lc, x_percentile));
  if (!calib_u || !out_h || !out_h->W_xH) return fail(QUAMBA_EINVAL, "calibrate: NULL pointer");
  return calibrate_hadx(dims, w, reinterpret_cast<const __half *>(calib_u), nb, Lc, x_percentile, out_q, out_s, out_h,
                        ws, ws_bytes, as_stream(stream));
}

int quamba_calibrate_xasym(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u, int nb,
                           int Lc, double x_percentile, quamba_qweights *out_q, quamba_scales *out_s,
                           quamba_xasym *out_a, void *ws, size_t ws_bytes, void *stream) {
  QUAMBA_TRY(check_calibrate_args(dims, w, out_q, out_s, ws, nb, Lc, x_percentile));
  if (!calib_u || !out_a || !out_a->col_bias) return fail(QUAMBA_EINVAL, "calibrate: NULL pointer");
  return calibrate_xasym(dims, w, reinterpret_cast<const __half *>(calib_u), nb, Lc, x_percentile, out_q, out_s, out_a,
                         ws, ws_bytes, as_stream(stream));
}

int quamba_mixer_prefill_xasym(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                               const quamba_xasym *xa, const quamba_half *u, int Bt, int L, quamba_half *out,
                               float *ssm_state, quamba_half *conv_state, const quamba_taps *taps, void *ws,
                               size_t ws_bytes, void *stream) {
  if (!u || !xa) return fail(QUAMBA_EINVAL, "u or xa is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, L, false,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes,
                   as_stream(stream), nullptr, nullptr, nullptr, xa);
}

int quamba_mixer_decode_xasym(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_xasym *xa, const quamba_half *u, int Bt, quamba_half *out, float *ssm_state,
                              quamba_half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes, void *stream) {
  if (!u || !xa) return fail(QUAMBA_EINVAL, "u or xa is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, 1, true,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes,
                   as_stream(stream), nullptr, nullptr, nullptr, xa);
}

int quamba_calibrate_xfmt(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u, int nb,
                          int Lc, int format, double x_percentile, quamba_qweights *out_q, quamba_scales *out_s,
                          quamba_xfmt *out_f, void *ws, size_t ws_bytes, void *stream) {
  QUAMBA_TRY(check_calibrate_args(dims, w, out_q, out_s, ws, nb, Lc, x_percentile));
  if (!calib_u || !out_f || !out_f->W_x_bf16 || !aligned(out_f->W_x_bf16, 16))
    return fail(QUAMBA_EINVAL, "calibrate: NULL pointer or unaligned W_x_bf16");
  if (format != QUAMBA_XFMT_E4M3 && format != QUAMBA_XFMT_LOG2) return fail(QUAMBA_EINVAL, "calibrate: unknown x format %d", format);
  return calibrate_xfmt(dims, w, reinterpret_cast<const __half *>(calib_u), nb, Lc, format, x_percentile, out_q, out_s,
                        out_f, ws, ws_bytes, as_stream(stream));
}

int quamba_mixer_prefill_xfmt(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_xfmt *xf, const quamba_half *u, int Bt, int L, quamba_half *out,
                              float *ssm_state, quamba_half *conv_state, const quamba_taps *taps, void *ws,
                              size_t ws_bytes, void *stream) {
  if (!xf) return fail(QUAMBA_EINVAL, "variant: xf is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, L, false, reinterpret_cast<__half *>(out),
                   ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes, as_stream(stream), nullptr,
                   nullptr, nullptr, nullptr, xf);
}

int quamba_mixer_decode_xfmt(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                             const quamba_xfmt *xf, const quamba_half *u, int Bt, quamba_half *out, float *ssm_state,
                             quamba_half *conv_state, const quamba_taps *taps, void *ws, size_t ws_bytes, void *stream) {
  if (!xf) return fail(QUAMBA_EINVAL, "variant: xf is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, 1, true, reinterpret_cast<__half *>(out),
                   ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes, as_stream(stream), nullptr,
                   nullptr, nullptr, nullptr, xf);
}

int quamba_x_encode(int format, const float *v, size_t n, float inv_s, uint8_t *codes, void *stream) {
  return launch_x_encode(format, v, n, inv_s, codes, as_stream(stream));
}

int quamba_xfmt_proj(int format, const uint8_t *x_code, int M, int N, int K, const uint16_t *W_bf16, int e0, int e1,
                     const float *m, int8_t *out_q, float *acc_f32, void *ws, size_t ws_bytes, void *stream) {
  if (!m) return fail(QUAMBA_EINVAL, "xfmt_proj: NULL multipliers");
  if (e0 < 0 || e1 < e0 || e1 > N) return fail(QUAMBA_EINVAL, "xfmt_proj: column ranges e0=%d e1=%d N=%d", e0, e1, N);
  return launch_xfmt_proj(format, x_code, M, N, K, W_bf16, e0, e1, m[0], m[1], m[2], out_q, acc_f32, ws, ws_bytes,
                          as_stream(stream));
}

size_t quamba_xdyn_workspace_bytes(const quamba_dims *dims, int batch, int L) {
  if (check_dims(dims) != QUAMBA_OK || batch < 1 || L < 1) return 0;
  return make_plan(dims, batch, L, false, true).total;
}

int quamba_mixer_prefill_xdyn(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_half *u, int Bt, int L, quamba_half *out, float *ssm_state,
                              quamba_half *conv_state, const quamba_taps *taps, float *s_x_out, quamba_half *x16_out,
                              void *ws, size_t ws_bytes, void *stream) {
  const DynX dyn{s_x_out, reinterpret_cast<__half *>(x16_out)};
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, L, false, reinterpret_cast<__half *>(out),
                   ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes, as_stream(stream), nullptr,
                   nullptr, nullptr, nullptr, nullptr, &dyn);
}

int quamba_mixer_decode_xdyn(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                             const quamba_half *u, int Bt, quamba_half *out, float *ssm_state, quamba_half *conv_state,
                             const quamba_taps *taps, float *s_x_out, quamba_half *x16_out, void *ws, size_t ws_bytes,
                             void *stream) {
  const DynX dyn{s_x_out, reinterpret_cast<__half *>(x16_out)};
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, 1, true, reinterpret_cast<__half *>(out),
                   ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes, as_stream(stream), nullptr,
                   nullptr, nullptr, nullptr, nullptr, &dyn);
}

size_t quamba_hadx_workspace_bytes(const quamba_dims *dims, int batch, int L) {
  if (check_dims(dims) != QUAMBA_OK || batch < 1 || L < 1) return 0;
  return make_plan(dims, batch, L, true).total;
}

int quamba_mixer_prefill_hadx(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_hadx *hx, const quamba_half *u, int Bt, int L, quamba_half *out,
                              float *ssm_state, quamba_half *conv_state, const quamba_taps *taps,
                              const quamba_hadx_taps *hx_taps, void *ws, size_t ws_bytes, void *stream) {
  if (!u || !hx) return fail(QUAMBA_EINVAL, "u or hx is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, L, false,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes,
                   as_stream(stream), nullptr, hx, hx_taps);
}

int quamba_mixer_decode_hadx(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                             const quamba_hadx *hx, const quamba_half *u, int Bt, quamba_half *out, float *ssm_state,
                             quamba_half *conv_state, const quamba_taps *taps, const quamba_hadx_taps *hx_taps, void *ws,
                             size_t ws_bytes, void *stream) {
  if (!u || !hx) return fail(QUAMBA_EINVAL, "u or hx is NULL");
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, 1, true,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws, ws_bytes,
                   as_stream(stream), nullptr, hx, hx_taps);
}

}  // extern "C"

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};  // address of `scratch` on each device, resolved on first use

// Address of the current device's copy of `scratch` (each GPU has its own, at its own address).
int scratch_of_current_device(void **out) {
  int dev = -1;
  QUAMBA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(QUAMBA_EUNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    QUAMBA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || !aligned(p, 256)) return fail(QUAMBA_EHIP, "scratch symbol resolved to %p", p);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return QUAMBA_OK;
}

}  // namespace

extern "C" int quamba_mixer_decode_noalloc(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                                           const quamba_half *u, int Bt, quamba_half *out, float *ssm_state,
                                           quamba_half *conv_state, const quamba_taps *taps, void *stream) {
  if (!u) return fail(QUAMBA_EINVAL, "u is NULL");
  QUAMBA_TRY(check_dims(dims));
  if (Bt < 1) return fail(QUAMBA_EINVAL, "batch=%d must be >= 1", Bt);
  const size_t need = make_plan(dims, Bt, 1).total;
  if (need > sizeof(scratch))
    return fail(QUAMBA_EWORKSPACE, "decode_noalloc: a step of %d sequences at d_model=%d d_inner=%d needs %zu bytes of "
                                   "scratch, the built-in buffer holds %zu; use quamba_mixer_decode with a workspace",
                Bt, dims->d_model, dims->d_inner, need, sizeof(scratch));
  void *ws = nullptr;
  QUAMBA_TRY(scratch_of_current_device(&ws));
  return run_mixer(dims, qw, sc, reinterpret_cast<const __half *>(u), nullptr, Bt, 1, true,
                   reinterpret_cast<__half *>(out), ssm_state, reinterpret_cast<__half *>(conv_state), taps, ws,
                   sizeof(scratch), as_stream(stream));
}

extern "C" void quamba_debug_set_fuse_dt(int v) { quamba::g_fuse_dt_hook.store(v); }
extern "C" void quamba_debug_set_fuse_decode(int v) { quamba::g_fuse_decode_hook.store(v); }
