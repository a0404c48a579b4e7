/*
 * quamba.h - C ABI of the MI355X (gfx950) W8A8 Mamba-mixer library.
 *
 * The library implements the quantized Mamba block of "Quamba" (arXiv 2410.13229):
 * static per-tensor int8 projections, fused int8 causal conv + SiLU, a selective scan that
 * dequantizes its int8 inputs in-kernel, and a fused Hadamard transform + quantization in
 * front of an output projection whose weight has the Hadamard matrix folded in.
 *
 * Conventions for every entry point
 *   - plain C; returns 0 (QUAMBA_OK) or a negative QUAMBA_E* code; the text of the last
 *     error of the calling thread is available from quamba_last_error().
 *   - every pointer is a DEVICE pointer unless the comment says "host"; quamba_dims,
 *     quamba_scales and the pointer-holding structs themselves live in host memory.
 *   - all buffers are caller-owned; the library allocates no device memory and frees none.
 *     Scratch comes from the caller's workspace `ws` (size from the matching
 *     *_workspace_bytes query, 256-byte aligned).
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and the call returns without synchronising, except the calibration calls, which
 *     synchronise the stream to hand the scales back in host memory, and graph-replayed
 *     generation (quamba_model_generate with use_graph), which waits for its last replay and
 *     lets the HIP runtime allocate what its graph objects need.
 *   - calls that share no output, state or workspace buffer may be in flight on different
 *     streams (and from different host threads) at once; independent sequences overlap well: one
 *     call's projections use the matrix cores while another's scan uses the vector units.  What the
 *     library keeps between calls: the process-wide tuning hooks at the end of this file (defaults =
 *     the measured choices; only tests and tuning runs touch them), the per-device scratch buffer of
 *     quamba_mixer_decode_noalloc (its calls on one GPU must not overlap), and the one-time
 *     per-device set-up of kernel attributes.
 *   - alignment: workspaces 256 bytes; weights, conv_b, fp16 / int8 activations and ssm_state 16
 *     bytes; conv_state and fp16 outputs 8 bytes (what any allocator returns; a view that starts
 *     inside a tensor may not qualify and is refused with QUAMBA_EINVAL).
 *   - fp16 tensors are IEEE binary16 (quamba_half = raw 16-bit storage).
 *   - tensors are dense row-major with the last index fastest; weights are [out, in].
 *   - notation: Dm = d_model, Di = d_inner, N = d_state (16), R = dt_rank, W = d_conv (4),
 *     Bt = batch, L = sequence length, M = Bt*L tokens.
 */
#ifndef QUAMBA_H
#define QUAMBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t quamba_half;

enum {
  QUAMBA_OK = 0,
  QUAMBA_EINVAL = -1,       /* null pointer, non-positive size, misaligned buffer            */
  QUAMBA_EUNSUPPORTED = -2, /* d_state != 16, d_conv != 4, d_inner without a k*2^m Hadamard
                               factorisation (k in 1, 12, 20; 2^m >= 16), sizes not
                               multiples of 16                                               */
  QUAMBA_EWORKSPACE = -3,   /* workspace smaller than the *_workspace_bytes query            */
  QUAMBA_EHIP = -4          /* a HIP runtime call failed                                     */
};

typedef struct {
  int32_t d_model, d_inner, d_state, dt_rank, d_conv;
} quamba_dims;

/* fp32 master weights of one mixer (Section 3.1): in_proj rows [0,Di) give x, rows [Di,2Di)
 * give the gate z; x_proj rows are dt | B | C. */
typedef struct {
  const float *W_in;    /* [2*Di, Dm] */
  const float *conv_w;  /* [Di, W]    */
  const float *conv_b;  /* [Di]       */
  const float *W_x;     /* [R+2N, Di] */
  const float *W_dt;    /* [Di, R]    */
  const float *dt_bias; /* [Di]       */
  const float *A_log;   /* [Di, N]    A = -exp(A_log) */
  const float *D;       /* [Di]       */
  const float *W_out;   /* [Dm, Di]   */
} quamba_fp_weights;

/* int8 weights (Section 3.2 Eq. 2, Section 4.2): same shapes as above; A holds q(-exp(A_log));
 * W_outH holds q(W_out^H) with row m = H_n W_out[m, :] (Section 4.2 fold).  The two bias
 * vectors stay fp32. */
typedef struct {
  int8_t *W_in, *conv_w, *W_x, *W_dt, *A, *D, *W_outH;
  float *conv_b, *dt_bias;
} quamba_qweights;

/* Static per-tensor scales (Eq. 2; the scan input x uses the percentile maximum of Section
 * 4.2) and the fp32 multipliers the fused epilogues apply.  Host memory.  Each multiplier is
 * the stated product evaluated in double and rounded once to fp32:
 *   inv_s_u = 1/s_u            m_in_x = s_u s_Win / s_xpre     m_in_z = s_u s_Win / s_z
 *   m_conv  = s_cw s_xpre      inv_s_x = 1/s_x
 *   m_x_dt  = s_x s_Wx / s_dtl m_x_B  = s_x s_Wx / s_B         m_x_C  = s_x s_Wx / s_C
 *   m_dt    = s_dtl s_Wdt / s_dt                inv_s_y = 1/s_y
 *   m_out   = s_y s_WoutH / Di   (carries the 1/n of the fold identity) */
typedef struct {
  float s_u, s_xpre, s_z, s_x, s_dtl, s_B, s_C, s_dt, s_y;
  float s_Win, s_cw, s_Wx, s_Wdt, s_A, s_D, s_WoutH;
  float inv_s_u, m_in_x, m_in_z, m_conv, inv_s_x, m_x_dt, m_x_B, m_x_C, m_dt, inv_s_y, m_out;
} quamba_scales;

/* Optional copies of the intermediates, for parity tests.  Any member may be NULL; the struct
 * pointer itself may be NULL.  All are dense [M, cols] with M = Bt*L (decode: M = Bt).
 * Asking for acc_dt makes dt_proj run as a GEMM of its own; otherwise the scan kernels form
 * dt_q themselves where the shapes allow (same codes either way). */
typedef struct {
  int8_t *u_q;      /* [M, Dm]    quantized block input                  */
  int32_t *acc_in;  /* [M, 2*Di]  in_proj accumulators                   */
  int8_t *xz_q;     /* [M, 2*Di]  x_pre | z                              */
  int8_t *x_q;      /* [M, Di]    conv + SiLU output = scan input        */
  int32_t *acc_x;   /* [M, R+2N]  x_proj accumulators                    */
  int8_t *dbc_q;    /* [M, R+2N]  dt_low | B | C                         */
  int32_t *acc_dt;  /* [M, Di]    dt_proj accumulators                   */
  int8_t *dt_q;     /* [M, Di]                                            */
  float *y_f32;     /* [M, Di]    gated scan output before fp16 rounding */
  quamba_half *g16; /* [M, Di]    gated scan output, fp16                */
  float *gH_f32;    /* [M, Di]    H_n g before quantization              */
  int8_t *gH_q;     /* [M, Di]                                            */
  int32_t *acc_out; /* [M, Dm]    out_proj accumulators                  */
} quamba_taps;

/* Text of the last error raised on the calling thread ("" if none).  Host pointer, valid
 * until the next failing call on the same thread. */
const char *quamba_last_error(void);

/* ---------------------------------------------------------------------------------------
 * Whole-mixer entry points
 * ------------------------------------------------------------------------------------- */

/* Bytes of workspace quamba_mixer_prefill / quamba_mixer_decode need for `batch` sequences
 * of length `L` (decode: L = 1).  Returns 0 for unsupported dims. */
size_t quamba_workspace_bytes(const quamba_dims *dims, int batch, int L);

/* Bytes of workspace quamba_calibrate needs for an [nb, Lc, Dm] calibration batch. */
size_t quamba_calibrate_workspace_bytes(const quamba_dims *dims, int nb, int Lc);

/* Calibration (Section 5.1 "Quantization setup"; Section 4.2): runs the unquantized mixer in
 * fp32 on `calib_u` [nb, Lc, Dm] (fp16), takes absmax/127 as the scale of every activation
 * and weight, except the scan input x whose scale is the nearest-rank `x_percentile`-th
 * percentile of |x| over the whole batch divided by 127 (rank = ceil(p/100 * count));
 * collects the scale of y^H = H_n (y SiLU(z)); forms W_out^H; quantizes all weights into
 * `out_q` (device buffers provided by the caller); fills `out_s` (host) including the
 * epilogue multipliers.  Synchronises `stream` once before returning. */
int quamba_calibrate(const quamba_dims *dims, const quamba_fp_weights *w,
                     const quamba_half *calib_u, int nb, int Lc, double x_percentile,
                     quamba_qweights *out_q, quamba_scales *out_s /* host */,
                     void *ws, size_t ws_bytes, void *stream);

/* Calibration with a choice of rule for the scale of the scan input x.  Section 5.1 mentions,
 * next to the percentile, a clipping optimisation as the enhanced variant and Table "percentiles"
 * sets the two side by side; the paper cites the algorithm without printing it and does not say
 * which tensors it clips, so here it replaces the percentile for x only:
 *   QUAMBA_X_PERCENTILE  s_x = percentile maximum / 127 (what quamba_calibrate does)
 *   QUAMBA_X_MSE_CLIP    s_x = c / 127 with c the scalar minimising
 *                        (4^-8 / 3) c^2 #{0 < |x| <= c} + sum_{|x| > c} (|x| - c)^2
 *                        (rounding noise inside the clip + overshoot outside), see quamba_clip_search;
 *                        x_percentile is checked but not used.
 * Everything else is as in quamba_calibrate. */
#define QUAMBA_X_PERCENTILE 0
#define QUAMBA_X_MSE_CLIP 1
int quamba_calibrate_x_rule(const quamba_dims *dims, const quamba_fp_weights *w,
                            const quamba_half *calib_u, int nb, int Lc, int x_rule, double x_percentile,
                            quamba_qweights *out_q, quamba_scales *out_s /* host */,
                            void *ws, size_t ws_bytes, void *stream);

/* ---- The comparison variant of Appendix H (the rotation recipe for Transformers moved onto the
 * Mamba block), on the scan-input path.  The paper measures it to show what its own recipe
 * avoids: forward Hadamard & quantize and a backward Hadamard between the conv and the scan,
 * with the Hadamard matrix folded into the linear layer that reads x.  The wiring (the figure is
 * not in the text, so this is a reading):
 *   x16   = fp16(SiLU(conv(x_pre_q)))                         (conv output, not quantized)
 *   xH_q  = q(H_n x16, s_xH), s_xH = max|H_n x| / 127          (forward transform + quantize)
 *   x_proj reads xH_q with W_xH = q(rows of W_x transformed by H_n), 1/n in the multipliers
 *   x_hat = fp16((s_xH / n) H_n^T xH_q)                       (backward transform)
 *   the scan takes x_hat in half precision in place of s_x x_q
 * and everything else is the Quamba path.  The layout transposes the paper lists come from the
 * kernels it reused; this library is token-major throughout and has none.
 * quamba_hadx: the variant's extra calibration results; W_xH [dt_rank + 2 d_state, d_inner] is
 * device memory provided by the caller, the scalars are host values. */
typedef struct quamba_hadx {
  int8_t *W_xH;
  float s_xH, s_WxH, inv_s_xH, m_xh_dt, m_xh_B, m_xh_C, xhat_scale /* s_xH / n */;
} quamba_hadx;

/* optional taps of the variant, device pointers, any may be NULL: x16, x_hat [M, d_inner] fp16,
 * xH_q [M, d_inner] int8 */
typedef struct quamba_hadx_taps {
  quamba_half *x16;
  int8_t *xH_q;
  quamba_half *xhat16;
} quamba_hadx_taps;

/* quamba_calibrate plus the variant's extras (fills *out_h on the host, writes out_h->W_xH on
 * the device); same workspace as quamba_calibrate. */
int quamba_calibrate_hadx(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u,
                          int nb, int Lc, double x_percentile, quamba_qweights *out_q,
                          quamba_scales *out_s /* host */, quamba_hadx *out_h /* host */, void *ws,
                          size_t ws_bytes, void *stream);

/* The variant's mixer: arguments as quamba_mixer_prefill / quamba_mixer_decode plus `hx`; `taps->x_q`,
 * if given, receives xH_q.  Workspace: quamba_hadx_workspace_bytes (decode: L = 1). */
size_t quamba_hadx_workspace_bytes(const quamba_dims *dims, int batch, int L);
int quamba_mixer_prefill_hadx(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_hadx *hx, const quamba_half *u, int Bt, int L, quamba_half *out,
                              float *ssm_state, quamba_half *conv_state, const quamba_taps *taps,
                              const quamba_hadx_taps *hx_taps, void *ws, size_t ws_bytes, void *stream);
int quamba_mixer_decode_hadx(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                             const quamba_hadx *hx, const quamba_half *u, int Bt, quamba_half *out,
                             float *ssm_state, quamba_half *conv_state, const quamba_taps *taps,
                             const quamba_hadx_taps *hx_taps, void *ws, size_t ws_bytes, void *stream);

/* Stage of the variant: x_hat [M, n] = fp16(scale * H_n^T xH_q [M, n]) (the integer sums are exact);
 * n = k 2^m as for quamba_hadamard_quant; pointers 16-byte aligned. */
int quamba_hadamard_inverse(const int8_t *xH_q, int M, int n, float scale, quamba_half *x_hat, void *stream);

/* ---- Asymmetric 8-bit grid with percentile clipping for the scan input x (Appendix K, "MinMax Asym.
 * Per."): x is the output of SiLU, bounded below by about -0.28 and reaching far above, so an affine
 * grid over [lo, hi] has about half the step of the symmetric one over [-hi, hi]; the price is a
 * zero point in the operators that read x.  The paper gives no formulas; this reading:
 *   lo = min(min x, 0), hi = the percentile maximum, s = (hi - lo) / 255, zp = clamp(rne(-128 - lo / s))
 *   x_q = clamp(rne(fp32(x * (1/s)) + zp))  (conv epilogue);  x = s (x_q - zp)  (inside the scan)
 *   x_proj: sums + col_bias[n], col_bias[n] = -zp * sum_k W_x_q[n, k], multipliers with s in place of s_x
 * quamba_xasym: col_bias [dt_rank + 2 d_state] int32 is device memory provided by the caller (16-byte
 * aligned), the scalars are host values.  Entry points as quamba_calibrate / quamba_mixer_prefill /
 * quamba_mixer_decode, plus `xa`; same workspaces. */
typedef struct quamba_xasym {
  int32_t *col_bias;
  int32_t zero_point;
  float s_x, inv_s_x, m_x_dt, m_x_B, m_x_C;
} quamba_xasym;
int quamba_calibrate_xasym(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u,
                           int nb, int Lc, double x_percentile, quamba_qweights *out_q,
                           quamba_scales *out_s /* host */, quamba_xasym *out_a /* host */, void *ws,
                           size_t ws_bytes, void *stream);
int quamba_mixer_prefill_xasym(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                               const quamba_xasym *xa, const quamba_half *u, int Bt, int L, quamba_half *out,
                               float *ssm_state, quamba_half *conv_state, const quamba_taps *taps, void *ws,
                               size_t ws_bytes, void *stream);
int quamba_mixer_decode_xasym(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_xasym *xa, const quamba_half *u, int Bt, quamba_half *out,
                              float *ssm_state, quamba_half *conv_state, const quamba_taps *taps, void *ws,
                              size_t ws_bytes, void *stream);

/* ---- Non-uniform 8-bit formats for the scan input x (Appendix K: row "MinMax Sym. Log2", and the E4M3
 * float its last paragraph names).  The appendix reports log2 as slightly better than Quamba's grid but
 * without a matrix-multiply form on the frameworks it used; here x_proj has one: every decoded value and
 * every int8 weight code is exact in bfloat16, so x_proj runs on the bf16 matrix units with fp32 sums.
 * The paper gives no formulas; this reading (t = fp32(x) * fp32(1/s), one multiply):
 *   QUAMBA_XFMT_LOG2  s = max|x| over the calibration batch; t = f 2^E, 1 <= f < 2, goes to 2^k with
 *                     k = E + (f >= fp32(sqrt 2)); code = sign bit | e, e = -k in 0..126 (t > 1 saturates
 *                     at e = 0), 127 = zero (also anything below 2^-126.5);  x = sign s 2^-e
 *   QUAMBA_XFMT_E4M3  1-4-3 bits, bias 7, subnormals m 2^-9, largest finite value 448, no infinities, the
 *                     two not-a-number codes never produced; s = max^p(|x|) / 448; t goes to the nearest
 *                     value, ties to the even mantissa, saturating at +-448;  x = s value(code)
 *   x_proj: acc[n] = sum_k W_x_q[n, k] value(code_k) (fp32 sums in a fixed order: K is cut in equal
 *           ranges whose sums are added in ascending order); outputs clamp(rne(acc * m)), m = s s_Wx / s_out
 * quamba_xfmt: W_x_bf16, (dt_rank + 2 d_state) * d_inner 16-bit words of device memory provided by the caller
 * (16-byte aligned) and written by the calibration: the int8 codes of W_x as bfloat16 bit patterns, in the
 * order the matrix unit consumes them, with N = dt_rank + 2 d_state:
 *   W_x_bf16[(s N + n) 16 + 8 h + j] = bf16(W_x_q[n, 32 (s / 2) + 16 h + 8 (s % 2) + j]),  s < d_inner / 16, h < 2, j < 8
 * the scalars are host values.  Entry points as quamba_calibrate / quamba_mixer_prefill / quamba_mixer_decode, plus
 * `xf`; same workspaces.  taps->x_q receives the code bytes, taps->acc_x the fp32 sums (as bit patterns
 * in the int32 buffer); d_inner must be a multiple of 32 and dt_rank + 2 d_state at most 320. */
#define QUAMBA_XFMT_E4M3 1
#define QUAMBA_XFMT_LOG2 2
typedef struct quamba_xfmt {
  uint16_t *W_x_bf16;
  int32_t format;
  float s_x, inv_s_x, m_x_dt, m_x_B, m_x_C;
} quamba_xfmt;
int quamba_calibrate_xfmt(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *calib_u,
                          int nb, int Lc, int format, double x_percentile, quamba_qweights *out_q,
                          quamba_scales *out_s /* host */, quamba_xfmt *out_f /* host */, void *ws,
                          size_t ws_bytes, void *stream);
int quamba_mixer_prefill_xfmt(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_xfmt *xf, const quamba_half *u, int Bt, int L, quamba_half *out,
                              float *ssm_state, quamba_half *conv_state, const quamba_taps *taps, void *ws,
                              size_t ws_bytes, void *stream);
int quamba_mixer_decode_xfmt(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                             const quamba_xfmt *xf, const quamba_half *u, int Bt, quamba_half *out,
                             float *ssm_state, quamba_half *conv_state, const quamba_taps *taps, void *ws,
                             size_t ws_bytes, void *stream);
/* Stages of the variant.  quamba_x_encode: codes[i] = encode(fp32(v[i]) * inv_s) for n fp32 values.
 * quamba_xfmt_proj: out_q [M, N] int8 = clamp(rne(acc * m)) with acc as above over x_code [M, K] and
 * W_bf16 (N * K words in the order above); columns [0, e0) use m[0], [e0, e1) m[1], [e1, N) m[2] (multiples of 4); acc_f32 [M, N]
 * (may be NULL) receives the sums; ws: quamba_gemm_workspace_bytes(M, N, K) bytes, 256-byte aligned.
 * K a multiple of 32, N a multiple of 4 and at most 320; pointers 16-byte aligned. */
int quamba_x_encode(int format, const float *v, size_t n, float inv_s, uint8_t *codes, void *stream);
int quamba_xfmt_proj(int format, const uint8_t *x_code, int M, int N, int K, const uint16_t *W_bf16, int e0, int e1,
                     const float *m /* host, 3 */, int8_t *out_q, float *acc_f32, void *ws, size_t ws_bytes,
                     void *stream);

/* ---- Dynamic 8-bit quantization of the scan input x (Appendix K, row "Dynamic / MinMax Sym."): the scale
 * of x is not calibrated but taken from the values of the call (all sequences and tokens it processes):
 *   x16 = fp16(SiLU(conv)),  s = max|x16| / 127 (1 if that is 0),  x_q = clamp(rne(fp32(x16) * (1 / s)))
 *   x_proj outputs clamp(rne(acc * m)), m = (s * s_Wx) / s_out;  x = s x_q inside the scan
 * every division and product a single correctly rounded fp32 operation, formed on the device by each reader
 * from one word holding max|x16|: no host round trip, and the whole step stays a fixed launch sequence.
 * The appendix's point is the price: three small kernels more than the static path (maximum, quantization,
 * requantization of the x_proj sums) and the conv output kept in half precision between them.
 * qw / sc come from quamba_calibrate (its s_x is not used).  s_x_out (device, one float, may be NULL)
 * receives the scale the call used, x16_out (device [Bt*L, d_inner] fp16, may be NULL) the half-precision
 * x; taps as for quamba_mixer_prefill (acc_x: the raw x_proj sums).  ws: quamba_xdyn_workspace_bytes.
 * d_inner must be a multiple of 8. */
size_t quamba_xdyn_workspace_bytes(const quamba_dims *dims, int batch, int L);
int quamba_mixer_prefill_xdyn(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                              const quamba_half *u, int Bt, int L, quamba_half *out, float *ssm_state,
                              quamba_half *conv_state, const quamba_taps *taps, float *s_x_out, quamba_half *x16_out,
                              void *ws, size_t ws_bytes, void *stream);
int quamba_mixer_decode_xdyn(const quamba_dims *dims, const quamba_qweights *qw, const quamba_scales *sc,
                             const quamba_half *u, int Bt, quamba_half *out, float *ssm_state, quamba_half *conv_state,
                             const quamba_taps *taps, float *s_x_out, quamba_half *x16_out, void *ws, size_t ws_bytes,
                             void *stream);

/* The unquantized mixer (Section 3.1: in_proj, causal conv + SiLU, selection, selective scan,
 * gate, out_proj) in fp32 from the fp32 master weights, each of the nb sequences of length L from
 * an empty history: u [nb, L, Dm] fp16 in, out [nb * L, Dm] fp32.  It is what calibration observes
 * and the reference the quantized mixer's error is measured against; plain untuned kernels.
 * Workspace: quamba_calibrate_workspace_bytes(dims, nb, L), 256-byte aligned.  Enqueues only. */
int quamba_mixer_fp32(const quamba_dims *dims, const quamba_fp_weights *w, const quamba_half *u, int nb,
                      int L, float *out, void *ws, size_t ws_bytes, void *stream);

/* The clipping scalar of QUAMBA_X_MSE_CLIP for any fp32 device array x[0, n), for a quantizer of
 * `bits` bits (2..16): starting from c = mean|x|, repeat
 *   c <- sum(|x| : |x| > c) / (4^-bits / 3 * #{0 < |x| <= c} + #{|x| > c})
 * until c stops changing, nothing lies outside c, or max_iters (1..1024) updates were made; sums
 * in fp64, added in a fixed order (same result on every run).  Writes c (0 for an all-zero
 * array) and, if iters_out is not NULL, the number of updates made, both HOST memory;
 * synchronises the stream.  Workspace: quamba_clip_search_workspace_bytes(), 256-byte aligned. */
size_t quamba_clip_search_workspace_bytes(void);
int quamba_clip_search(const float *x, size_t n, int bits, int max_iters, double *clip_out /* host */,
                       int *iters_out /* host, may be NULL */, void *ws, size_t ws_bytes, void *stream);

/* Quantized mixer over whole sequences, starting from an empty conv history (Sections 4.2,
 * 4.3): quantize u -> int8 in_proj -> int8 causal conv + SiLU -> int8 x_proj, dt_proj ->
 * selective scan (int8 in, fp32 state, SiLU(z) gate, fp16 out) -> Hadamard + quantize ->
 * int8 out_proj with W_out^H, fp16 out.
 *   u          [Bt, L, Dm] fp16 in
 *   out        [Bt, L, Dm] fp16 out
 *   ssm_state  [Bt, Di, N] fp32: holds h_0 on entry and h_L on return; NULL = start from
 *              zeros and do not return the state
 *   conv_state [Bt, Di, W-1] fp16 out (last W-1 dequantized conv inputs, oldest first);
 *              may be NULL
 * quamba_mixer_prefill_q takes the block input already quantized with s_u (what the fused
 * add+RMSNorm+quant of the previous block produces) and skips the first step. */
int quamba_mixer_prefill(const quamba_dims *dims, const quamba_qweights *qw,
                         const quamba_scales *sc /* host */, const quamba_half *u, int Bt, int L,
                         quamba_half *out, float *ssm_state, quamba_half *conv_state,
                         const quamba_taps *taps, void *ws, size_t ws_bytes, void *stream);
int quamba_mixer_prefill_q(const quamba_dims *dims, const quamba_qweights *qw,
                           const quamba_scales *sc /* host */, const int8_t *u_q, int Bt, int L,
                           quamba_half *out, float *ssm_state, quamba_half *conv_state,
                           const quamba_taps *taps, void *ws, size_t ws_bytes, void *stream);

/* One generation step (L = 1) on carried state: same chain; the conv runs in fp32 over
 * [conv_state, s_xpre * x_pre_q] with dequantized weights and the window shifts by one; the
 * scan is one recurrence step.  ssm_state [Bt, Di, N] fp32 and conv_state [Bt, Di, W-1] fp16
 * are updated in place (both required).  u, out: [Bt, Dm] fp16. */
int quamba_mixer_decode(const quamba_dims *dims, const quamba_qweights *qw,
                        const quamba_scales *sc /* host */, const quamba_half *u, int Bt,
                        quamba_half *out, float *ssm_state, quamba_half *conv_state,
                        const quamba_taps *taps, void *ws, size_t ws_bytes, void *stream);
int quamba_mixer_decode_q(const quamba_dims *dims, const quamba_qweights *qw,
                          const quamba_scales *sc /* host */, const int8_t *u_q, int Bt,
                          quamba_half *out, float *ssm_state, quamba_half *conv_state,
                          const quamba_taps *taps, void *ws, size_t ws_bytes, void *stream);

/* quamba_mixer_decode for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same step,
 * same kernels, same results bit for bit; the scratch is a buffer of QUAMBA_NOALLOC_SCRATCH_BYTES built
 * into the library's device image (every GPU the library runs on holds it until the process ends).
 * The call allocates and frees nothing.  A step that needs more than the buffer (quamba_workspace_bytes(dims,
 * Bt, 1) > QUAMBA_NOALLOC_SCRATCH_BYTES; the 2.8B layer fits up to 128 sequences) is refused with
 * QUAMBA_EWORKSPACE.  The device that `stream` belongs to must be current.  All calls on one GPU share
 * that GPU's buffer: calls that overlap on one GPU (different streams or threads) race; nothing in the
 * buffer has to start at zero, every step overwrites what it reads.  The first call on a device looks
 * the buffer's address up (not a stream operation: make one call before capturing a graph). */
#define QUAMBA_NOALLOC_SCRATCH_BYTES (48u << 20)
int quamba_mixer_decode_noalloc(const quamba_dims *dims, const quamba_qweights *qw,
                                const quamba_scales *sc /* host */, const quamba_half *u, int Bt,
                                quamba_half *out, float *ssm_state, quamba_half *conv_state,
                                const quamba_taps *taps, void *stream);

/* Fused residual add + RMSNorm + static quantization between blocks (Section 4.3 "Fused
 * RMSNorm"): res <- fp16(x_out + res) in place; u_q = q(RMSNorm(res) * weight, 1/s) with
 * the norm taken in fp32 over the stored fp16 residual.
 *   x_out, res [M, Dm] fp16; weight [Dm] fp16; u_q [M, Dm] int8 out. */
int quamba_add_rmsnorm_quant(const quamba_half *x_out, quamba_half *res, const quamba_half *weight,
                             float eps, float inv_s, int8_t *u_q, int M, int Dm, void *stream);

/* ---------------------------------------------------------------------------------------
 * Stage entry points (the kernels the mixer calls, exposed one by one)
 * ------------------------------------------------------------------------------------- */

/* Eq. 2 in fused form: q[i] = clamp(rne(float(x[i]) * inv_s), -128, 127). x fp16, count n. */
int quamba_quantize_f16(const quamba_half *x, int8_t *q, size_t n, float inv_s, void *stream);

/* int8 GEMM on the matrix cores (Section 4.3 "Projection layers"):
 *   acc[m, j] = sum_k A[m, k] * Wt[j, k]   (int32, exact)
 * A [M, K] with row stride lda, Wt [N, K] with row stride ldw (K, lda, ldw multiples of 16;
 * N, ldo, col_end0, col_end1 multiples of 4).  Column j belongs to range 0 if j < col_end0,
 * range 1 if j < col_end1, else range 2, and is scaled by mult[range].
 *   out_i8  != NULL: out_i8[m, j] = clamp(rne(float(acc) * mult), -128, 127), row stride ldo
 *   out_f16 != NULL: out_f16[m, j] = fp16(float(acc) * mult), row stride ldo
 *   acc_out != NULL: raw accumulators, dense [M, N]
 * At least one output is required; out_i8 and out_f16 are mutually exclusive.
 * ws (may be NULL) is scratch of quamba_gemm_workspace_bytes(M, N, K) bytes: with it, problems
 * with few output tiles and deep K are split along K and summed by a second kernel (integer
 * sums: the result is the same either way). */
size_t quamba_gemm_workspace_bytes(int M, int N, int K);
int quamba_gemm_i8(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
                   int col_end0, int col_end1, const float mult[3] /* host */,
                   int8_t *out_i8, quamba_half *out_f16, int ldo, int32_t *acc_out,
                   void *ws, size_t ws_bytes, void *stream);

/* Fused int8 causal depthwise conv + SiLU + requantization (Section 4.3 "Fused causal
 * convolution"), width 4, empty history at t < 0 of every sequence:
 *   x_q[b,t,d] = q(SiLU(float(sum_j w_q[d,j] * xpre_q[b,t-3+j,d]) * m_conv + conv_b[d]), inv_s_x)
 * xpre_q has row stride ldx (it is the left half of the in_proj output); x_q is dense
 * [Bt*L, Di].  conv_state (may be NULL) [Bt, Di, 3] fp16 receives fp16(s_xpre * xpre_q) of
 * the last three tokens, oldest first (zeros where L < 3). */
int quamba_conv_silu_quant(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b,
                           int Bt, int L, int Di, float m_conv, float inv_s_x, float s_xpre,
                           int8_t *x_q, quamba_half *conv_state, void *stream);

/* Decode form of the same operator: window = [conv_state (3, fp16), s_xpre * xpre_q] in fp32,
 * weights s_cw * w_q; conv_state shifts by one in place. xpre_q [Bt, Di] with row stride ldx. */
int quamba_conv_step(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b,
                     int Bt, int Di, float s_cw, float s_xpre, float inv_s_x,
                     int8_t *x_q, quamba_half *conv_state, void *stream);

/* Quantized selective scan with gate (Section 3.1 Eq. 1; Section 4.2 "Quantization for
 * Selective SSM"): all inputs int8 and dequantized inside the kernel with the static scales:
 *   x = s_x x_q, dt = softplus(s_dt dt_q + dt_bias), A = s_A A_q, B = s_B B_q, C = s_C C_q,
 *   D = s_D D_q, z = s_z z_q;
 *   h_t = exp(dt_t A) h_{t-1} + dt_t B_t x_t;  y_t = C_t . h_t + D x_t;  g_t = y_t SiLU(z_t)
 * with fp32 state.  x_q, dt_q dense [Bt*L, Di]; z_q row stride ldz; B_q and C_q row stride
 * ldbc (columns of the x_proj output); A_q [Di, 16]; D_q [Di]; dt_bias [Di] fp32.
 *   g16   [Bt*L, Di] fp16 out          y_f32 (may be NULL) same shape, value before rounding
 *   ssm_state [Bt, Di, 16] fp32 in/out (NULL: zeros in, nothing out)
 * Range of g16: the fp32 value is converted with round-to-nearest-even and NOT saturated: a gated output
 * beyond the largest finite half (|g| >= 65520) becomes +-infinity, as the IEEE conversion defines (the
 * recurrent state stays fp32 and is not affected).  The Hadamard stage then turns the whole token row into
 * infinities / NaNs and its int8 codes are unspecified, so static scales must leave that margin: with the
 * paper's observation of output outliers of a few hundred (Appendix I, J) the margin is two orders of magnitude.
 * quamba_scan_prefill runs a chunked three-pass scan over L; it needs
 * quamba_scan_workspace_bytes(Bt, L, Di) bytes of workspace.  quamba_scan_step is L = 1. */
size_t quamba_scan_workspace_bytes(int Bt, int L, int Di);
int quamba_scan_prefill(const int8_t *x_q, const int8_t *dt_q, const int8_t *z_q, int ldz,
                        const int8_t *B_q, const int8_t *C_q, int ldbc, const int8_t *A_q,
                        const int8_t *D_q, const float *dt_bias, const quamba_scales *sc /* host */,
                        int Bt, int L, int Di, quamba_half *g16, float *y_f32, float *ssm_state,
                        void *ws, size_t ws_bytes, void *stream);
/* The same scan with dt_proj fused into its first pass (Section 4.3 fuses operators to save
 * launches and traffic): dt_q = q(W_dt_q dtlow_q, m_dt) with dtlow_q [Bt*L, lddl] (the dt_low
 * columns of the x_proj output, row stride lddl), W_dt_q [Di, R], m_dt = s_dtlow s_Wdt / s_dt.
 * dt_q [Bt*L, Di] is an OUTPUT here (written before the scan reads it).  Needs R and lddl
 * multiples of 16 (R >= 16), Di a multiple of 4, dtlow_q and W_dt_q 16-byte aligned, else
 * QUAMBA_EUNSUPPORTED; everything else as quamba_scan_prefill. */
int quamba_scan_prefill_dtproj(const int8_t *x_q, const int8_t *dtlow_q, int lddl,
                               const int8_t *W_dt_q, int R, float m_dt, int8_t *dt_q,
                               const int8_t *z_q, int ldz, const int8_t *B_q, const int8_t *C_q,
                               int ldbc, const int8_t *A_q, const int8_t *D_q, const float *dt_bias,
                               const quamba_scales *sc /* host */, int Bt, int L, int Di,
                               quamba_half *g16, float *y_f32, float *ssm_state,
                               void *ws, size_t ws_bytes, void *stream);
int quamba_scan_step(const int8_t *x_q, const int8_t *dt_q, const int8_t *z_q, int ldz,
                     const int8_t *B_q, const int8_t *C_q, int ldbc, const int8_t *A_q,
                     const int8_t *D_q, const float *dt_bias, const quamba_scales *sc /* host */,
                     int Bt, int Di, quamba_half *g16, float *y_f32, float *ssm_state,
                     void *stream);

/* Fused fast Hadamard transform + quantization (Section 4.2 "SSM outputs", Eq. 3;
 * Section 3.3): per row, yH = H_n g with n = k*2^m (k in 1, 12, 20; H_n = H_k (x) H_{2^m},
 * H_12 / H_20 from the first Paley construction, H_{2^m} in natural Sylvester order), then
 * yH_q = clamp(rne(yH * inv_s_y), -128, 127).  g [M, n] fp16; yH_q [M, n] int8;
 * yH_f32 (may be NULL) [M, n] the transform before quantization. */
int quamba_hadamard_quant(const quamba_half *g, int M, int n, float inv_s_y, int8_t *yH_q,
                          float *yH_f32, void *stream);

/* Calibration of one block of a stack (Section 5.1: per-layer static scales; Section 4.3 for the
 * norm between blocks).  The caller carries the UNQUANTIZED residual stream in fp32:
 *   res [nb*Lc, d_model] in/out, out [nb*Lc, d_model] in/out (start: res = hidden, out = 0).
 * The call forms res += out, u = RMSNorm(res) * norm_w (fp16 [d_model]), calibrates the block on u
 * exactly as quamba_calibrate does on its calib_u, and leaves this block's unquantized output in
 * out for the next call.  Same workspace size as quamba_calibrate; synchronises the stream. */
int quamba_calibrate_block(const quamba_dims *dims, const quamba_fp_weights *w,
                           const quamba_half *norm_w, float eps, float *res, float *out, int nb,
                           int Lc, double x_percentile, quamba_qweights *out_q,
                           quamba_scales *out_s /* host */, void *ws, size_t ws_bytes, void *stream);

/* ---- Whole-model shell.  Section 5.2 reports time to first token (prefill), time per output
 * token (one generation step) and time to last token of the full language model; this is that
 * loop around the quantized blocks:
 *   res = E[token] (fp16), out = 0;
 *   block l: (u_q, res) = add_rmsnorm_quant(out, res; norm_w_l, 1/s_u,l); out = mixer_l(u_q)
 *   y = fp16(RMSNorm(out + res) * norm_f); logits = y E^T (fp32 sums); next = argmax
 * The embedding and the head are one fp16 matrix and are not quantized (Section 4.3 quantizes
 * the blocks).  `layers` is a HOST array of n_layers entries whose weight pointers are device
 * memory and whose scales are host values; embedding [vocab, d_model] and the norm weights
 * [d_model] are fp16 device memory, 16-byte aligned; d_model <= 8192. */
typedef struct quamba_layer {
  quamba_qweights q;
  quamba_scales s;
  const quamba_half *norm_w;
} quamba_layer;

typedef struct quamba_model {
  quamba_dims dims;
  int n_layers;
  int vocab;
  float eps;
  const quamba_half *embedding;
  const quamba_half *norm_f;
  const quamba_layer *layers;
} quamba_model;

/* The shell's own stages, one entry point each (all buffers device memory, 16-byte aligned):
 *   quamba_embed       res[m, :] = embedding[clamp(tokens[m], 0, vocab-1), :], out[m, :] = 0; fp16 [M, Dm]
 *   quamba_final_norm  y[b, :] = fp16(RMSNorm(fp16(out[r] + res[r])) * weight), r = b*L + L-1: the last
 *                      position of each of Bt sequences of L rows; y fp16 [Bt, Dm]; Dm <= 8192
 *   quamba_lm_head     logits[b, v] = sum_k y[b, k] embedding[v, k], fp32 sums of fp16 products; [Bt, vocab]
 *   quamba_argmax      next_token[b] = lowest index of the largest logit of row b
 * Dm a multiple of 8. */
int quamba_embed(const quamba_half *embedding, const int32_t *tokens, int M, int Dm, int vocab,
                 quamba_half *res, quamba_half *out, void *stream);
int quamba_final_norm(const quamba_half *out, const quamba_half *res, const quamba_half *weight,
                      float eps, int Bt, int L, int Dm, quamba_half *y, void *stream);
int quamba_lm_head(const quamba_half *y, const quamba_half *embedding, int Bt, int vocab, int Dm,
                   float *logits, void *stream);
int quamba_argmax(const float *logits, int Bt, int vocab, int32_t *next_token, void *stream);

/* Bytes of workspace for batch sequences of L tokens (generation: L = 1); 0 on bad arguments. */
size_t quamba_model_workspace_bytes(const quamba_model *model, int batch, int L);

/* Prefill of fresh sequences: tokens int32 [Bt, L] (device; ids outside [0, vocab) are clamped).
 *   logits      fp32 [Bt, vocab] of the last position, 16-byte aligned (may be NULL)
 *   next_token  int32 [Bt]: argmax of those logits, lowest index among equal maxima (may be NULL)
 *   ssm_states  fp32 [n_layers, Bt, d_inner, 16], conv_states fp16 [n_layers, Bt, d_inner, 3]:
 *               OUTPUTS here (the recurrent state starts from zero), inputs of the decode calls
 * Enqueued on `stream`, not synchronised. */
int quamba_model_prefill(const quamba_model *model, const int32_t *tokens, int Bt, int L,
                         float *logits, int32_t *next_token, float *ssm_states,
                         quamba_half *conv_states, void *ws, size_t ws_bytes, void *stream);

/* One generation step on the carried states (in/out): tokens int32 [Bt]. */
int quamba_model_decode(const quamba_model *model, const int32_t *tokens, int Bt, float *logits,
                        int32_t *next_token, float *ssm_states, quamba_half *conv_states,
                        void *ws, size_t ws_bytes, void *stream);

/* Greedy generation of n_new tokens per sequence from first_tokens [Bt] (device; typically the
 * next_token of the prefill): step i feeds the token chosen by step i - 1.  tokens_out int32
 * [n_new, Bt] receives the chosen tokens.  The current token, the step counter and the log stay
 * on the device, so a step is a fixed sequence of launches: with use_graph != 0 the first step
 * runs eagerly, the second is captured from `stream` (which must not be the default stream)
 * into a HIP graph, and the graph is replayed for the rest; the call then returns after the last
 * replay has finished.  With use_graph == 0 every step is enqueued eagerly and the call does not
 * synchronise. */
int quamba_model_generate(const quamba_model *model, const int32_t *first_tokens, int Bt,
                          int n_new, int32_t *tokens_out, float *ssm_states,
                          quamba_half *conv_states, void *ws, size_t ws_bytes, int use_graph,
                          void *stream);

/* ---------------------------------------------------------------------------------------
 * Diagnostics: instruction-rate probes behind the roofline statements (no part of the method).
 * A probe is one kernel of register-only loops on every SIMD of the chip (256 CUs x 4 SIMDs x
 * waves_per_simd waves, `iters` rounds); the caller times the launch and divides:
 *   QUAMBA_PROBE_FMA_F32          8 independent v_fma_f32 per round
 *   QUAMBA_PROBE_EXP_F32          8 independent v_exp_f32 per round (the decay factor of Eq. 1)
 *   QUAMBA_PROBE_SCAN_MIX         8 state updates of Eq. 1 per round: multiply, exponential, multiply,
 *                                 two multiply-adds each
 *   QUAMBA_PROBE_MFMA_I8          4 independent v_mfma_i32_32x32x32_i8 per round, all-zero operands
 *   QUAMBA_PROBE_MFMA_I8_RANDOM   the same with the caller's operands: the first 4096 bytes of `ws`
 *                                 (4 operand registers x 64 lanes x 16 int8), e.g. seeded random codes
 * *instr_per_call (host) receives the number of counted instructions (state updates for SCAN_MIX,
 * 65536 integer operations per MFMA) of the launch.  Workspace: quamba_probe_workspace_bytes; after the
 * launch its bytes [4096, 4112) hold two uint64: the ticks of the shader clock and of the constant-rate
 * clock between the start and the end of the first wave (their ratio times the constant rate is the
 * shader clock the probe ran at). */
#define QUAMBA_PROBE_FMA_F32 0
#define QUAMBA_PROBE_EXP_F32 1
#define QUAMBA_PROBE_SCAN_MIX 2
#define QUAMBA_PROBE_MFMA_I8 3
#define QUAMBA_PROBE_MFMA_I8_RANDOM 4
#define QUAMBA_PROBE_MUL_F32 5        /* 8 independent v_mul_f32 per round */
#define QUAMBA_PROBE_FMA_EXP_INDEP 6  /* 4 v_fma_f32 and 4 v_exp_f32 per round, all independent */
#define QUAMBA_PROBE_MIX_NOEXP 7      /* SCAN_MIX with a multiply-add in the exponential's place */
#define QUAMBA_PROBE_MIX_GROUPED 8    /* SCAN_MIX with the 8 exponentials of a round issued as one run */
size_t quamba_probe_workspace_bytes(int waves_per_simd);
int quamba_probe_rate(int probe, int waves_per_simd, int iters, double *instr_per_call /* host */,
                      void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * Tuning hooks: process-wide switches that choose between kernels which compute the same
 * thing; tests use them to run the non-default forms, tuning runs to compare them.  Each is
 * one atomic word that a call reads once at its start, so a call is consistent in itself; a
 * hook changed while calls are in flight applies to whichever calls start after it.  Results
 * do not depend on them beyond what the tests of the alternative forms state (bit-identical,
 * except where a row's sum of squares is accumulated in another order).
 *   quamba_debug_set_gemm_variant(v)   v >= 0 forces GEMM kernel configuration v (0..13) where the
 *                                      shape allows it, and switches the launcher's row split off;
 *                                      -1 = chosen per shape (default)
 *   quamba_debug_set_gemm_split(v)     v > 1 forces a K split into v ranges over the grid; 0 = default
 *   quamba_debug_set_gemv_max_rows(v)  generation takes the few-row streaming kernels up to v
 *                                      sequences (0..4); negative = default (2)
 *   quamba_debug_set_fuse_dt(v)        0: dt_proj always as a GEMM of its own; 1 = default (inside
 *                                      the scan where the shape allows and acc_dt is not tapped)
 *   quamba_debug_set_fuse_decode(v)    0: generation without the fused epilogues and hand-overs
 *                                      (conv step in in_proj, split-K sums added up by the consumer,
 *                                      Hadamard inside out_proj, fused few-sequence kernels); 1 = default
 *   quamba_debug_set_scan_variant(v)   prefill scan: 1 = always the three-pass chunked form, 2 = one sweep per
 *                                      sequence wherever its layout rules hold, 0 = default (the cheaper of
 *                                      the two by the library's estimate for the shape)
 * ------------------------------------------------------------------------------------- */
void quamba_debug_set_gemm_variant(int v);
void quamba_debug_set_gemm_split(int v);
void quamba_debug_set_gemv_max_rows(int v);
void quamba_debug_set_fuse_dt(int v);
void quamba_debug_set_fuse_decode(int v);
void quamba_debug_set_scan_variant(int v);

#ifdef __cplusplus
}
#endif
#endif /* QUAMBA_H */
