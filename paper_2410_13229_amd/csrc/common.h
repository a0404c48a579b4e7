// Shared host-side helpers of the library: error reporting and launch checks.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "quamba.h"

namespace quamba {

// Per-thread text of the last error; returns `code` so callers can `return fail(...)`.
int fail(int code, const char *fmt, ...);

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// (k, m) with n = k * 2^m, k in {1, 12, 20}; false if there is none.
bool hadamard_factor(int n, int *k, int *m);

}  // namespace quamba

#define QUAMBA_HIP(expr)                                                                       \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess)                                                                      \
      return ::quamba::fail(QUAMBA_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                            __FILE__, __LINE__);                                               \
  } while (0)

#define QUAMBA_LAUNCH_CHECK() QUAMBA_HIP(hipGetLastError())

// ---- internal launchers (one per .hip file); all enqueue on `st` and return a QUAMBA_* code
namespace quamba {

// Optional tail of a generation-step in_proj (Section 4.3 fuses operators to save launches): the
// output columns below `e0` are the conv input of one token per row, and the epilogue, besides
// storing them, runs the conv step on each group of four (window of row m, channel n at
// state[(m e0 + n) 3], shifted in place) and writes the codes of x to x_q [M, e0].  Off when
// `state` is NULL.
struct ConvStepEpi {
  int8_t *x_q;
  const int8_t *w_q;   // [e0, 4]
  const float *bias;   // [e0]
  __half *state;       // [M, e0, 3]
  float s_cw, s_xpre, inv_s_x;
};

struct GemmEpilogue {
  int8_t *out_i8;
  __half *out_f16;
  int32_t *acc;
  int ldo;
  int e0, e1;
  float m0, m1, m2;
  // optional int32 term per output column [N], added to the sums before the multiplier (the
  // zero-point correction of an asymmetric input grid); 16-byte aligned; the `acc` tap stays raw
  const int32_t *col_bias;
  ConvStepEpi conv;  // only where gemm_fuses_conv_step says so
  // K split over the grid (gemm_splits > 1): leave the raw partial sums [splits][M][N] at the start of
  // the workspace and launch no reduce kernel; the consumer adds them up and applies the multipliers
  bool defer_reduce;
};

// generation takes the few-row streaming kernels up to this many sequences (at most 4); tuning hook
int gemv_max_rows();

// Which kernel launch_gemm_i8 runs for a shape and how it splits K over the grid.  A caller whose
// own launches depend on that (who adds up the partial sums, where the conv step runs) asks once
// and hands the same plan to launch_gemm_i8, so the two cannot disagree.
struct GemmPlan {
  bool gemv;  // the few-row streaming kernel
  int kind, splits, slices_per_split;
  // the launch ends in an epilogue that can carry the conv step (the 64 x 32, 32 x 32 and two-K-group 64 x 64
  // tiles of a wide generation-step output, or the reduce kernel of a split K)
  bool fuses_conv_step() const { return !gemv && (kind == 7 || kind == 11 || kind == 13 || splits > 1); }
  int k_splits() const { return gemv ? 1 : splits; }
};
// partials_wanted: the caller adds up the partial sums of a split K itself (deferred reduce), so the split form is
// kept where a form that covers K inside one launch would otherwise replace GEMM + reduce kernel.
GemmPlan gemm_plan(int M, int N, int K, const void *ws, size_t ws_bytes, bool partials_wanted = false);

// `ws` (may be NULL) lets skinny problems split K; gemm_workspace_bytes is the most they use.
size_t gemm_workspace_bytes(int M, int N);
// `plan`: the result of gemm_plan for the same shape and workspace (NULL: chosen here).
int launch_gemm_i8(const int8_t *A, int lda, const int8_t *Wt, int ldw, int M, int N, int K,
                   const GemmEpilogue &epi, void *ws, size_t ws_bytes, hipStream_t st,
                   const GemmPlan *plan = nullptr);

int launch_quantize_f16(const __half *x, int8_t *q, size_t n, float inv_s, hipStream_t st);

int launch_conv_prefill(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b,
                        int Bt, int L, int Di, float m_conv, float inv_s_x, float s_xpre,
                        int8_t *x_q, __half *conv_state, hipStream_t st, __half *x16 = nullptr,
                        int x_zero_point = 0, int x_format = 0);

int launch_conv_step(const int8_t *xpre_q, int ldx, const int8_t *w_q, const float *conv_b, int Bt,
                     int Di, float s_cw, float s_xpre, float inv_s_x, int8_t *x_q,
                     __half *conv_state, hipStream_t st, __half *x16 = nullptr, int x_zero_point = 0,
                     int x_format = 0);

// x_proj on one-byte codes of a non-uniform format, the encoder as a stage, and the bf16 copy of int8 weight codes
int launch_xfmt_proj(int format, const uint8_t *x_code, int M, int N, int K, const uint16_t *W_bf16, int e0, int e1,
                     float m0, float m1, float m2, int8_t *out_q, float *acc_f32, void *ws, size_t ws_bytes,
                     hipStream_t st);
int launch_x_encode(int format, const float *v, size_t n, float inv_s, uint8_t *codes, hipStream_t st);
int launch_i8_to_bf16(const int8_t *q, int N, int K, uint16_t *out, hipStream_t st);

// per-call scale of the scan input: *slot = bits of max|x16|; readers derive the scale from it
int launch_dyn_absmax_f16(const __half *x, size_t n, unsigned *slot, hipStream_t st);
int launch_quantize_f16_dyn(const __half *x, int8_t *q, size_t n, const unsigned *slot, hipStream_t st);
int launch_requant_dyn(const int32_t *acc, int8_t *out, int M, int N, int e0, int e1, const unsigned *slot, float s_W,
                       float so0, float so1, float so2, hipStream_t st);
int launch_dyn_export(const unsigned *slot, float *out, hipStream_t st);

int launch_add_rmsnorm_quant(const __half *x_out, __half *res, const __half *weight, float eps,
                             float inv_s, int8_t *u_q, int M, int Dm, hipStream_t st);
// the same with x_out given as `splits` (<= 8) int32 partial sums [splits][M][Dm]: x_out = fp16(m_out * their sum)
int launch_add_rmsnorm_quant_partial(const int32_t *partial, int splits, float m_out, __half *res, const __half *weight,
                                     float eps, float inv_s, int8_t *u_q, int M, int Dm, hipStream_t st);

struct ScanArgs {
  const int8_t *x_q, *dt_q, *z_q, *B_q, *C_q, *A_q, *D_q;
  const float *dt_bias;
  int ldz, ldbc;
  float s_x, s_dt, s_z, s_B, s_C, s_A, s_D;
  int Bt, L, Di;
  __half *g16;
  float *y_f32;
  float *ssm_state;
  // prefill only, optional: dt_q = q(W_dt dt_low, m_dt) is computed by the scan itself from the
  // dt_low codes [Bt*L, lddl] and W_dt [Di, R] and written to dt_out [Bt*L, Di]; dt_q is ignored
  const int8_t *dtlow_q, *W_dt;
  int lddl, R;
  float m_dt;
  int8_t *dt_out;
  // optional: the scan input given in half precision [Bt*L, Di] instead of s_x * x_q
  // (the Appendix H comparison variant); x_q and s_x are then ignored
  const __half *x_f16;
  // zero point of an asymmetric x grid (Appendix K): x = s_x (x_q - x_zero_point); 0 = symmetric
  int x_zero_point;
  // QUAMBA_XFMT_E4M3 / QUAMBA_XFMT_LOG2: x_q holds one-byte codes of that format, x = s_x * value(code); 0 = the grid above
  int x_format;
  // optional: the scale of x is not s_x but derived from this device word (bits of the call's max|x|)
  const unsigned *s_x_slot;
  // optional (generation with the fused dt_proj only): x_proj's raw sums
  // as dbc_splits (<= 8) partial results [dbc_splits][Bt][R + 2 d_state] of a K split; the step adds
  // them up and requantizes the dt_low | B | C columns itself with these multipliers;
  // dtlow_q, B_q, C_q are then ignored
  const int32_t *dbc_part;
  int dbc_splits;
  float m_x_dt, m_x_B, m_x_C;
  // prefill only, optional: memory the kernels after the scan will read (the weights of the next projections).
  // The scan is bound by its arithmetic and leaves the memory idle, so a few extra workgroups of its launch read
  // these ranges (16-byte aligned) and thereby bring them into the last-level cache; nothing is written
  const void *warm_ptr[3];
  size_t warm_bytes[3];
};

size_t scan_workspace_bytes(int Bt, int L, int Di);
int launch_scan_prefill(const ScanArgs &a, void *ws, size_t ws_bytes, hipStream_t st);
int launch_scan_step(const ScanArgs &a, hipStream_t st);

int launch_hadamard_quant(const __half *g, int M, int n, float inv_s_y, int8_t *yH_q, float *yH_f32,
                          hipStream_t st);
// x_hat = fp16(scale * H_n^T xH_q): the backward transform of the Appendix H comparison variant
bool hadamard_fuses_out_proj(int n, int Dm);
int launch_hadamard_out_proj(const __half *g, int M, int n, float inv_s_y, const int8_t *W, int Dm, float m_out,
                             __half *out, int8_t *codes, hipStream_t st);
int launch_hadamard_inverse(const int8_t *xH_q, int M, int n, float scale, __half *x_hat, hipStream_t st);

// generation with M <= 4 rows: [add + RMSNorm + quant] -> in_proj -> conv step in one kernel.
// Either u_q (already quantized input [M, Dm]) or out_prev / res_in / res_out / norm_w (res_out must
// not alias res_in: every workgroup reads res_in while workgroup 0 writes res_out).
struct DecodeInArgs {
  const __half *out_prev, *res_in;
  __half *res_out;
  const __half *norm_w;
  float eps, inv_s_u;
  const int8_t *u_q;
  const int8_t *W_in;
  int Dm, Di, M;
  float m_in_x, m_in_z;
  const int8_t *conv_w;
  const float *conv_b;
  float s_cw, s_xpre, inv_s_x;
  int8_t *x_q;        // [M, Di]
  int8_t *xz_q;       // [M, 2 Di]: x_pre codes | z codes
  int32_t *acc_in;    // [M, 2 Di] raw sums, may be NULL
  __half *conv_state; // [M, Di, 3], in/out
};
int launch_decode_in(const DecodeInArgs &a, hipStream_t st);

// one quantized mixer on already quantized input (prefill: fresh conv history; decode: L == 1 on
// carried states), its workspace size, and the dimension check of the entry points
size_t mixer_workspace_bytes(const quamba_dims *d, int Bt, int L);
// out_proj's result left as the partial sums of a K split (generation in a stack of blocks: the next
// block's add + RMSNorm + quantization adds them up, which saves the reduce kernel).  The caller sets
// `want`; the mixer sets splits (1: `out` was written as usual), partial [splits][M][d_model] (inside
// the mixer's workspace: valid until the next mixer call on it) and the multiplier of the sums.
struct OutPartial {
  bool want;
  int splits;
  const int32_t *partial;
  float m_out;
};
int mixer_run_q(const quamba_dims *d, const quamba_qweights *qw, const quamba_scales *sc, const int8_t *u_q, int Bt,
                int L, bool decode, __half *out, float *ssm_state, __half *conv_state, void *ws, size_t ws_bytes,
                hipStream_t st, OutPartial *defer_out = nullptr, const quamba_qweights *next_qw = nullptr);
// next_qw (prefill, optional): the weights of the block that runs after this one; its in_proj and x_proj weights
// and this block's out_proj weights are read into the last-level cache under the scan (ScanArgs::warm_ptr)
int check_model_dims(const quamba_dims *d);

// generation with at most 4 sequences: the block's own residual add + RMSNorm + quantization runs
// inside the mixer's first kernel.  res_out must not alias res_in.
struct NormIn {
  const __half *out_prev, *res_in;
  __half *res_out;
  const __half *norm_w;
  float eps;
};
bool mixer_decode_norm_available(const quamba_dims *d, int Bt);
int mixer_decode_norm(const quamba_dims *d, const quamba_qweights *qw, const quamba_scales *sc, const NormIn &norm,
                      int Bt, __half *out, float *ssm_state, __half *conv_state, void *ws, size_t ws_bytes,
                      hipStream_t st);

}  // namespace quamba
