"""CPU oracle for the W8A8 Mamba-mixer path (test infrastructure only).

A plain, slow, numpy implementation of what the quantized mixer computes, written from
the paper's statement of the method (Sections 3.1-3.3, 4.2, 4.3 and 5.1).  It exists to
check the HIP library; it is NOT a fallback.  Only tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it, and it imports nothing from the HIP
package.

Precision policy
  * Every value that feeds a rounding-to-integer decision is formed in fp32 with the
    operation order written in the function, so the HIP path can take the same decision.
  * Everything else (the fp reference mixer, the recurrence of the selective scan, the
    dense Hadamard product) is fp64.

Pins (tests/test_oracle_*.py): Hadamard orthogonality and the Sylvester closed form,
fold identity of the output projection, quantizer error bound / saturation / idempotence,
nearest-rank percentile vs a sort, integer GEMM vs int64 loops, conv vs an explicit
Toeplitz product and causality, scan vs cumulative sum / unrolled sum / chunk splitting /
the LTI error bound of Theorem 4.1; the fused residual add + RMSNorm + quantizer vs its closed form
on constant rows (graded weight; eps inside the root); the model shell: final norm closed form, head of a one-hot
vector, and generation by carried state against re-running the prefill on the grown sequence.

parity unpinned: the end-to-end numbers of ``q_prefill`` / ``q_decode`` (the paper prints
no worked example of a quantized mixer); they are pinned only relatively, against the fp
reference mixer and through the ablation behaviour of Table "quamba_ablation".
"""
from .hadamard import hadamard_matrix, hadamard_factor, sylvester, paley1  # noqa: F401
from .quantizer import (rne, quantize, requant_acc, absmax_scale, percentile_max,  # noqa: F401
                        int_matmul, optimal_clip, clip_mse_model)
from .mixer import (fp_forward, calibrate, q_prefill, q_decode, selective_scan,  # noqa: F401
                    causal_conv_fp, add_rmsnorm_quant, silu, softplus, q_scan, q_hadamard_quant,
                    q_out_proj, q_conv_prefill, q_conv_step)
from .stack import calibrate_stack, q_stack_prefill, q_stack_decode  # noqa: F401
from .model import (embed, final_norm, lm_head, greedy, model_prefill, model_decode,  # noqa: F401
                    model_generate)
from .mamba_had import (calibrate_hadx, q_prefill_hadx, q_decode_hadx,  # noqa: F401
                        hadamard_inverse_dequant)
from .x_asym import calibrate_xasym, q_prefill_xasym, q_decode_xasym, quantize_asym  # noqa: F401
from .x_formats import (calibrate_xfmt, q_prefill_xfmt, q_decode_xfmt, encode_e4m3, decode_e4m3,  # noqa: F401
                        encode_log2, decode_log2)
from .x_dynamic import q_prefill_xdyn, q_decode_xdyn, dynamic_scale, dynamic_multipliers  # noqa: F401
