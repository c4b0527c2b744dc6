"""CPU oracle for the sparsified FFN training step (test infrastructure only).

A plain, slow numpy restatement of what the paper's Section 3 (Alg. 1 and Alg. 2),
Section 2.2 (2:4 magnitude pruning / soft-thresholding), Section 2.3 (V:N:M format) and
Section 3.3 / Alg. 3 (neuron-level experts producing the V:N:M format) and Section 3.4's closing paragraph (fp8 operands,
quantised in the sparsification passes) compute.  bf16 tensors are uint16 bit patterns; every contraction is a float64 matmul
on explicitly masked dense matrices.  Nothing here is imported by the product package:
only tests, the smoke check and the benchmark's cpu_baseline leg may use it, and it
shares no code with the HIP kernels.
"""
from .bf16 import bits_to_f32, bits_to_f64, f32_to_bits, f64_to_bits
from .sparse24 import (prune24_positions, prune24_compress, prune24_decompress,
                       prune24_dense)
from .vnm import (sqrelu, vnm_select_columns, vnm_compress, vnm_decompress,
                  sqrelu_vnm_compress, dsqrelu_vnm, vnm_to_24)
from .gemm import spmm24, vnm_spmm, vnm_wgrad, dense_nt
from .ffn import ffn_sparse_step_ref, ffn_dense_ref, ffn_sparse_step_grouped_ref
from .router import (route_scores, route_scores_plain, route_margin_is_clear, route_top1, expert_permutation, cluster_rows, expert_matmul, venom_from_compact,
                     moe_to_venom, scatter_compact, ffn_router_step_ref)
from . import fp8
from .fp8 import (e4m3_decode, e4m3_encode, quantize_fp8, prune24_compress_fp8, sqrelu_vnm_compress_fp8, spmm24_fp8, vnm_spmm_fp8, ffn_sparse_step_fp8_ref, ffn_sparse_step_fp8_grouped_ref)
