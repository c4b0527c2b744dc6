"""MI355X (gfx950) sparsified Transformer-FFN training step: thin Python binding over libsparseffn.so.

Every function marshals arguments into the C ABI of include/sparseffn.h; all arithmetic runs in
the HIP kernels.  torch is used for device memory and streams only.
"""
from .binding import (SffnError, lib_path, load, version, workspace_bytes, workspace_layout,
                      prune24_compress, sqrelu_vnm_compress, spmm24_fwd, spmm24_dgrad, vnm_spmm,
                      dsqrelu_vnm, vnm_wgrad, ffn_sparse_step, FfnStep, FfnStepGrouped,
                      venom_route, venom_route_launch, venom_expert_matmul, moe_to_venom, FfnRouterStep,
                      MODE_HARD, MODE_SOFT, FLAG_KEEP_DENSE, FLAG_UNFUSED, FLAG_FP8_WGRAD, FLAG_LEAN, FLAG_WEIGHTS_PACKED, FLAG_DW_FP32_ACCUMULATE, buffer_sizes, profile_enable, profile_read, dense_sqrelu, dense_dsqrelu,
                      ffn_sparse_step_noalloc, NOALLOC_WORKSPACE_MAX,
                      prune24_compress_prepared, spmm24_prepared,
                      quantize_fp8, prune24_compress_fp8, sqrelu_vnm_compress_fp8, spmm24_fp8, vnm_spmm_fp8, FfnStepFp8, FfnStepFp8Grouped)
