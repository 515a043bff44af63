"""MI355X-native QLoRA linear layer: NF4 + Double Quantization + LoRA, hand-written HIP for gfx950.

The public functions mirror the C ABI of include/qlora.h one to one.
"""
from .binding import (FP4_E2M1, FP4_E3M0, INT4, INT8, NF2, NF3, NF4, NF4Weight, qlora_quant_sizes, qlora_quantize_int8, QloraError, lib, nf4_alloc, qlora_codebook_4bit,
                      qlora_quantize_4bit, pack_keep_mask, qlora_linear_bwd_dropout,
                      qlora_linear_dropout_sizes, qlora_linear_fwd_dropout, qlora_linear_bwd, qlora_linear_bwd_acc, qlora_linear_bwd_sizes, qlora_linear_fwd,
                      qlora_linear_fwd_multi, qlora_linear_fwd_multi_sizes, qlora_linear_fwd_sizes, qlora_nf4_dequant, qlora_nf4_quantize, qlora_nf4_sizes,
                      qlora_profile_gemm, qlora_profile_gemm_read, qlora_workspace_init, workspace_alloc,
                      qlora_linear_list_sizes, qlora_linear_fwd_list, qlora_linear_bwd_list, qlora_workspace_check,
                      qlora_fewtok_poll_limit, qlora_bwd_fused_dequant, qlora_mfma_probe, qlora_hbm_probe, qlora_nf4_quantize_static, STATIC_QUANT_MAX_WEIGHTS,
                      qlora_grad_sqnorm, qlora_adam_step, qlora_adam_config,
                      qlora_linear_fwd_stacked, qlora_linear_fwd_stacked_sizes,
                      qlora_linear_bwd_stacked, qlora_linear_bwd_stacked_sizes,
                      qlora_kbit_sizes, qlora_kbit_pack, qlora_kbit_unpack)

# the paper-level names used in prose
nf4_quantize = qlora_nf4_quantize
nf4_dequant = qlora_nf4_dequant

__all__ = ["qlora_bwd_fused_dequant", "qlora_mfma_probe", "qlora_hbm_probe", "qlora_kbit_sizes", "qlora_kbit_pack", "qlora_kbit_unpack", "qlora_linear_bwd_stacked", "qlora_linear_bwd_stacked_sizes", "qlora_linear_fwd_stacked", "qlora_linear_fwd_stacked_sizes", "qlora_grad_sqnorm", "qlora_adam_step", "qlora_adam_config", "qlora_nf4_quantize_static", "STATIC_QUANT_MAX_WEIGHTS", "nf4_alloc", "NF4Weight", "QloraError", "lib", "qlora_nf4_sizes", "qlora_nf4_quantize", "qlora_nf4_dequant",
           "qlora_linear_fwd_sizes", "qlora_linear_bwd_sizes", "qlora_linear_fwd", "qlora_linear_bwd",
           "qlora_linear_fwd_multi_sizes", "qlora_linear_fwd_multi", "qlora_linear_bwd_acc",
           "qlora_codebook_4bit", "qlora_quantize_4bit", "NF4", "FP4_E2M1", "FP4_E3M0", "INT4", "INT8", "NF3", "NF2", "qlora_quant_sizes", "qlora_quantize_int8", "qlora_linear_dropout_sizes", "qlora_linear_fwd_dropout", "qlora_linear_bwd_dropout", "pack_keep_mask",
           "nf4_quantize", "nf4_dequant", "qlora_profile_gemm", "qlora_profile_gemm_read", "qlora_workspace_init",
           "workspace_alloc", "qlora_linear_list_sizes", "qlora_linear_fwd_list", "qlora_linear_bwd_list",
           "qlora_workspace_check", "qlora_fewtok_poll_limit"]
