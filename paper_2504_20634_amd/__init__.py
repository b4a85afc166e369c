"""Few-bit stochastic rounding (arXiv 2504.20634) for AMD MI355X: a C-ABI HIP library
(include/fbsr.h, built into paper_2504_20634_amd/libfbsr.so) and this thin ctypes binding."""
from . import binding
from .binding import (FMT_BF16, FMT_E4M3, FMT_E5M2, FMT_BINARY8P4, RNE, SRFF, SRF, SRC, SRC_TIES_ODD, RNO, RNA, SRC_BF16, SRC_FP16,
                      FROM_BF16, FROM_FP16, FROM_FP32, FbsrError, Format8, format8_named, format8_check, format16_check, fbsr_round_format16,
                      bias_stats_workspace_bytes, fbsr_bias_stats, fbsr_bias_stats_format8, fbsr_bias_stats_static, fbsr_qat_adamw_step, fbsr_qat_adamw_step_format8, fbsr_round, fbsr_round_block_scaled,
                      fbsr_round_format8, fbsr_round_from16, fbsr_sgd_update)

__all__ = ["binding", "FMT_BF16", "FMT_E4M3", "FMT_E5M2", "FMT_BINARY8P4", "RNE", "SRFF", "SRF", "SRC", "SRC_TIES_ODD", "RNO", "RNA", "SRC_BF16",
           "SRC_FP16", "FROM_BF16", "FROM_FP16", "FROM_FP32", "FbsrError", "Format8", "format8_named", "format8_check", "format16_check", "fbsr_round_format16",
           "fbsr_round_format8", "fbsr_qat_adamw_step_format8", "bias_stats_workspace_bytes", "fbsr_bias_stats", "fbsr_bias_stats_format8", "fbsr_bias_stats_static", "fbsr_qat_adamw_step", "fbsr_round", "fbsr_round_block_scaled", "fbsr_round_from16", "fbsr_sgd_update"]
