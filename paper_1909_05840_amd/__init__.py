"""MI355X (gfx950) implementation of Q-BERT's group-wise k-bit quantized linear layer.

The work is done by hand-written HIP kernels behind the C ABI in include/qbert.h
(libqbert.so); this package is the thin Python binding of that ABI plus the seeded synthetic
workloads.  Nothing is imported from, or falls back to, any CPU implementation.
"""
from .binding import (QBError, load_library, qb_status_string, qb_packed_nbytes, qb_bwd_workspace_nbytes, qb_workspace_nbytes,
                      qb_quantize_groupwise, qb_quantize_groupwise_batched, qb_quantize_act, qb_quantize_act_batched, qb_qlinear_fwd, qb_qlinear_fwd_batched, qb_qlinear_fwd_q8, qb_qlinear_bwd_ste, qb_qlinear_bwd_ste_static,
                      qb_unpack_codes, qb_embedding_quantize, qb_embedding_gather, qb_embedding_quantize_bits,
                      qb_embedding_gather_bits, qb_quantize_act_dyn, qb_qlinear_fwd_dyn, qb_quantize_groupwise_clip, qb_quantize_act_dyn_tensor, qb_qlinear_bwd_ste_masked,
                      qb_quantize_groupwise_asym, qb_quantize_groupwise_asym_range, qb_qlinear_fwd_asym, qb_qlinear_fwd_asym_dyn, qb_qlinear_bwd_ste_asym,
                      qb_power_iteration, qb_sensitivity_omega, qb_rank_by_sensitivity, qb_probe_mfma_i8,
                      EXPORTS, LIB_PATH)
from . import workloads

__all__ = ["QBError", "load_library", "qb_status_string", "qb_packed_nbytes", "qb_bwd_workspace_nbytes", "qb_workspace_nbytes",
           "qb_quantize_groupwise", "qb_quantize_groupwise_batched", "qb_quantize_act", "qb_quantize_act_batched", "qb_qlinear_fwd", "qb_qlinear_fwd_batched", "qb_qlinear_fwd_q8", "qb_qlinear_bwd_ste", "qb_qlinear_bwd_ste_static",
           "qb_unpack_codes", "qb_embedding_quantize", "qb_embedding_gather", "qb_embedding_quantize_bits",
           "qb_embedding_gather_bits", "qb_quantize_act_dyn", "qb_qlinear_fwd_dyn", "qb_quantize_groupwise_clip", "qb_quantize_act_dyn_tensor", "qb_qlinear_bwd_ste_masked", "qb_quantize_groupwise_asym", "qb_quantize_groupwise_asym_range",
           "qb_qlinear_fwd_asym", "qb_qlinear_fwd_asym_dyn", "qb_qlinear_bwd_ste_asym", "qb_power_iteration", "qb_sensitivity_omega",
           "qb_rank_by_sensitivity", "qb_probe_mfma_i8", "workloads", "EXPORTS", "LIB_PATH"]
