"""MI355X-native SpecTr-GBV verification (multi-draft greedy block verification).

The work is done by hand-written HIP kernels in ``libspecgbv.so`` behind the C ABI of
``include/specgbv.h``; this package is only the argument-marshalling binding.
"""
from .binding import (ALGO_AUTO, ALGO_CHAIN, ALGO_SPLIT, MAX_PENDING, STATIC_SCRATCH_BYTES, SpecGBVError, pending_state_views, load_library, specgbv_carry_advance,
                      specgbv_carry_workspace_bytes, specgbv_last_error,
                      specgbv_modify_target, specgbv_modify_workspace_bytes, specgbv_pending_state_bytes,
                      specgbv_read_intermediates,
                      specgbv_read_sample_intermediates, specgbv_sample_tokens, specgbv_sample_workspace_bytes,
                      specgbv_verify, specgbv_verify_ex, specgbv_verify_kseq, specgbv_read_kseq_intermediates, specgbv_verify_static, specgbv_version, specgbv_workspace_bytes,
                      specgbv_workspace_carry)

__all__ = ["ALGO_AUTO", "ALGO_CHAIN", "ALGO_SPLIT", "MAX_PENDING", "STATIC_SCRATCH_BYTES", "SpecGBVError", "pending_state_views", "load_library", "specgbv_carry_advance",
           "specgbv_carry_workspace_bytes", "specgbv_last_error",
           "specgbv_modify_target", "specgbv_modify_workspace_bytes", "specgbv_pending_state_bytes",
           "specgbv_read_intermediates",
           "specgbv_read_sample_intermediates", "specgbv_sample_tokens", "specgbv_sample_workspace_bytes",
           "specgbv_verify", "specgbv_verify_ex", "specgbv_verify_kseq", "specgbv_read_kseq_intermediates", "specgbv_verify_static", "specgbv_version", "specgbv_workspace_bytes",
           "specgbv_workspace_carry"]
