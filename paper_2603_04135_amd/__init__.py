"""MI355X-native DPPO policy-loss hot path: selection, dense packing, fused LM-head
log-probabilities and the reweighted GRPO loss forward+backward, as hand-written HIP
kernels for gfx950 behind a C ABI (include/dppo.h). This package is the thin Python
binding of that library."""
from .binding import (HEAD_BAD_POSITION, HEAD_BAD_TARGET, HEAD_SEQ_TOO_LONG, DppoError, alloc_workspace, dppo_gather_f32, dppo_token_norm_coef, dppo_variance_terms, dppo_history_update, dppo_loss_fwd_bwd, dppo_mfma_rate_probe, dppo_pack,
                      dppo_select, dppo_timing_enable, dppo_timing_read, dppo_timing_tile_phases, dppo_token_logprob, dppo_token_logprob_noalloc, dppo_static_scratch_bytes, dppo_workspace_bytes, dppo_workspace_min_bytes,
                      library_path, load)

__all__ = ["HEAD_BAD_POSITION", "HEAD_BAD_TARGET", "HEAD_SEQ_TOO_LONG", "DppoError", "alloc_workspace", "dppo_gather_f32", "dppo_token_norm_coef", "dppo_variance_terms", "dppo_history_update", "dppo_loss_fwd_bwd", "dppo_mfma_rate_probe", "dppo_pack", "dppo_select",
           "dppo_timing_enable", "dppo_timing_read", "dppo_timing_tile_phases", "dppo_token_logprob", "dppo_token_logprob_noalloc", "dppo_static_scratch_bytes", "dppo_workspace_bytes", "dppo_workspace_min_bytes", "library_path", "load"]
