"""MI355X (gfx950) library for Probabilistic Chunk Masking and the masked GRPO actor step.

The work is done by hand-written HIP kernels behind the C boundary declared in
``include/pcm.h`` and built into ``libpcm.so`` next to this file.  This package only
marshals arguments: PyTorch supplies device memory and the current stream, every step of
the path runs in the library.  There is no CPU or PyTorch fallback: importing the binding
without the built library raises.
"""
from .binding import (  # noqa: F401
    PCM_BF16,
    PCM_F32,
    PcmError,
    grpo_masked_actor_step,
    grpo_masked_actor_step_workspace_bytes,
    lib,
    library_path,
    pcm_adamw_clip_step,
    pcm_importance_weights,
    pcm_kept_phase_counts,
    pcm_label_phases,
    pcm_measure_mfma_rate,
    pcm_pack_head_weights,
    pcm_profile_collect,
    pcm_profile_enable,
    pcm_sample_chunks,
    pcm_score_phases,
    pcm_state_bytes,
    pcm_state_init,
    pcm_update_keep_probs,
    pcm_version,
)
