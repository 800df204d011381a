/* Plain C99 client of the library: the header must compile as C, and the host-side entry points must
 * link and answer without a GPU.  Built and run by tests/test_library_symbols.py. */
#include <stdio.h>
#include <string.h>

#include "pcm.h"
#include "pcm_measure.h"

int main(void) {
    int64_t numel[2] = {4096 * 3 + 1, 5};
    pcm_loss_options opt;
    memset(&opt, 0, sizeof opt);
    opt.eps_low = 0.2f;
    opt.eps_high = 0.4f;
    opt.normalisation = PCM_NORM_TOKEN_MEAN;
    opt.ratio_level = PCM_RATIO_CHUNK;
    if (strstr(pcm_version(), "pcm") == NULL) return 1;
    if (pcm_state_bytes(5) != 16 + 24 * 5) return 2;
    if (pcm_score_phases_workspace_bytes(8, 8, 64, 56, 5) == 0) return 3;
    if (grpo_masked_actor_step_workspace_bytes(768, 56, 4096, 11008, 256, PCM_BF16, 1) == 0) return 4;
    if (pcm_adamw_clip_step_workspace_bytes(2, numel) == 0) return 5;
    /* argument validation happens on the host before any GPU call */
    if (pcm_state_init(NULL, 5, NULL) != PCM_EINVAL) return 6;
    if (grpo_masked_actor_step_ex(NULL, NULL, NULL, NULL, NULL, NULL, 1, 1, 1, 1, 256, 256, 256, PCM_BF16, NULL, NULL, NULL,
                                  NULL, &opt, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != PCM_EINVAL)
        return 7;
    if (pcm_sample_chunks_ex(NULL, NULL, NULL, NULL, 1, 1, 1, 1, PCM_SELECT_RANDOM, 0, 0, NULL, NULL, NULL, NULL, 0, NULL) !=
        PCM_EINVAL)
        return 8;
    if (pcm_label_phases(NULL, NULL, 1, 1, 1, 1, 0, 0.0f, NULL, NULL) != PCM_EINVAL) return 9;
    printf("%s: %d stages, status -2 = %s\n", pcm_version(), pcm_profile_stage_count(), pcm_status_string(PCM_EWORKSPACE));
    return 0;
}
