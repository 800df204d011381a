"""Seeded synthetic inputs shaped like the paper's rollouts (Sec. 5.1, App. D).

This package only *draws data*: rewards, phase labels, continuous actions and
their bin indices, trunk hidden states and head weights.  It contains none of
the method's arithmetic (no advantages, scores, keep probabilities, sampling or
head math), so both the HIP path and the CPU checker may be fed from it.
"""
from .rollouts import (  # noqa: F401
    CONFIGS,
    RolloutConfig,
    make_head_numpy,
    make_gripper_actions,
    make_head_torch,
    make_hidden_numpy,
    make_hidden_torch,
    make_rollouts,
    perturb_numpy,
    perturb_torch,
    ragged_n_chunks,
    to_bf16_grid,
)
