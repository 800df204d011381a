"""GPU parity of pcm_label_phases (through the C boundary) against the checker: labels are integers,
so the comparison is exact.  Inputs: synthetic gripper traces with grasp cycles (workloads), at the
shapes of all configurations, plus ragged, degenerate and threshold cases."""
import numpy as np
import pytest
import torch

from oracle import pcm_oracle as O
from workloads import CONFIGS, make_gripper_actions, ragged_n_chunks

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pcm():
    import paper_2605_16154_amd as m
    m.lib()
    return m


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def both(pcm, actions, n_chunks, L, D, **kw):
    ref = O.label_phases(actions, n_chunks, L, D, **kw)
    got = pcm.pcm_label_phases(dev(actions), None if n_chunks is None else dev(n_chunks), L, D, **kw)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), ref)
    return ref


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4", "cfg5"])
def test_labels_match_checker(pcm, name):
    cfg = CONFIGS[name]
    a = make_gripper_actions(cfg, 0)
    ref = both(pcm, a, None, cfg.L, cfg.D)
    assert len(np.unique(ref)) == 5                      # every phase occurs in the synthetic traces
    both(pcm, a, ragged_n_chunks(cfg), cfg.L, cfg.D)


def test_degenerate_shapes_thresholds_and_other_dimension(pcm):
    cfg = CONFIGS["cfg1"].with_(n_groups=9)              # T = 72: a ragged last workgroup
    a = make_gripper_actions(cfg, 3)
    both(pcm, a, None, cfg.L, cfg.D, close_threshold=0.5)
    both(pcm, a, None, cfg.L, cfg.D, close_threshold=2.0)                  # command never active: all approach
    both(pcm, a, None, cfg.L, cfg.D, close_threshold=-2.0)                 # always active: all active-grip
    both(pcm, a, None, cfg.L, cfg.D, gripper_dim=0)                        # a noise dimension as the gripper
    both(pcm, a, np.zeros(cfg.T, np.int32), cfg.L, cfg.D)                  # no valid chunk anywhere
    # one chunk per trajectory, one timestep per chunk, one value per timestep
    one = np.array([[[1.0]], [[-1.0]]], dtype=np.float32)
    assert list(both(pcm, one, None, 1, 1).reshape(-1)) == [O.PHASE_ACTIVE_GRIP, O.PHASE_APPROACH]
    # long trajectories (several chunks per lane), L = 20 so that 0.1 / 0.5 / 0.75 are hit exactly
    rng = np.random.default_rng(5)
    N, L, D = 4096, 20, 3
    counts = rng.choice([0, 1, 2, 9, 10, 14, 15, 20], size=(3, N), p=[0.3, 0.1, 0.1, 0.1, 0.1, 0.1, 0.1, 0.1])
    act = -np.ones((3, N, L, D), dtype=np.float32)
    for i in range(3):
        for j in range(N):
            act[i, j, :counts[i, j], D - 1] = 1.0
    both(pcm, act.reshape(3, N, L * D), np.array([N, 1000, 37], np.int32), L, D)


def test_bad_arguments_are_rejected(pcm):
    a = torch.zeros((2, 4, 6), device="cuda")
    with pytest.raises(pcm.PcmError):
        pcm.pcm_label_phases(a, None, 3, 2, gripper_dim=2)
    with pytest.raises(pcm.PcmError):
        pcm.pcm_label_phases(a, None, 4, 2)
