"""Pins of the checker's gripper-based phase labeler (App. D, phase allotment rules): traces labelled by hand,
one for each rule, each threshold and each overlap of windows that the priority order resolves."""
import numpy as np

from oracle import pcm_oracle as O

AP, PG, AG, RR, TL = O.PHASE_APPROACH, O.PHASE_PRE_GRASP, O.PHASE_ACTIVE_GRIP, O.PHASE_RELEASE_RAMP, O.PHASE_TAIL
L, D = 20, 2          # 20 timesteps per chunk so that g_f = 0.05, 0.1, 0.45, 0.5, 0.75 are all exact counts


def trace(fractions):
    """One trajectory whose chunk j has round(f * L) close timesteps (gripper = last dimension)."""
    N = len(fractions)
    a = -np.ones((1, N, L * D), dtype=np.float32)
    for j, f in enumerate(fractions):
        n = int(round(f * L))
        steps = np.arange(L)[::-1][:n] if j % 2 else np.arange(L)[:n]       # where in the chunk does not matter
        a[0, j, steps * D + (D - 1)] = 1.0
    return a


def labels(fractions, n_chunks=None):
    return list(O.label_phases(trace(fractions), n_chunks, L, D)[0])


def test_one_grasp_cycle_every_phase():
    #        approach      pre-grasp window        grasp interval     release window     tail
    f = [0.0, 0.05, 0.3,   0.2, 0.1, 0.45,         0.8, 1.0, 0.75,    0.4, 0.0, 0.2,     0.0, 0.05]
    want = [AP, AP, AP,    PG, PG, PG,             AG, AG, AG,        RR, RR, RR,        TL, TL]
    assert labels(f) == want


def test_thresholds_are_inclusive_where_the_rules_say_so():
    # 0.75 is sustained, 0.7 is not (but still active-grip); 0.5 is active-grip, 0.45 is not
    assert labels([0.0, 0.7, 0.0]) == [AP, AG, AP]                 # no sustained interval: nothing to approach, all approach
    assert labels([0.0, 0.75, 0.0]) == [AP, AG, RR]
    assert labels([0.45, 0.8]) == [PG, AG] and labels([0.5, 0.8]) == [AG, AG]
    # pre-grasp needs g_f >= 0.1: an open chunk inside the window stays approach
    assert labels([0.05, 0.1, 0.05, 0.9]) == [AP, PG, AP, AG]


def test_windows_are_three_chunks_wide_and_checked_chunk_by_chunk():
    f = [0.2, 0.2, 0.2, 0.2, 0.2, 0.9, 0.2, 0.2, 0.2, 0.2, 0.2]
    assert labels(f) == [AP, AP, PG, PG, PG, AG, RR, RR, RR, TL, TL]
    # a chunk that fails its threshold does not close the window for the chunks further out
    assert labels([0.2, 0.0, 0.2, 0.9]) == [PG, AP, PG, AG]


def test_priority_where_windows_of_two_grasps_overlap():
    # two chunks between two grasp intervals: both the release window of the first and the pre-grasp window
    # of the second; pre-grasp wins when the gripper has begun closing, release-ramp otherwise
    f = [0.9, 0.3, 0.0, 0.9, 0.0]
    assert labels(f) == [AG, PG, RR, AG, RR]
    # further apart: release window, then approach to the next grasp, then its pre-grasp window
    f = [0.9, 0.0, 0.0, 0.0, 0.0, 0.0, 0.2, 0.2, 0.9, 0.0, 0.0, 0.0, 0.0]
    assert labels(f) == [AG, RR, RR, RR, AP, AP, PG, PG, AG, RR, RR, RR, TL]
    # an isolated half-closed chunk after the last grasp is active-grip (re-grasp attempt), its neighbours tail
    f = [0.9, 0.0, 0.0, 0.0, 0.0, 0.6, 0.0]
    assert labels(f) == [AG, RR, RR, RR, TL, AG, TL]


def test_no_grasp_ragged_and_other_gripper_dimension():
    assert labels([0.0, 0.3, 0.05, 0.6, 0.0]) == [AP, AP, AP, AG, AP]
    # chunks beyond n_chunks do not exist: the grasp at slot 3 is not seen, slots >= 3 are left 0
    assert labels([0.2, 0.2, 0.2, 0.9, 0.0], n_chunks=np.array([3])) == [AP, AP, AP, 0, 0]
    assert labels([0.2, 0.9], n_chunks=np.array([0])) == [0, 0]
    # gripper in another dimension and a different command threshold
    a = trace([0.0, 0.3, 0.9, 0.0])
    b = np.zeros_like(a)
    b[..., 0::D] = a[..., (D - 1)::D] * 0.5 + 0.25        # close = 0.75, open = -0.25, in dimension 0
    assert list(O.label_phases(b, None, L, D, gripper_dim=0, close_threshold=0.5)[0]) == [AP, PG, AG, RR]
    assert list(O.label_phases(b, None, L, D, gripper_dim=0, close_threshold=0.8)[0]) == [AP, AP, AP, AP]
