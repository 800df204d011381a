"""GPU parity of the selection stage against the CPU checker, through the C-ABI: bit-exact.

Covers Eq. 1 / Eq. 5 (pcm_score_phases), Eq. 7-9 (pcm_update_keep_probs), Eq. 10 and the
compaction (pcm_sample_chunks), separately on checker-produced inputs and chained over steps.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pcm_oracle as O
from workloads import CONFIGS, make_rollouts, ragged_n_chunks

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pcm():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_16154_amd as pcm
    pcm.lib()
    return pcm


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def bits(x):
    return np.ascontiguousarray(x).view(np.int64)


def _score_both(pcm, cfg, ro, reward=None, n_chunks=None):
    reward = ro["reward"] if reward is None else reward
    n_chunks_np = ro["n_chunks"] if n_chunks is None else n_chunks
    adv_o, act_o = O.advantages(reward, cfg.G)
    C_o, valid_o = O.phase_scores(ro["actions"], ro["phase"], reward, n_chunks_np, cfg.n_groups, cfg.G, cfg.K)
    C, valid, adv, act = pcm.pcm_score_phases(dev(ro["actions"]), dev(ro["phase"]), dev(reward), dev(n_chunks_np),
                                              cfg.n_groups, cfg.G, cfg.K, 1e-6)
    torch.cuda.synchronize()
    return (C_o, valid_o, adv_o, act_o), (C.cpu().numpy(), valid.cpu().numpy(), adv.cpu().numpy(), act.cpu().numpy())


@pytest.mark.parametrize("name,steps", [("cfg1", 3), ("cfg2", 3), ("cfg4", 1), ("cfg5", 1)])
def test_score_phases_bit_exact(pcm, name, steps):
    cfg = CONFIGS[name]
    for step in range(steps):
        ro = make_rollouts(cfg, step)
        (C_o, valid_o, adv_o, act_o), (C, valid, adv, act) = _score_both(pcm, cfg, ro)
        assert np.array_equal(bits(C), bits(C_o)), (name, step, C, C_o)
        assert np.array_equal(valid, valid_o)
        assert np.array_equal(adv.view(np.int32), adv_o.astype(np.float32).view(np.int32))
        assert np.array_equal(act, act_o)


def test_score_phases_ragged_collapsed_and_null_n_chunks(pcm):
    cfg = CONFIGS["cfg2"].with_(seed=21)
    ro = make_rollouts(cfg, 0)
    reward = ro["reward"].copy()
    reward[8:16] = 0                      # one collapsed group
    reward[24:32] = 1                     # another
    n = ragged_n_chunks(cfg)
    (C_o, valid_o, adv_o, act_o), (C, valid, adv, act) = _score_both(pcm, cfg, ro, reward, n)
    assert np.array_equal(bits(C), bits(C_o)) and np.array_equal(valid, valid_o)
    assert np.array_equal(act, act_o) and not act[8:16].any() and not adv[24:32].any()
    # NULL n_chunks means every slot is valid
    C2, valid2, _, _ = pcm.pcm_score_phases(dev(ro["actions"]), dev(ro["phase"]), dev(reward), None,
                                            cfg.n_groups, cfg.G, cfg.K, 1e-6)
    C2_o, valid2_o = O.phase_scores(ro["actions"], ro["phase"], reward, None, cfg.n_groups, cfg.G, cfg.K)
    assert np.array_equal(bits(C2.cpu().numpy()), bits(C2_o)) and np.array_equal(valid2.cpu().numpy(), valid2_o)


def test_score_phases_degenerate_shapes(pcm):
    # every group collapsed: nothing valid; A not a multiple of 4 (scalar load path); K = 1; N = 1
    rng = np.random.default_rng(0)
    # ... the largest K with the widest chunk (the phases are pooled in several blocks); a large group;
    # many groups (one slice each); ragged trajectories over several slices
    for (n_groups, G, N, A, K) in [(3, 4, 5, 7, 1), (2, 2, 1, 56, 3), (5, 3, 17, 13, 6), (1, 8, 700, 56, 4),
                                   (2, 3, 40, 256, 64), (3, 40, 9, 56, 5), (2500, 2, 3, 8, 2), (4, 8, 130, 56, 9)]:
        T = n_groups * G
        actions = rng.uniform(-1, 1, size=(T, N, A)).astype(np.float32)
        phase = rng.integers(0, K, size=(T, N)).astype(np.uint8)
        reward = rng.integers(0, 2, size=T).astype(np.uint8)
        n_chunks = rng.integers(0, N + 1, size=T).astype(np.int32) if K == 9 else None
        C_o, valid_o = O.phase_scores(actions, phase, reward, n_chunks, n_groups, G, K)
        C, valid, adv, act = pcm.pcm_score_phases(dev(actions), dev(phase), dev(reward),
                                                  None if n_chunks is None else dev(n_chunks), n_groups, G, K, 1e-6)
        assert np.array_equal(bits(C.cpu().numpy()), bits(C_o)), (n_groups, G, N, A, K)
        assert np.array_equal(valid.cpu().numpy(), valid_o)
    T = 8
    C, valid, adv, act = pcm.pcm_score_phases(dev(np.ones((T, 4, 56), np.float32)), dev(np.zeros((T, 4), np.uint8)),
                                              dev(np.ones(T, np.uint8)), None, 1, 8, 3, 1e-6)
    assert not valid.cpu().numpy().any() and not C.cpu().numpy().any() and not act.cpu().numpy().any()


def test_phase_ids_beyond_the_last_phase_follow_one_rule(pcm):
    # ids >= K count as phase K - 1 in the score and in the sampler (and in the N_c / b_c weights)
    cfg = CONFIGS["cfg2"]
    ro = make_rollouts(cfg, 1)
    K = cfg.K - 2                                               # the batch holds ids up to K + 1
    phase = ro["phase"].copy()
    phase[::3, ::5] = 200                                       # and some far out of range
    C_o, valid_o = O.phase_scores(ro["actions"], phase, ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, K)
    C, valid, adv, act = pcm.pcm_score_phases(dev(ro["actions"]), dev(phase), dev(ro["reward"]), dev(ro["n_chunks"]),
                                              cfg.n_groups, cfg.G, K, 1e-6)
    assert np.array_equal(bits(C.cpu().numpy()), bits(C_o)) and np.array_equal(valid.cpu().numpy(), valid_o)
    assert valid_o[K - 1]                                       # the last phase did collect the strays
    _sample_both(pcm, np.array([0.2, 1.0, 0.45]), phase, ro["n_chunks"], act.cpu().numpy(), cfg.B, seed=3, step=8,
                 weights=True)


def test_keep_probs_chain_bit_exact(pcm):
    rng = np.random.default_rng(5)
    K = 7
    state = pcm.pcm_state_init(K, "cuda")
    ref = O.KeepProbState(K)
    for t in range(13):
        C = rng.uniform(0, 4, size=K)
        valid = (rng.random(K) < 0.8).astype(np.uint8)
        if t == 7:
            valid[:] = 0
        p = pcm.pcm_update_keep_probs(state, dev(C), dev(valid), 0.1, 5)
        p_o = ref.update(C, valid, 0.1, 5)
        assert np.array_equal(bits(p.cpu().numpy()), bits(p_o)), t
    words = state.cpu().numpy()
    assert words[0] == 13 and words[1] == ref.since        # step counter, steps since refresh
    # all-zero scores on the first step: floor everywhere
    state = pcm.pcm_state_init(3, "cuda")
    p = pcm.pcm_update_keep_probs(state, dev(np.zeros(3)), dev(np.ones(3, np.uint8)), 0.25, 5)
    assert np.array_equal(p.cpu().numpy(), [0.25, 0.25, 0.25])


def _sample_both(pcm, p, phase, n_chunks, active, B, seed, step, selector="pcm", weights=False):
    kept_o, off_o, nk_o = O.sample_chunks(p, phase, n_chunks, active, B, seed, step, selector=selector)
    d_nch = None if n_chunks is None else dev(n_chunks)
    kept, off, nk = pcm.pcm_sample_chunks(dev(p), dev(phase), d_nch, None if active is None else dev(active), B, seed,
                                          step, selector=selector)
    torch.cuda.synchronize()
    assert int(nk.item()) == nk_o
    assert np.array_equal(off.cpu().numpy(), off_o)
    assert np.array_equal(kept.cpu().numpy()[:nk_o], kept_o)
    # realised allocation per phase (Sec. 5.2): exact counts
    d_act = None if active is None else dev(active)
    got_kept, got_elig = pcm.pcm_kept_phase_counts(dev(phase), d_nch, d_act, kept, nk, len(p))
    ref_kept, ref_elig = O.kept_phase_counts(phase, n_chunks, active, kept_o, len(p))
    assert np.array_equal(got_kept.cpu().numpy(), ref_kept) and np.array_equal(got_elig.cpu().numpy(), ref_elig)
    if weights:
        w = pcm.pcm_importance_weights(dev(phase), d_nch, kept, off, len(p))
        torch.cuda.synchronize()
        ref = O.importance_weights(phase, n_chunks, kept_o, len(p))
        assert np.array_equal(w.cpu().numpy()[:nk_o].view(np.int32), ref.view(np.int32))   # bit for bit
    return kept_o, off_o


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_sample_chunks_bit_exact(pcm, name):
    cfg = CONFIGS[name]
    ro = make_rollouts(cfg, 0)
    rng = np.random.default_rng(cfg.seed)
    p = np.maximum(0.1, rng.random(cfg.K))
    p[rng.integers(0, cfg.K)] = 1.0
    _, active = O.advantages(ro["reward"], cfg.G)
    _sample_both(pcm, p, ro["phase"], ro["n_chunks"], active, cfg.B, seed=cfg.seed, step=3)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4", "cfg5"])
@pytest.mark.parametrize("selector", ["random", "top_phase", "stratified"])
def test_ablation_selectors_bit_exact(pcm, name, selector):
    cfg = CONFIGS[name]
    ro = make_rollouts(cfg, 0)
    rng = np.random.default_rng(cfg.seed + 17)
    p = np.maximum(0.1, rng.random(cfg.K))
    p[rng.integers(0, cfg.K)] = 1.0
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, off = _sample_both(pcm, p, ro["phase"], ro["n_chunks"], active, cfg.B, seed=cfg.seed, step=5, selector=selector)
    if selector == "top_phase":
        assert np.all(ro["phase"].reshape(-1)[kept] == int(np.argmax(p)))


def test_ablation_selectors_edge_cases(pcm):
    cfg = CONFIGS["cfg1"].with_(n_groups=9)
    ro = make_rollouts(cfg, 1)
    n = ragged_n_chunks(cfg)
    active = (np.arange(cfg.T) % 5 != 0).astype(np.uint8)
    p_tie = np.array([0.4, 1.0, 1.0, 0.1])                     # tie: the lower index wins
    for selector in ("random", "top_phase", "stratified"):
        _sample_both(pcm, p_tie, ro["phase"], n, active, cfg.B, seed=2 ** 40 + 7, step=2 ** 33 + 1, selector=selector)
        _sample_both(pcm, p_tie, ro["phase"], n, None, cfg.N + 5, seed=1, step=0, selector=selector)
        _sample_both(pcm, p_tie, ro["phase"], None, np.zeros(cfg.T, np.uint8), cfg.B, seed=1, step=0, selector=selector)
    # a top phase that no trajectory contains: nothing is kept
    p_none = np.array([0.1, 0.1, 0.1, 0.1, 1.0])
    kept, off = _sample_both(pcm, p_none, np.minimum(ro["phase"], 3), None, None, cfg.B, 1, 0, selector="top_phase")
    assert len(kept) == 0
    rng = np.random.default_rng(2)
    for N, B in [(100, 17), (4096, 64), (3000, 5)]:
        phase = np.sort(rng.integers(0, 9, size=(6, N)), axis=1).astype(np.uint8)
        pk = np.maximum(0.1, rng.random(9))
        nn = rng.integers(0, N + 1, size=6).astype(np.int32)
        for selector in ("random", "top_phase", "stratified"):
            _sample_both(pcm, pk, phase, nn, None, B, seed=N, step=B, selector=selector)
    # stratified budgets with caps that bind (a heavy phase with few chunks), many phases, more than 64 draws
    phase = np.sort(rng.integers(0, 40, size=(5, 700)), axis=1).astype(np.uint8)
    phase[:, :3] = 0
    phase[:, 3:] = np.maximum(phase[:, 3:], 1)
    pk = np.full(40, 0.1)
    pk[0] = 1.0
    _sample_both(pcm, pk, phase, None, None, 150, seed=9, step=4, selector="stratified", weights=True)
    _sample_both(pcm, pk, phase[:, :7].copy(), None, None, 5, seed=9, step=4, selector="stratified", weights=True)   # N < K


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4", "cfg5"])
def test_importance_weights_bit_exact(pcm, name):
    cfg = CONFIGS[name]
    ro = make_rollouts(cfg, 0)
    rng = np.random.default_rng(cfg.seed + 3)
    p = np.maximum(0.1, rng.random(cfg.K))
    _, active = O.advantages(ro["reward"], cfg.G)
    _sample_both(pcm, p, ro["phase"], ro["n_chunks"], active, cfg.B, seed=cfg.seed, step=1, weights=True)
    if name == "cfg1":
        n = ragged_n_chunks(cfg)
        _sample_both(pcm, p, ro["phase"], n, None, cfg.B, seed=3, step=1, weights=True)
        _sample_both(pcm, p, ro["phase"], n, None, cfg.B, seed=3, step=1, selector="top_phase", weights=True)


def test_sample_chunks_edge_cases(pcm):
    cfg = CONFIGS["cfg1"].with_(n_groups=9)              # T = 72: several workgroups and a ragged tail
    ro = make_rollouts(cfg, 1)
    p = np.array([1.0, 0.1, 0.37, 0.1])
    n = ragged_n_chunks(cfg)
    active = (np.arange(cfg.T) % 5 != 0).astype(np.uint8)
    _sample_both(pcm, p, ro["phase"], n, active, cfg.B, seed=2 ** 40 + 7, step=2 ** 33 + 1)   # 64-bit seed and step
    _sample_both(pcm, p, ro["phase"], n, None, cfg.N + 5, seed=1, step=0)                     # B >= N keeps all
    _sample_both(pcm, p, ro["phase"], None, np.zeros(cfg.T, np.uint8), cfg.B, seed=1, step=0)  # nothing active
    _sample_both(pcm, p, ro["phase"], None, None, 1, seed=1, step=0)                          # B = 1
    # long trajectories: several chunk slots per lane, N not a multiple of 64
    rng = np.random.default_rng(1)
    for N, B in [(100, 17), (1000, 40), (4096, 64), (3000, 5)]:
        phase = np.sort(rng.integers(0, 9, size=(6, N)), axis=1).astype(np.uint8)
        pk = np.maximum(0.1, rng.random(9))
        nn = rng.integers(0, N + 1, size=6).astype(np.int32)
        _sample_both(pcm, pk, phase, nn, None, B, seed=N, step=B)
    # many short trajectories: the offsets scan runs over several trajectories per thread, with a ragged last run
    T, N = 3001, 5
    phase = rng.integers(0, 3, size=(T, N)).astype(np.uint8)
    nn = rng.integers(0, N + 1, size=T).astype(np.int32)
    act = (rng.random(T) < 0.7).astype(np.uint8)
    for selector in ("pcm", "top_phase"):
        _sample_both(pcm, np.array([0.2, 1.0, 0.5]), phase, nn, act, 2, seed=5, step=6, selector=selector)


def test_ten_chained_steps_bit_exact(pcm):
    """All three selection calls back to back for 10 steps, GPU feeding GPU and checker feeding checker."""
    cfg = CONFIGS["cfg2"]
    state = pcm.pcm_state_init(cfg.K, "cuda")
    ref = O.KeepProbState(cfg.K)
    refreshed = []
    for step in range(cfg.n_steps):
        ro = make_rollouts(cfg, step)
        adv_o, act_o = O.advantages(ro["reward"], cfg.G)
        C_o, valid_o = O.phase_scores(ro["actions"], ro["phase"], ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, cfg.K)
        p_o = ref.update(C_o, valid_o, 0.1, 5)
        kept_o, off_o, nk_o = O.sample_chunks(p_o, ro["phase"], ro["n_chunks"], act_o, cfg.B, cfg.seed, step)

        phase, n_chunks = dev(ro["phase"]), dev(ro["n_chunks"])
        C, valid, adv, act = pcm.pcm_score_phases(dev(ro["actions"]), phase, dev(ro["reward"]), n_chunks,
                                                  cfg.n_groups, cfg.G, cfg.K, 1e-6)
        p = pcm.pcm_update_keep_probs(state, C, valid, 0.1, 5)
        kept, off, nk = pcm.pcm_sample_chunks(p, phase, n_chunks, act, cfg.B, cfg.seed, step)
        torch.cuda.synchronize()
        assert np.array_equal(bits(p.cpu().numpy()), bits(p_o)), step
        assert int(nk.item()) == nk_o == cfg.T * cfg.B
        assert np.array_equal(kept.cpu().numpy(), kept_o), step
        refreshed.append(p_o.copy())
    # refresh at t = 0 and t = 5 only
    assert all(np.array_equal(refreshed[t], refreshed[0]) for t in range(5))
    assert all(np.array_equal(refreshed[t], refreshed[5]) for t in range(5, 10))
    assert not np.array_equal(refreshed[0], refreshed[5])
