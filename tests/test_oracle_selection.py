"""Pins for the CPU checker's selection stage (Eq. 1, 5, 7-10 of the paper).

Each test compares the checker with something it did not compute itself: a closed
form, the plain textbook definition, published generator vectors, a hand-worked
example or brute-force enumeration.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import pcm_oracle as O
from workloads import CONFIGS, make_rollouts, ragged_n_chunks


# ---------------------------------------------------------------- Eq. 1 advantages

@pytest.mark.parametrize("G,s", [(8, 4), (8, 2), (8, 7), (10, 3), (10, 1)])
def test_advantage_closed_form(G, s):
    # binary rewards with s successes: mu = s/G, sigma = sqrt(mu(1-mu))
    reward = np.array([1] * s + [0] * (G - s), dtype=np.uint8)
    eps = 1e-6
    adv, active = O.advantages(reward, G, eps)
    mu = s / G
    sigma = math.sqrt(mu * (1 - mu))
    assert np.allclose(adv[:s], (1 - mu) / (sigma + eps), rtol=1e-15, atol=0)
    assert np.allclose(adv[s:], -mu / (sigma + eps), rtol=1e-15, atol=0)
    assert abs(adv.sum()) < 1e-12                     # zero mean within the group (App. B, Lemma 1 proof)
    assert active.all()


def test_advantage_limits_eps_to_zero():
    # eps -> 0: +sqrt((1-mu)/mu) and -sqrt(mu/(1-mu)); G=8, s=4 gives +-1; s=2 gives sqrt(3), -1/sqrt(3)
    adv, _ = O.advantages(np.array([1, 1, 1, 1, 0, 0, 0, 0]), 8, eps=0.0)
    assert np.array_equal(adv, [1, 1, 1, 1, -1, -1, -1, -1])
    adv, _ = O.advantages(np.array([1, 1, 0, 0, 0, 0, 0, 0]), 8, eps=0.0)
    assert np.allclose(adv[:2], math.sqrt(3), rtol=1e-15)
    assert np.allclose(adv[2:], -1 / math.sqrt(3), rtol=1e-15)


def test_advantage_collapsed_groups_are_zero():
    reward = np.array([1] * 8 + [0] * 8 + [1, 0] * 4, dtype=np.uint8)
    adv, active = O.advantages(reward, 8)
    assert np.array_equal(adv[:16], np.zeros(16))
    assert np.array_equal(active, [0] * 16 + [1] * 8)


# ---------------------------------------------------------------- Eq. 5 phase score

def _plain_score(actions, phase, reward, n_chunks, n_groups, G, K):
    """Eq. 5 written directly with conditional means in fp64 (no integer convention)."""
    T, N, A = actions.shape
    tot = np.zeros(K)
    cnt = np.zeros(K, dtype=int)
    valid_chunk = np.arange(N)[None, :] < n_chunks[:, None]
    for g in range(n_groups):
        sl = slice(g * G, (g + 1) * G)
        r = reward[sl].astype(bool)
        if r.all() or (~r).all():
            continue
        a, ph, vc = actions[sl].astype(np.float64), phase[sl], valid_chunk[sl]
        for c in range(K):
            pos = a[(ph == c) & vc & r[:, None]]
            neg = a[(ph == c) & vc & ~r[:, None]]
            if len(pos) == 0 or len(neg) == 0:
                continue
            tot[c] += np.linalg.norm(pos.mean(0) - neg.mean(0))
            cnt[c] += 1
    return np.where(cnt > 0, tot / np.maximum(cnt, 1), 0.0), (cnt > 0).astype(np.uint8)


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_phase_score_matches_plain_definition(name):
    cfg = CONFIGS[name]
    ro = make_rollouts(cfg, step=0)
    C, valid = O.phase_scores(ro["actions"], ro["phase"], ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, cfg.K)
    C_ref, valid_ref = _plain_score(ro["actions"], ro["phase"], ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, cfg.K)
    assert np.array_equal(valid, valid_ref)
    # the 2^-24 action grid perturbs each mean by at most 2^-25
    assert np.allclose(C, C_ref, rtol=0, atol=math.sqrt(cfg.A) * 2.0 ** -24)


def test_phase_score_ragged_and_collapsed_matches_plain_definition():
    cfg = CONFIGS["cfg1"].with_(n_groups=5, seed=11)
    ro = make_rollouts(cfg, step=3)
    reward = ro["reward"].copy()
    reward[8:16] = 1                                     # a collapsed group is ignored (Sec. 4.1)
    n_chunks = ragged_n_chunks(cfg)
    C, valid = O.phase_scores(ro["actions"], ro["phase"], reward, n_chunks, cfg.n_groups, cfg.G, cfg.K)
    C_ref, valid_ref = _plain_score(ro["actions"], ro["phase"], reward, n_chunks, cfg.n_groups, cfg.G, cfg.K)
    assert np.array_equal(valid, valid_ref)
    assert np.allclose(C, C_ref, rtol=0, atol=1e-6)


def test_phase_score_planted_gap():
    # a mean gap delta in every dim of one phase and none elsewhere: C -> delta*sqrt(A) there,
    # noise floor sigma*sqrt(A(1/n+ + 1/n-)) elsewhere
    rng = np.random.default_rng(0)
    G, N, A, K, delta, sigma = 8, 64, 56, 4, 0.5, 0.05
    phase = np.repeat(np.arange(K, dtype=np.uint8), N // K)[None, :].repeat(G, 0)
    reward = np.array([1, 0] * (G // 2), dtype=np.uint8)
    actions = (sigma * rng.standard_normal((G, N, A))).astype(np.float32)
    actions[reward == 1, 16:32] += np.float32(delta / 2)
    actions[reward == 0, 16:32] -= np.float32(delta / 2)
    C, valid = O.phase_scores(actions, phase, reward, None, 1, G, K)
    assert valid.all()
    assert abs(C[1] - delta * math.sqrt(A)) < 0.05
    floor = sigma * math.sqrt(A * (2.0 / (G // 2 * N // K)))
    for c in (0, 2, 3):
        assert C[c] < 3 * floor


def test_phase_score_hand_example():
    # one group of two trajectories, two chunks each, A = 2; phase 0 = first chunk, phase 1 = second
    actions = np.array([[[0.5, 0.25], [0.0, 0.0]],       # success
                        [[-0.5, 0.25], [0.75, -1.0]]],   # failure
                       dtype=np.float32)
    phase = np.array([[0, 1], [0, 1]], dtype=np.uint8)
    reward = np.array([1, 0], dtype=np.uint8)
    C, valid = O.phase_scores(actions, phase, reward, None, 1, 2, 3)
    assert np.array_equal(valid, [1, 1, 0])
    assert C[0] == 1.0                                   # |(0.5,0.25)-(-0.5,0.25)| = 1
    assert C[1] == 1.25                                  # |(0,0)-(0.75,-1)| = 1.25
    assert C[2] == 0.0


def test_phase_score_symmetries():
    cfg = CONFIGS["cfg1"]
    ro = make_rollouts(cfg, step=1)
    args = (ro["phase"], ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, cfg.K)
    C, valid = O.phase_scores(ro["actions"], *args)
    # swapping the outcome labels leaves the norm unchanged
    C_sw, valid_sw = O.phase_scores(ro["actions"], ro["phase"], 1 - ro["reward"], *args[2:])
    assert np.array_equal(C, C_sw) and np.array_equal(valid, valid_sw)
    # translating every action by a constant on the integer grid leaves it unchanged
    C_tr, _ = O.phase_scores(ro["actions"] * np.float32(0.5) + np.float32(0.25), *args)
    C_half, _ = O.phase_scores(ro["actions"] * np.float32(0.5), *args)
    assert np.allclose(C_tr, C_half, rtol=0, atol=1e-6)
    # scaling by alpha scales the score by |alpha| (exact for a power of two away from the grid's floor)
    assert np.allclose(C_half, 0.5 * C, rtol=0, atol=1e-6)


def test_phase_absent_from_one_outcome_is_skipped():
    # App. D.2: a phase present only in successes (or only in failures) is skipped for that update
    actions = np.ones((2, 2, 1), dtype=np.float32)
    phase = np.array([[0, 1], [0, 0]], dtype=np.uint8)    # phase 1 only in the successful rollout
    C, valid = O.phase_scores(actions, phase, np.array([1, 0], dtype=np.uint8), None, 1, 2, 2)
    assert np.array_equal(valid, [1, 0]) and C[1] == 0.0


def test_phase_ids_beyond_the_last_phase_count_as_the_last():
    # One rule for input outside the labelling's range, in the score and in the sampler alike: an id >= K is
    # read as K - 1.  Pinned by relabelling the input by hand and calling the functions on in-range labels.
    cfg = CONFIGS["cfg1"]
    ro = make_rollouts(cfg, 2)
    K = cfg.K - 1                                               # the batch holds ids 0 .. K, one more than announced
    assert ro["phase"].max() == K
    relabelled = np.minimum(ro["phase"], K - 1)
    args = (ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, K)
    C, valid = O.phase_scores(ro["actions"], ro["phase"], *args)
    C_ref, valid_ref = O.phase_scores(ro["actions"], relabelled, *args)
    assert np.array_equal(C, C_ref) and np.array_equal(valid, valid_ref)
    p = np.array([1.0, 0.3, 0.6])
    got = O.sample_chunks(p, ro["phase"], ro["n_chunks"], None, cfg.B, 5, 1)
    want = O.sample_chunks(p, relabelled, ro["n_chunks"], None, cfg.B, 5, 1)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


# ---------------------------------------------------------------- Eq. 7-9 keep probabilities

def _read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[line[0]] = [float(x) for x in line[1:]]
    return out


def test_keep_probs_hand_worked(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "keep_probs_worked.txt"))
    st = O.KeepProbState(4)
    p = st.update(np.array(g["C"]), np.ones(4, dtype=np.uint8), p_min=g["p_min"][0], T_rc=5)
    assert np.array_equal(p, g["p"])


def test_keep_probs_eq8_through_shares():
    # Eq. 8 as printed: rho_c = S_c / sum S, rho~_c = rho_c / max rho; must agree with S_c / max S
    rng = np.random.default_rng(3)
    for _ in range(50):
        C = rng.uniform(0, 5, size=6)
        st = O.KeepProbState(6)
        p = st.update(C, np.ones(6, dtype=np.uint8), p_min=0.1, T_rc=5)
        rho = C / C.sum()
        assert np.allclose(st.shares, rho, rtol=1e-15)
        assert np.allclose(p, np.maximum(0.1, rho / rho.max()), rtol=4e-16, atol=0)
        assert p.max() == 1.0 and p.min() >= 0.1        # max_c rho~ = 1; p in [p_min, 1]


def test_keep_probs_scale_invariance_and_schedule():
    # Sec. 4.3: share normalisation is scale-invariant; refresh at t = 0, then every T_rc steps;
    # p is held fixed in between (Sec. 4.4)
    rng = np.random.default_rng(4)
    Cs = rng.uniform(0.1, 3, size=(12, 5))
    a, b = O.KeepProbState(5), O.KeepProbState(5)
    hist = []
    for t in range(12):
        pa = a.update(Cs[t], np.ones(5, dtype=np.uint8), 0.1, 5)
        pb = b.update(Cs[t] * 8.0, np.ones(5, dtype=np.uint8), 0.1, 5)
        assert np.array_equal(pa, pb)
        hist.append(pa)
    first = np.maximum(0.1, Cs[0] / Cs[0].max())
    for t in range(0, 5):
        assert np.allclose(hist[t], first, rtol=4e-16)
    S = Cs[1:6].sum(0)
    for t in range(5, 10):
        assert np.allclose(hist[t], np.maximum(0.1, S / S.max()), rtol=1e-15)
    S = Cs[6:11].sum(0)
    assert np.allclose(hist[10], np.maximum(0.1, S / S.max()), rtol=1e-15)
    assert np.array_equal(hist[10], hist[11])


def test_keep_probs_skipped_phase_and_all_zero():
    st = O.KeepProbState(3)
    p = st.update(np.array([2.0, 9.9, 1.0]), np.array([1, 0, 1], dtype=np.uint8), 0.1, 5)
    assert np.array_equal(p, [1.0, 0.1, 0.5])             # invalid phase contributes no entry
    st = O.KeepProbState(3)
    p = st.update(np.zeros(3), np.zeros(3, dtype=np.uint8), 0.1, 5)
    assert np.array_equal(p, [0.1, 0.1, 0.1])             # nothing valid: floor everywhere


# ---------------------------------------------------------------- RNG

def test_philox_known_answers(golden_dir):
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert list(O.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_rng64_packs_words_and_uses_all_inputs():
    base = O.rng64(1, 2, 3, 4)
    w = O.philox4x32_10((3, 4, 2, 0), (1, 0))
    assert base == w[0] | (w[1] << 32)
    assert len({base, O.rng64(2, 2, 3, 4), O.rng64(1, 3, 3, 4), O.rng64(1, 2, 4, 4), O.rng64(1, 2, 3, 5),
                O.rng64(1 + (1 << 32), 2, 3, 4), O.rng64(1, 2 + (1 << 32), 3, 4)}) == 7


# ---------------------------------------------------------------- Eq. 10 sampler

def _pl_inclusion(weights, m):
    """Exact inclusion probabilities of successive weighted sampling w/o replacement, by enumeration."""
    n = len(weights)
    W = sum(weights)
    incl = [Fraction(0)] * n
    for tup in itertools.permutations(range(n), m):
        pr, rem = Fraction(1), W
        for k in tup:
            pr *= Fraction(weights[k], rem)
            rem -= weights[k]
        for k in tup:
            incl[k] += pr
    return incl


@pytest.mark.parametrize("weights,m", [([3, 1, 2, 6], 2), ([10, 1, 1, 1, 5], 3), ([1, 1, 1, 1, 1, 1], 2),
                                       ([6554, 65536, 32768, 6554], 1)])
def test_sampler_inclusion_matches_enumeration(weights, m):
    exact = _pl_inclusion(weights, m)
    assert sum(exact) == m
    trials = 40000
    hits = np.zeros(len(weights))
    for s in range(trials):
        picks = O.sample_trajectory(weights, m, seed=s % 200, step=s // 200, traj=7)
        assert len(set(picks)) == m
        hits[picks] += 1
    for k, pk in enumerate(exact):
        pk = float(pk)
        sd = math.sqrt(pk * (1 - pk) / trials)
        assert abs(hits[k] / trials - pk) < 4 * sd + 1e-12, (k, hits[k] / trials, pk)


def test_sampler_first_draw_is_inverse_cdf():
    # m = 1: index k is picked iff floor(x W / 2^64) lands in k's weight interval
    w = [5, 0, 7, 1]
    for s in range(200):
        x = O.rng64(s, 0, 0, 0)
        t = (x * sum(w)) >> 64
        expect = 0 if t < 5 else (2 if t < 12 else 3)
        assert O.sample_trajectory(w, 1, s, 0, 0) == [expect]


def test_weight_quantisation():
    q = O.quantise_keep_probs(np.array([1.0, 0.5, 0.1, 0.0, 2.0, float("nan"), 1e-9]))
    assert list(q) == [65536, 32768, 6554, 1, 65536, 1, 1]


def test_sample_chunks_set_properties_and_budget_fractions(golden_dir):
    consts = _read_golden(os.path.join(golden_dir, "paper_constants.txt"))
    cfg = CONFIGS["cfg2"]
    ro = make_rollouts(cfg, 0)
    p = np.array([1.0, 0.5, 0.1, 0.1, 0.3])
    for B in (8, 12, 16):
        kept, off, n_kept = O.sample_chunks(p, ro["phase"], None, None, B, seed=1, step=0)
        assert n_kept == cfg.T * B == len(kept)
        assert round(100 * n_kept / (cfg.T * cfg.N)) == consts[f"budget_fraction_B{B}_N64"][0]
        assert np.array_equal(off, np.arange(cfg.T + 1) * B)
        per = kept.reshape(cfg.T, B)
        assert (np.diff(per, axis=1) > 0).all()            # ascending, no duplicates
        assert (per // cfg.N == np.arange(cfg.T)[:, None]).all()


def test_sample_chunks_ragged_inactive_and_full_budget():
    cfg = CONFIGS["cfg1"]
    ro = make_rollouts(cfg, 0)
    n = ragged_n_chunks(cfg)
    active = np.ones(cfg.T, dtype=np.uint8)
    active[5] = 0
    p = np.array([1.0, 0.2, 0.1, 0.6])
    kept, off, n_kept = O.sample_chunks(p, ro["phase"], n, active, cfg.B, seed=9, step=4)
    for i in range(cfg.T):
        mine = kept[off[i]:off[i + 1]]
        want = 0 if not active[i] else min(cfg.B, n[i])
        assert len(mine) == want                           # |K_i| = min(B, N_i)  (Eq. 10)
        assert ((mine - i * cfg.N) < n[i]).all() and (mine >= i * cfg.N).all()
    # B >= N keeps every chunk: the unmasked objective's index set
    kept, off, n_kept = O.sample_chunks(p, ro["phase"], None, None, cfg.N + 3, seed=9, step=4)
    assert np.array_equal(kept, np.arange(cfg.T * cfg.N))


def test_allocation_tracks_weight_times_phase_size():
    # Sec. 4.3: E[b_c] grows with N_c * p_c; equal weights give b_c ~ B N_c / N (uniform allocation)
    cfg = CONFIGS["cfg2"].with_(n_groups=32)
    ro = make_rollouts(cfg, 0)
    ph = ro["phase"]
    sizes = np.array([(ph == c).sum() for c in range(cfg.K)], dtype=float)
    kept, _, n_kept = O.sample_chunks(np.ones(cfg.K), ph, None, None, cfg.B, seed=3, step=0)
    counts = np.bincount(ph.reshape(-1)[kept], minlength=cfg.K)
    assert np.allclose(counts / n_kept, sizes / sizes.sum(), atol=0.03)
    p = np.array([1.0, 0.1, 0.1, 0.5, 0.1])
    kept, _, n_kept = O.sample_chunks(p, ph, None, None, cfg.B, seed=3, step=0)
    counts = np.bincount(ph.reshape(-1)[kept], minlength=cfg.K)
    pred = sizes * p / (sizes * p).sum()
    # budget is ~19% of the chunks, so without-replacement saturation flattens the allocation a little
    assert np.argmax(counts) == np.argmax(pred)
    assert np.all(np.abs(counts / n_kept - pred) < 0.12)


# --------------------------------------------------------------------------- ablation selectors (Sec. 5.2, RQ4)

def test_random_selector_keeps_every_chunk_equally_often():
    # uniform sampling of m of N items without replacement includes each item with probability m / N
    T, N, K, B = 4, 10, 3, 4
    phase = np.array([[0] * 3 + [1] * 5 + [2] * 2] * T, dtype=np.uint8)
    p = np.array([1.0, 0.1, 0.4])
    counts = np.zeros(N)
    steps = 1500
    for s in range(steps):
        kept, off, nk = O.sample_chunks(p, phase, None, None, B, 99, s, selector="random")
        assert nk == T * B
        counts += np.bincount(kept % N, minlength=N)
    freq = counts / (steps * T)
    sigma = math.sqrt(0.4 * 0.6 / (steps * T))
    assert np.all(np.abs(freq - B / N) < 5 * sigma), freq
    # and it ignores the keep probabilities altogether
    a = O.sample_chunks(p, phase, None, None, B, 7, 3, selector="random")[0]
    b = O.sample_chunks(p[::-1].copy(), phase, None, None, B, 7, 3, selector="random")[0]
    assert np.array_equal(a, b)


def test_top_phase_selector_keeps_only_the_highest_phase():
    T, N, K, B = 3, 12, 4, 5
    phase = np.array([[0, 0, 1, 1, 1, 1, 1, 1, 2, 2, 3, 3],        # 6 chunks of phase 1 -> keeps 5
                      [1, 0, 0, 0, 2, 2, 2, 3, 3, 3, 1, 0],        # 2 chunks of phase 1 -> keeps both
                      [0, 0, 0, 2, 2, 2, 3, 3, 3, 3, 0, 0]],       # none -> keeps nothing
                     dtype=np.uint8)
    p = np.array([0.3, 1.0, 1.0, 0.1])                             # tie between phases 1 and 2: lowest index wins
    kept, off, nk = O.sample_chunks(p, phase, None, None, B, 5, 0, selector="top_phase")
    assert list(np.diff(off)) == [5, 2, 0] and nk == 7
    assert all(phase[g // N, g % N] == 1 for g in kept)
    assert sorted(kept[5:] % N) == [0, 10]
    # a ragged trajectory: chunks beyond n_chunks are not eligible
    kept, off, nk = O.sample_chunks(p, phase, np.array([4, 12, 12]), None, B, 5, 0, selector="top_phase")
    assert list(np.diff(off)) == [2, 2, 0] and sorted(kept[:2]) == [2, 3]


def test_importance_weights_hand_example_and_phase_totals():
    N, K = 8, 3
    phase = np.array([[0, 0, 0, 1, 1, 2, 2, 2], [2, 2, 2, 2, 0, 0, 1, 1]], dtype=np.uint8)
    kept = np.array([0, 3, 4, 7, 8 + 0, 8 + 1, 8 + 6])             # traj 0: phases 0,1,1,2; traj 1: 2,2,1
    w = O.importance_weights(phase, None, kept, K)
    assert np.array_equal(w, np.array([3 / 1, 2 / 2, 2 / 2, 3 / 1, 4 / 2, 4 / 2, 2 / 1], dtype=np.float32))
    # unbiasedness identity of the ratio estimator: over a phase's kept chunks the weights add up to N_c
    cfg = CONFIGS["cfg2"]
    ro = make_rollouts(cfg, 1)
    nch = ragged_n_chunks(cfg, 1)
    p = np.array([1.0, 0.1, 0.5, 0.2, 0.7])
    kept, off, nk = O.sample_chunks(p, ro["phase"], nch, None, cfg.B, cfg.seed, 1)
    w = O.importance_weights(ro["phase"], nch, kept, cfg.K).astype(np.float64)
    for i in range(0, cfg.T, 7):
        mine = kept[off[i]:off[i + 1]]
        wi = w[off[i]:off[i + 1]]
        for c in range(cfg.K):
            sel = ro["phase"][i, mine % cfg.N] == c
            if sel.any():
                n_c = int((ro["phase"][i, :nch[i]] == c).sum())
                assert abs(wi[sel].sum() - n_c) < 1e-4 * n_c


# --------------------------------------------------------------------------- stratified sampling (App. C, Theorem 1)

def test_stratified_allocation_hand_examples_and_invariants():
    # m = 12 over weights N_c q_c = (10*4, 20*1, 30*1) = (40, 20, 30): shares 5.33, 2.67, 4.0 -> floors 5, 2, 4, one
    # chunk left for the largest remainder (phase 1: 60 mod 90... remainders 30, 60, 0)
    assert O.stratified_allocation([4, 1, 1], [10, 20, 30], 12) == [5, 3, 4]
    # caps: phase 0 would get 9 of 12 but has only 3 chunks; the rest flows on by remainder order, then around again
    assert O.stratified_allocation([9, 1, 1], [3, 5, 5], 12) == [3, 5, 4]
    assert O.stratified_allocation([1, 1, 1], [4, 4, 4], 12) == [4, 4, 4]
    assert O.stratified_allocation([5, 5], [0, 7], 3) == [0, 3]
    rng = np.random.default_rng(3)
    for _ in range(300):
        K = int(rng.integers(1, 8))
        q = rng.integers(1, 65537, size=K)
        n = rng.integers(0, 40, size=K)
        m = int(rng.integers(0, n.sum() + 1))
        b = O.stratified_allocation(q, n, m)
        assert sum(b) == m and all(0 <= b[c] <= n[c] for c in range(K))
        # within one chunk of the real-valued optimum of Theorem 1 wherever the cap does not bind
        D = float((n * q).sum())
        if D > 0 and all(m * n[c] * q[c] / D <= n[c] for c in range(K)):
            assert all(abs(b[c] - m * n[c] * q[c] / D) < 1.0 for c in range(K))


def test_stratified_selector_budgets_uniformity_and_unbiased_weights():
    T, N, K, B = 2, 12, 3, 6
    phase = np.array([[0] * 2 + [1] * 6 + [2] * 4, [2] * 5 + [0] * 7], dtype=np.uint8)
    p = np.array([1.0, 0.25, 0.5])
    q = O.quantise_keep_probs(p)
    budgets = [O.stratified_allocation(q, [int((phase[i] == c).sum()) for c in range(K)], B) for i in range(T)]
    f = np.random.default_rng(4).standard_normal((T, N))          # any per-chunk quantity
    counts = np.zeros((T, N))
    est = np.zeros(T)
    steps = 3000
    for s in range(steps):
        kept, off, nk = O.sample_chunks(p, phase, None, None, B, 21, s, selector="stratified")
        w = O.importance_weights(phase, None, kept, K).astype(np.float64)
        for i in range(T):
            mine = kept[off[i]:off[i + 1]] % N
            assert [int((phase[i, mine] == c).sum()) for c in range(K)] == budgets[i]   # the budget is deterministic
            counts[i, mine] += 1
            est[i] += (w[off[i]:off[i + 1]] * f[i, mine]).sum()
    for i in range(T):
        for c in range(K):
            members = np.where(phase[i] == c)[0]
            if len(members) == 0:
                continue
            want = budgets[i][c] / len(members)                    # uniform within the phase
            sigma = math.sqrt(max(want * (1 - want), 1e-9) / steps)
            assert np.all(np.abs(counts[i, members] / steps - want) <= 5 * sigma + 1e-12)
        # with N_c / b_c weights the sampled sum is an unbiased estimate of the full sum (phases with b_c = 0 excluded)
        covered = [c for c in range(K) if budgets[i][c] > 0]
        full = sum(f[i, phase[i] == c].sum() for c in covered)
        spread = np.abs(f[i]).sum() * N / B
        assert abs(est[i] / steps - full) < 5 * spread / math.sqrt(steps)


def test_kept_phase_counts_hand_example_and_totals():
    # Sec. 5.2's realised allocation: kept chunks per phase next to the chunks that could have been kept
    phase = np.array([[0, 0, 1, 2], [1, 1, 2, 2], [0, 1, 1, 9]], dtype=np.uint8)      # 9 is out of range: read as K - 1
    kept = np.array([0, 2, 5, 7, 11])                                              # phases 0, 1, 1, 2, 2
    got, eligible = O.kept_phase_counts(phase, np.array([4, 3, 4]), np.array([1, 1, 1], np.uint8), kept, 3)
    assert np.array_equal(got, [1, 2, 2])
    assert np.array_equal(eligible, [3, 5, 3])                                     # trajectory 1 has 3 valid slots
    got, eligible = O.kept_phase_counts(phase, None, np.array([1, 0, 1], np.uint8), kept[[0, 1, 4]], 3)
    assert np.array_equal(got, [1, 1, 1]) and np.array_equal(eligible, [3, 3, 2])  # the inactive trajectory drops out
    cfg = CONFIGS["cfg2"]
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    p = np.array([1.0, 0.1, 0.5, 0.1, 0.3])
    kept, _, nk = O.sample_chunks(p, ro["phase"], ro["n_chunks"], active, cfg.B, cfg.seed, 0)
    got, eligible = O.kept_phase_counts(ro["phase"], ro["n_chunks"], active, kept, cfg.K)
    assert got.sum() == nk and np.array_equal(got, np.bincount(ro["phase"].reshape(-1)[kept], minlength=cfg.K))
    assert eligible.sum() == ro["n_chunks"][active.astype(bool)].sum() and np.all(got <= eligible)
    # the phase with keep probability 1 receives a larger share of its chunks than the ones at the floor
    share = got / np.maximum(eligible, 1)
    assert share[0] > share[1] and share[0] > share[3]
