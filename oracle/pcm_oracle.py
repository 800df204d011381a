"""CPU checker for Probabilistic Chunk Masking and the masked GRPO actor step.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 restatement of what
the paper's training step computes (Algorithm 1): it exists so that tests, the
smoke check and the benchmark's CPU-baseline leg have something independent to
compare the GPU library against.  It shares no code, tables or helpers with the
GPU library and must never be imported by it.

Every function names the passage of the paper it follows.  Where the paper is
silent or ambiguous the reading taken is stated in the docstring.

Parity status of each function (what pins it is in tests/test_oracle_*.py):
  advantages          pinned: closed form for binary rewards (Eq. 1)
  phase_scores        pinned: plain conditional-mean definition (Eq. 5), planted gaps,
                      symmetries
  KeepProbState       pinned: hand-worked example, Eq. 8 written via rho_c, invariants
  philox4x32_10       pinned: published known-answer vectors of the generator
  sample_chunks       pinned: brute-force Plackett-Luce enumeration on tiny inputs
  compact / sample    pinned: set properties (|K_i| = min(B, N_i), ascending, unique)
  label_phases        pinned: hand-labelled gripper traces, one per rule and per overlap of windows
  kept_phase_counts   pinned: hand example, totals (kept sums to the kept count, eligible to the valid
                      slots of active trajectories), agreement with a histogram of the kept chunks' labels
  selectors, weights  pinned: uniform inclusion frequencies of "random", phase purity and counts of
                      "top_phase", sum of N_c / b_c over a phase's kept chunks = N_c, hand example
  actor_step          pinned: head forward against explicit loops over the definition, log-softmax
                      and entropy against scipy, loss and every weight gradient against a library's
                      reverse-mode autodiff of the clipped surrogate (torch, fp64, CPU; its
                      cross_entropy routine in the rho = 1 case), finite differences, all-kept =
                      unmasked, zero gradient for uniform rewards, additivity over groups.  (The
                      paper prints no value for the head, so there is no golden number.)
  clip_grad_norm,     pinned: closed forms (first step moves every weight by lr * g / (|g| + eps),
  adamw_step          norm after clipping, decoupled decay with zero gradient) and agreement with
                      torch.optim.AdamW + torch.nn.utils.clip_grad_norm_ run in fp64 on the CPU
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
ACTION_SCALE_BITS = 24          # actions enter the score as integers round(a * 2^24)
WEIGHT_SCALE = 65536            # keep probabilities enter the sampler as round(p * 2^16)
MASK32 = 0xFFFFFFFF
MASK64 = 0xFFFFFFFFFFFFFFFF


# ----------------------------------------------------------------------------------------
# Eq. 1 -- group-relative advantages
# ----------------------------------------------------------------------------------------

def advantages(reward, G, eps=1e-6):
    """Group-relative advantage of Eq. 1 for binary rewards.

    A_i = (r_i - mu) / (sigma + eps) with mu, sigma the mean and the population
    (1/G) standard deviation of the group's rewards.  A group whose rewards are
    all equal ("collapsed", Sec. 1 and App. A) has A_i = 0; it is detected on the
    integer success count, never on a float.  Returns (adv f64[T], active u8[T]).
    """
    reward = np.asarray(reward).astype(np.int64)
    T = reward.shape[0]
    assert T % G == 0
    adv = np.zeros(T, dtype=F64)
    active = np.zeros(T, dtype=np.uint8)
    for g in range(T // G):
        r = reward[g * G:(g + 1) * G]
        s = int(r.sum())
        if s == 0 or s == G:
            continue
        mu = F64(s) / F64(G)
        sigma = np.sqrt(mu * (F64(1.0) - mu))
        adv[g * G:(g + 1) * G] = (r.astype(F64) - mu) / (sigma + F64(eps))
        active[g * G:(g + 1) * G] = 1
    return adv, active


# ----------------------------------------------------------------------------------------
# Eq. 5 -- success-vs-failure action score per phase
# ----------------------------------------------------------------------------------------

def phase_scores(actions, phase, reward, n_chunks, n_groups, G, K):
    """Batch-level phase score C_c^(t) (Eq. 5; Sec. 4.3 first paragraph; App. D.2 last paragraph).

    For every group with both outcomes (Sec. 4.1: only groups with non-zero reward
    variance) and every phase c, the chunks (i, k) of the group with phase c are
    pooled into a success set and a failure set; the score of (group, phase) is the
    Euclidean norm of the difference of the two sets' mean action vectors (each
    chunk's action is its L*D values flattened).  A (group, phase) pair lacking
    either outcome is skipped (App. D.2).  The batch score is the unweighted mean
    over the groups that contributed; valid_c says whether any did.  The paper's
    labelling assigns every chunk one of the K phases; an id >= K (outside that
    domain) is counted as phase K-1 here and in the sampler alike.

    Arithmetic convention shared with the GPU library so that the sampler
    downstream sees identical keep probabilities: each action enters as the
    integer q = rint(a * 2^24) (round half to even), sums are exact integers,
    means are taken as double(sum)/double(count), squared differences are added
    for j ascending without fused multiply-add, the norm is sqrt of that sum
    times 2^-24, and the mean over groups adds g ascending and divides once.
    Returns (C f64[K], valid u8[K]).
    """
    actions = np.asarray(actions, dtype=np.float32)
    T, N, A = actions.shape
    phase = np.asarray(phase)
    reward = np.asarray(reward).astype(np.int64)
    n_chunks = np.full(T, N, dtype=np.int64) if n_chunks is None else np.asarray(n_chunks, dtype=np.int64)
    q = np.rint(actions.astype(F64) * F64(2.0 ** ACTION_SCALE_BITS)).astype(np.int64)
    unscale = F64(2.0 ** -ACTION_SCALE_BITS)

    total = np.zeros(K, dtype=F64)
    contributors = np.zeros(K, dtype=np.int64)
    for g in range(n_groups):
        rows = range(g * G, (g + 1) * G)
        s = int(reward[g * G:(g + 1) * G].sum())
        if s == 0 or s == G:
            continue
        # integer sums and counts per (outcome, phase): index 1 = success, 0 = failure
        S = np.zeros((2, K, A), dtype=np.int64)
        n = np.zeros((2, K), dtype=np.int64)
        for i in rows:
            o = int(reward[i])
            for k in range(int(n_chunks[i])):
                c = min(int(phase[i, k]), K - 1)        # an id beyond the last phase counts as the last
                S[o, c] += q[i, k]
                n[o, c] += 1
        for c in range(K):
            n_pos, n_neg = int(n[1, c]), int(n[0, c])
            if n_pos == 0 or n_neg == 0:
                continue
            acc = F64(0.0)
            for j in range(A):
                diff = F64(int(S[1, c, j])) / F64(n_pos) - F64(int(S[0, c, j])) / F64(n_neg)
                acc = acc + diff * diff
            total[c] = total[c] + np.sqrt(acc) * unscale
            contributors[c] += 1
    C = np.zeros(K, dtype=F64)
    valid = np.zeros(K, dtype=np.uint8)
    for c in range(K):
        if contributors[c] > 0:
            C[c] = total[c] / F64(int(contributors[c]))
            valid[c] = 1
    return C, valid


# ----------------------------------------------------------------------------------------
# Eq. 7-9 -- score buffer, share/max normalisation, keep probabilities
# ----------------------------------------------------------------------------------------

class KeepProbState:
    """Per-phase score buffers and keep probabilities (Eq. 7-9; Algorithm 1, buffer steps).

    The buffer of a phase is held as its running sum S_c and its entry count
    (Eq. 8 only needs the sum).  Each step appends the valid scores; on the first
    step and then whenever T_rc steps have been appended since the last refresh,
    the buffers are collapsed: S_c -> share rho_c = S_c / sum S -> rho~_c =
    rho_c / max rho (Eq. 8), p_c = max(p_min, rho~_c) (Eq. 9), buffers reset.
    Between refreshes p is held fixed (Sec. 4.4).

    Readings: the trigger counts steps (Sec. 4.3 "every T_rc steps"), because with
    skipped phases the per-phase buffer lengths differ; a skipped phase simply has
    no entry that step; Eq. 8 sums (it does not average); the specified value of
    rho~_c is S_c / max S (the share denominator cancels; rho_c is still formed in
    `shares` so a test can confirm the two routes agree); when every S_c is zero
    rho~_c = 0 for all c, i.e. p_c = p_min (uniform sampling).  Before the first
    update p_c = 1.
    """

    def __init__(self, K):
        self.K = K
        self.S = np.zeros(K, dtype=F64)
        self.cnt = np.zeros(K, dtype=np.int64)
        self.step = 0
        self.since = 0
        self.p = np.ones(K, dtype=F64)
        self.shares = np.zeros(K, dtype=F64)

    def update(self, C, valid, p_min=0.1, T_rc=5):
        C = np.asarray(C, dtype=F64)
        for c in range(self.K):
            if valid[c]:
                self.S[c] = self.S[c] + C[c]
                self.cnt[c] += 1
        self.since += 1
        if self.step == 0 or self.since == T_rc:
            S_max = F64(0.0)
            S_sum = F64(0.0)
            for c in range(self.K):
                S_sum = S_sum + self.S[c]
                if self.S[c] > S_max:
                    S_max = self.S[c]
            for c in range(self.K):
                rho_tilde = self.S[c] / S_max if S_max > 0 else F64(0.0)
                self.shares[c] = self.S[c] / S_sum if S_sum > 0 else F64(0.0)
                self.p[c] = rho_tilde if rho_tilde > p_min else F64(p_min)
            self.S[:] = 0
            self.cnt[:] = 0
            self.since = 0
        self.step += 1
        return self.p.copy()


# ----------------------------------------------------------------------------------------
# counter-based random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11)
# ----------------------------------------------------------------------------------------

_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85


def philox4x32_10(counter, key):
    """Philox-4x32 with 10 rounds as published; counter = 4 words, key = 2 words (32-bit each)."""
    c0, c1, c2, c3 = (int(x) & MASK32 for x in counter)
    k0, k1 = (int(x) & MASK32 for x in key)
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK32
        hi1, lo1 = p1 >> 32, p1 & MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & MASK32, lo1, (hi0 ^ c3 ^ k1) & MASK32, lo0
        k0 = (k0 + _PHILOX_W0) & MASK32
        k1 = (k1 + _PHILOX_W1) & MASK32
    return c0, c1, c2, c3


def rng64(seed, step, traj, rnd):
    """64 random bits for sampling round `rnd` of trajectory `traj` at training step `step`.

    Stateless and keyed by global ids, so the draw does not depend on how the work
    is laid out.  key = (seed low, seed high); counter = (traj, rnd, step low,
    step high); result = word0 | word1 << 32.
    """
    seed = int(seed) & MASK64
    step = int(step) & MASK64
    out = philox4x32_10((traj, rnd, step & MASK32, step >> 32), (seed & MASK32, seed >> 32))
    return out[0] | (out[1] << 32)


# ----------------------------------------------------------------------------------------
# App. D, phase allotment rules -- gripper-based phase labels
# ----------------------------------------------------------------------------------------

PHASE_APPROACH, PHASE_PRE_GRASP, PHASE_ACTIVE_GRIP, PHASE_RELEASE_RAMP, PHASE_TAIL = 0, 1, 2, 3, 4


def label_phases(actions, n_chunks, L, D, gripper_dim=None, close_threshold=0.0):
    """Deterministic gripper-based phase label of every chunk (App. D, phase allotment rules).

    actions [T, N, L*D]: L timesteps of D values per chunk; the gripper-close command of a
    timestep is active when its gripper value (dimension `gripper_dim`, the last one by
    default) exceeds `close_threshold`.  With n_j the number of active timesteps of chunk j
    (g_f = n_j / L, compared exactly through integers):
      sustained close   g_f >= 0.75; maximal runs of such chunks are the grasp intervals
      active-grip       g_f >= 0.5
      pre-grasp         one of the three chunks right before a grasp interval, 0.1 <= g_f < 0.5
      release-ramp      one of the three chunks right after a grasp interval, g_f < 0.5
      approach          g_f < 0.5 and a grasp interval begins later in the trajectory
      tail              what remains after the last grasp interval
    with priority active-grip > pre-grasp > release-ramp > approach > tail where windows overlap.
    Readings where the rules leave a gap: the window tests apply chunk by chunk (a chunk that
    fails its threshold does not end the window); a trajectory without any grasp interval is
    all approach (nothing has been grasped yet) apart from its active-grip chunks; chunks after
    the last interval that are neither in its release window nor open (g_f >= 0.1) are tail.
    Returns u8 [T, N]; chunk slots at and beyond n_chunks[i] get 0.
    """
    actions = np.asarray(actions)
    T, N, LD = actions.shape
    assert LD == L * D
    g = D - 1 if gripper_dim is None else gripper_dim
    n_chunks = np.full(T, N, dtype=np.int64) if n_chunks is None else np.asarray(n_chunks, dtype=np.int64)
    out = np.zeros((T, N), dtype=np.uint8)
    for i in range(T):
        Ni = int(min(max(n_chunks[i], 0), N))
        count = [int(sum(1 for t in range(L) if actions[i, j, t * D + g] > close_threshold)) for j in range(Ni)]
        sustained = [4 * c >= 3 * L for c in count]
        last = max((j for j in range(Ni) if sustained[j]), default=-1)
        for j in range(Ni):
            c = count[j]
            if 2 * c >= L:
                out[i, j] = PHASE_ACTIVE_GRIP
                continue
            before_grasp = any(sustained[k] for k in range(j + 1, min(j + 4, Ni)))
            after_grasp = any(sustained[k] for k in range(max(j - 3, 0), j))
            if before_grasp and 10 * c >= L:
                out[i, j] = PHASE_PRE_GRASP
            elif after_grasp:
                out[i, j] = PHASE_RELEASE_RAMP
            elif last < 0 or j < last:
                out[i, j] = PHASE_APPROACH
            else:
                out[i, j] = PHASE_TAIL
    return out


# ----------------------------------------------------------------------------------------
# Eq. 10 -- fixed-budget weighted sampling without replacement, then compaction
# ----------------------------------------------------------------------------------------

def quantise_keep_probs(p):
    """Integer sampling weights q_c = floor(p_c * 2^16 + 0.5), clamped to [1, 2^16]."""
    p = np.asarray(p, dtype=F64)
    q = np.ones(p.shape[0], dtype=np.int64)
    for c in range(p.shape[0]):
        x = p[c] * F64(WEIGHT_SCALE) + F64(0.5)
        if x >= WEIGHT_SCALE:
            q[c] = WEIGHT_SCALE
        elif x >= 1.0:
            q[c] = int(np.floor(x))
        else:                      # includes NaN
            q[c] = 1
    return q


def sample_trajectory(weights, m, seed, step, traj):
    """Successive (Plackett-Luce) sampling of m items without replacement (Eq. 10).

    `weights` are positive integers.  Round r draws x = rng64(seed, step, traj, r),
    maps it to t = floor(x * W_rem / 2^64) in [0, W_rem) and picks the first
    remaining index (ascending) whose inclusive running weight exceeds t, i.e.
    index k is picked with probability w_k / W_rem up to the 2^-64 granularity of
    x.  Returns the picks in draw order.
    """
    w = [int(x) for x in weights]
    W_rem = sum(w)
    picks = []
    for r in range(m):
        x = rng64(seed, step, traj, r)
        t = (x * W_rem) >> 64
        run = 0
        chosen = -1
        for k, wk in enumerate(w):
            run += wk
            if wk > 0 and run > t:
                chosen = k
                break
        assert chosen >= 0
        picks.append(chosen)
        W_rem -= w[chosen]
        w[chosen] = 0
    return picks


def stratified_allocation(q, n_c, m):
    """Per-phase budgets b_c of the stratified estimator (App. C, Theorem 1: b_c* = B N_c sqrt(V_c) / sum N_c' sqrt(V_c'),
    with the keep probability, as integer weight q_c, standing for sqrt(V_c)).

    m chunks are shared out over the phases in proportion to N_c q_c by the largest-remainder rule, never more than
    N_c to a phase: b_c = floor(m N_c q_c / D), D = sum N_c' q_c'; the chunks left over go one at a time to the
    phase with the largest remainder (m N_c q_c) mod D that still has room (lowest index on ties), and, if the caps
    leave some undistributed after every remainder has been served once, on in the same order.  All integers.
    The rounding rule is not in the paper (the theorem treats b_c as real numbers).
    """
    K = len(q)
    weight = [int(n_c[c]) * int(q[c]) for c in range(K)]
    D = sum(weight)
    assert 0 <= m <= sum(int(x) for x in n_c)
    if D == 0:
        return [0] * K
    b = [min(int(n_c[c]), (m * weight[c]) // D) for c in range(K)]
    rem = [(m * weight[c]) % D for c in range(K)]
    order = sorted(range(K), key=lambda c: (-rem[c], c))
    left = m - sum(b)
    while left > 0:
        progressed = False
        for c in order:
            if left > 0 and b[c] < int(n_c[c]):
                b[c] += 1
                left -= 1
                progressed = True
        assert progressed
    return b


def sample_chunks(keep_probs, phase, n_chunks, active, B, seed, step, selector="pcm"):
    """Kept set per trajectory and its compaction (Eq. 10; Algorithm 1 inner loop; Sec. 4.5).

    selector (Sec. 5.2, RQ4: the two ablations that bracket the method):
      "pcm"        weights = the phases' keep probabilities (the method);
      "random"     every chunk has the same weight: min(B, N_i) chunks uniformly at random;
      "top_phase"  only chunks of the single phase with the largest keep probability (lowest
                   index on ties) are eligible, with equal weights; a trajectory keeps
                   min(B, number of its chunks in that phase) of them (none if it has none).
      "stratified" the sampling scheme that the variance analysis of App. C assumes: a fixed budget b_c per
                   phase (stratified_allocation, from the keep probabilities and the trajectory's phase sizes),
                   then b_c chunks of phase c uniformly without replacement, phases in index order, the draw
                   counter running on across phases.

    Every chunk inherits its phase's keep probability as weight (Sec. 4.4); each
    active trajectory keeps min(B, N_i) chunks; trajectories of collapsed groups
    (active = 0) keep none, since their advantage, hence every term of Eq. 11, is
    zero.  Physical shrinking is expressed as the ascending list of global chunk
    ids i*N + k of the kept chunks, trajectories in order, plus the exclusive scan
    of per-trajectory kept counts.
    Returns (kept_idx i32[n_kept], offsets i32[T+1], n_kept).
    """
    phase = np.asarray(phase)
    T, N = phase.shape
    K = len(keep_probs)
    if selector in ("pcm", "stratified"):
        q = quantise_keep_probs(keep_probs)
    elif selector == "random":
        q = np.ones(K, dtype=np.int64)
    elif selector == "top_phase":
        best = 0
        for c in range(1, K):
            if keep_probs[c] > keep_probs[best]:
                best = c
        q = np.zeros(K, dtype=np.int64)
        q[best] = 1
    else:
        raise ValueError(selector)
    n_chunks = np.full(T, N, dtype=np.int64) if n_chunks is None else np.asarray(n_chunks, dtype=np.int64)
    kept = []
    offsets = np.zeros(T + 1, dtype=np.int32)
    for i in range(T):
        Ni = int(n_chunks[i])
        if (active is not None and not active[i]) or Ni == 0:
            offsets[i + 1] = offsets[i]
            continue
        ph = [min(int(phase[i, k]), K - 1) for k in range(Ni)]
        w = [int(q[c]) for c in ph]
        m = min(B, sum(1 for x in w if x > 0))
        if selector == "stratified":
            n_c = [sum(1 for c in ph if c == cc) for cc in range(K)]
            budget = stratified_allocation(q, n_c, m)
            picks, r = [], 0
            for cc in range(K):
                members = [k for k in range(Ni) if ph[k] == cc]
                for _ in range(budget[cc]):
                    x = rng64(seed, step, i, r)
                    t = (x * len(members)) >> 64          # uniform over the phase's remaining chunks, ascending
                    picks.append(members.pop(t))
                    r += 1
            picks.sort()
        else:
            picks = sorted(sample_trajectory(w, m, seed, step, i))
        kept.extend(i * N + k for k in picks)
        offsets[i + 1] = offsets[i] + m
    return np.asarray(kept, dtype=np.int32), offsets, int(offsets[T])


def importance_weights(phase, n_chunks, kept_idx, K):
    """Weights N_c / b_c of the ratio estimator (App. C, the unbiased alternative to Eq. 11).

    For a kept chunk of trajectory i and phase c: N_c = number of the trajectory's (valid) chunks
    in phase c, b_c = number of its kept chunks in phase c.  Summed over the kept chunks of one
    (trajectory, phase) the weights give back N_c.  Returns f32 [len(kept_idx)], the quotient
    of the two counts rounded once to single precision.
    """
    phase = np.asarray(phase)
    T, N = phase.shape
    n_chunks = np.full(T, N, dtype=np.int64) if n_chunks is None else np.asarray(n_chunks, dtype=np.int64)
    kept_idx = np.asarray(kept_idx, dtype=np.int64)
    out = np.zeros(len(kept_idx), dtype=np.float32)
    for j, g in enumerate(kept_idx):
        i, k = int(g) // N, int(g) % N
        c = min(int(phase[i, k]), K - 1)
        in_phase = [kk for kk in range(int(n_chunks[i])) if min(int(phase[i, kk]), K - 1) == c]
        kept_here = [int(x) % N for x in kept_idx if int(x) // N == i]
        b = sum(1 for kk in kept_here if min(int(phase[i, kk]), K - 1) == c)
        out[j] = np.float32(len(in_phase)) / np.float32(b)
    return out


def kept_phase_counts(phase, n_chunks, active, kept_idx, K):
    """Realised allocation of the budget over the phases (Sec. 5.2, the per-phase view of which chunks
    the sampler kept over training): for every phase the number of kept chunks, and the number of
    chunks the sampler could have kept (valid chunk slots of active trajectories).  Phase ids >= K
    count as K - 1, as everywhere.  Returns (kept i32[K], eligible i32[K])."""
    phase = np.asarray(phase)
    T, N = phase.shape
    n_chunks = np.full(T, N, dtype=np.int64) if n_chunks is None else np.asarray(n_chunks, dtype=np.int64)
    kept = np.zeros(K, dtype=np.int32)
    eligible = np.zeros(K, dtype=np.int32)
    for g in np.asarray(kept_idx, dtype=np.int64):
        kept[min(int(phase[int(g) // N, int(g) % N]), K - 1)] += 1
    for i in range(T):
        if active is not None and not active[i]:
            continue
        for k in range(min(max(int(n_chunks[i]), 0), N)):
            eligible[min(int(phase[i, k]), K - 1)] += 1
    return kept, eligible


# ----------------------------------------------------------------------------------------
# Eq. 2 / Eq. 11 -- (masked) GRPO actor step through the action head
# ----------------------------------------------------------------------------------------

def _silu_parts(u):
    s = 1.0 / (1.0 + np.exp(-u))
    return s, u * s


def head_forward(X, Wg, Wu, Wd, Wo):
    """Action head: gated MLP then bin logits.  u = X Wg, v = X Wu, a = silu(u) * v, y = a Wd, z = y Wo."""
    u = X @ Wg
    v = X @ Wu
    s, su = _silu_parts(u)
    a = su * v
    y = a @ Wd
    z = y @ Wo
    return u, v, s, su, a, y, z


def log_softmax_rows(z):
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    denom = e.sum(axis=1, keepdims=True)
    return (z - zmax) - np.log(denom), e / denom


def actor_step(hidden, tokens, logp_old, adv, kept_idx, N, A, Wg, Wu, Wd, Wo,
               eps_low=0.2, eps_high=0.2, loss_scale=1.0, want_grads=True,
               token_mean=False, entropy_coef=0.0, chunk_ratio=False, chunk_weight=None):
    """Masked GRPO actor step over the kept chunks (Eq. 11; Eq. 2 when every chunk is kept).

    Rows: the A action tokens of each kept chunk, in kept order.  For a row with
    hidden state x, target bin b, old log-probability l0 and trajectory advantage A_i:
    l = log softmax(z)[b]; rho = exp(l - l0); term = min(rho A_i, clip(rho, 1 - eps_low,
    1 + eps_high) A_i) (the PPO clipping that Eq. 2 leaves out for clarity; App. D gives
    its thresholds); loss = -loss_scale * sum of terms, so that loss_scale = 1/T gives
    the mean over trajectories of the sum over kept chunks of Eq. 11, the chunk's log
    probability being the sum of its tokens'.  With rho = 1 the gradient is that of
    -loss_scale * sum A_i log pi.  A ratio exactly on a clip boundary counts as unclipped.

    Variants of the training loss (App. D, and the estimator discussed under Eq. 11):
      token_mean    the sums are divided by the number of kept rows (scale = loss_scale / M);
      entropy_coef  subtracts entropy_coef * scale * sum over rows of the entropy of softmax(z)
                    (App. D: entropy coefficient 1e-3);
      chunk_ratio   one ratio per chunk, the ratio of the chunk's probabilities
                    rho_c = exp(sum over its A tokens of (l - l0)), one clipped term per chunk
                    (Eq. 2 is written per chunk; the per-token form above is the default);
      chunk_weight  f64 [len(kept_idx)], multiplies each chunk's term(s): the importance weights
                    N_c / b_c of the unbiased estimator (App. C) or any other reweighting.

    hidden [T*N*A, d], tokens [T*N*A], logp_old [T*N*A], adv [T], kept_idx: global chunk ids.
    Returns a dict with loss, logp (per kept row), ratio (per row), dz, and (if want_grads)
    dWg, dWu, dWd, dWo, dX plus stats = [fraction of rows whose policy-gradient term is clipped
    away, mean ratio, mean(l0 - l), rows, mean row entropy].
    """
    kept_idx = np.asarray(kept_idx, dtype=np.int64)
    rows = (kept_idx[:, None] * A + np.arange(A)[None, :]).reshape(-1)
    X = np.asarray(hidden)[rows].astype(F64)
    tok = np.asarray(tokens)[rows].astype(np.int64)
    l0 = np.asarray(logp_old)[rows].astype(F64)
    adv_row = np.repeat(np.asarray(adv, dtype=F64)[kept_idx // N], A)
    if chunk_weight is None:
        w_row = np.ones(rows.shape[0], dtype=F64)
    else:
        w_row = np.repeat(np.asarray(chunk_weight, dtype=F64), A)
    Wg, Wu, Wd, Wo = (np.asarray(w).astype(F64) for w in (Wg, Wu, Wd, Wo))
    M = X.shape[0]
    scale = F64(loss_scale)
    if token_mean:
        scale = scale / F64(M) if M else F64(0.0)

    u, v, s, su, a, y, z = head_forward(X, Wg, Wu, Wd, Wo)
    logsm, sm = log_softmax_rows(z)
    lp = logsm[np.arange(M), tok]
    delta = lp - l0
    if chunk_ratio:
        rho = np.repeat(np.exp(delta.reshape(-1, A).sum(axis=1)), A)
    else:
        rho = np.exp(delta)
    clipped = np.clip(rho, 1.0 - eps_low, 1.0 + eps_high)
    term = w_row * np.minimum(rho * adv_row, clipped * adv_row)
    if chunk_ratio:
        term_sum = term.reshape(-1, A)[:, 0].sum()          # one term per chunk
    else:
        term_sum = term.sum()
    entropy = -(sm * logsm).sum(axis=1)
    loss = -scale * term_sum - F64(entropy_coef) * scale * entropy.sum()
    flows = ((adv_row >= 0) & (rho <= 1.0 + eps_high)) | ((adv_row < 0) & (rho >= 1.0 - eps_low))
    out = {"loss": loss, "logp": lp, "ratio": rho, "rows": rows, "entropy": entropy}
    if M:
        out["stats"] = np.array([1.0 - flows.mean(), rho.mean(), (l0 - lp).mean(), float(M), entropy.mean()])
    else:
        out["stats"] = np.array([0.0, 0.0, 0.0, 0.0, 0.0])
    if not want_grads:
        return out
    # d(term)/d(l) of a row: rho * A_i where the unclipped branch is the active one; with a chunk ratio
    # every row of the chunk sees the chunk's term through rho_c, whose derivative in each l is rho_c
    gcoef = np.where(flows, w_row * rho * adv_row, 0.0)
    onehot = np.zeros_like(z)
    onehot[np.arange(M), tok] = 1.0
    dz = (-scale * gcoef)[:, None] * (onehot - sm)
    dz = dz + F64(entropy_coef) * scale * sm * (logsm + entropy[:, None])
    dWo = y.T @ dz
    dy = dz @ Wo.T
    dWd = a.T @ dy
    da = dy @ Wd.T
    dv = da * su
    du = da * v * (s * (1.0 + u * (1.0 - s)))
    dWg = X.T @ du
    dWu = X.T @ dv
    dX = du @ Wg.T + dv @ Wu.T
    out.update(dz=dz, dWg=dWg, dWu=dWu, dWd=dWd, dWo=dWo, dX=dX)
    return out


# ----------------------------------------------------------------------------------------
# App. D (training details) -- the optimizer step that follows the actor gradients
# ----------------------------------------------------------------------------------------

def clip_grad_norm(grads, max_norm, eps=1e-6):
    """Global-norm gradient clipping (App. D: "gradient clipping at 2.0").

    The norm is the Euclidean norm over all gradient tensors taken together; the gradients
    are multiplied by min(1, max_norm / (norm + eps)).  The paper gives the threshold only;
    the joint 2-norm and eps = 1e-6 are the convention of the pipeline it builds on.
    Returns (scaled gradients, norm before clipping).
    """
    total = F64(0.0)
    for g in grads:
        g = np.asarray(g, dtype=F64)
        total += np.sum(g * g)
    norm = np.sqrt(total)
    scale = min(F64(1.0), F64(max_norm) / (norm + F64(eps)))
    return [np.asarray(g, dtype=F64) * scale for g in grads], norm


def adamw_step(params, grads, m, v, t, lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
               max_grad_norm=2.0):
    """One AdamW update after global-norm clipping (App. D: lr 1e-5, betas (0.9, 0.999),
    weight decay 0, clipping at 2.0; eps is not stated, 1e-8 is the usual default).

    For every tensor, with g the clipped gradient and t >= 1 the step number:
        m <- beta1 m + (1 - beta1) g            v <- beta2 v + (1 - beta2) g^2
        theta <- theta (1 - lr wd)              (decoupled decay)
        theta <- theta - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
    Returns (params, m, v, grad_norm), all new fp64 arrays.
    """
    assert t >= 1
    g_clipped, norm = clip_grad_norm(grads, max_grad_norm)
    bc1 = F64(1.0) - F64(beta1) ** t
    bc2 = F64(1.0) - F64(beta2) ** t
    new_p, new_m, new_v = [], [], []
    for theta, g, m_i, v_i in zip(params, g_clipped, m, v):
        theta = np.asarray(theta, dtype=F64)
        m_n = F64(beta1) * np.asarray(m_i, dtype=F64) + (F64(1.0) - F64(beta1)) * g
        v_n = F64(beta2) * np.asarray(v_i, dtype=F64) + (F64(1.0) - F64(beta2)) * g * g
        theta_n = theta * (F64(1.0) - F64(lr) * F64(weight_decay))
        theta_n = theta_n - F64(lr) * (m_n / bc1) / (np.sqrt(v_n / bc2) + F64(eps))
        new_p.append(theta_n)
        new_m.append(m_n)
        new_v.append(v_n)
    return new_p, new_m, new_v, norm
