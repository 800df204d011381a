"""Pins for the CPU checker's actor step (Eq. 2 and Eq. 11 of the paper, with PPO clipping).

No number printed in the paper fixes the head's arithmetic, so the pins are what
the mathematics fixes: textbook definitions of softmax and matrix products
evaluated independently, finite differences of the scalar loss, a library's
reverse-mode autodiff of the clipped surrogate (and its cross-entropy routine in
the rho = 1 case), the all-kept mask reproducing the unmasked objective, zero
gradient for uniform rewards, additivity over groups.
"""
import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import pcm_oracle as O


def _problem(seed=0, T=4, G=4, N=5, A=3, d=6, ff=8, V=7, wstd=0.4):
    r = np.random.default_rng(seed)
    rows = T * N * A
    hidden = r.standard_normal((rows, d))
    tokens = r.integers(0, V, size=rows)
    W = {"Wg": r.standard_normal((d, ff)) * wstd, "Wu": r.standard_normal((d, ff)) * wstd,
         "Wd": r.standard_normal((ff, d)) * wstd, "Wo": r.standard_normal((d, V)) * wstd}
    reward = np.array([1, 0, 0, 1] * (T // 4), dtype=np.uint8)
    adv, _ = O.advantages(reward, G)
    return dict(hidden=hidden, tokens=tokens, adv=adv, N=N, A=A, T=T, **W)


def _call(p, kept, logp_old, **kw):
    return O.actor_step(p["hidden"], p["tokens"], logp_old, p["adv"], kept, p["N"], p["A"],
                        p["Wg"], p["Wu"], p["Wd"], p["Wo"], **kw)


def _logp_all(p, W=None):
    W = W or p
    *_, z = O.head_forward(p["hidden"].astype(np.float64), W["Wg"], W["Wu"], W["Wd"], W["Wo"])
    return (z - logsumexp(z, axis=1, keepdims=True))[np.arange(z.shape[0]), p["tokens"]]


def test_logsoftmax_and_matmul_against_independent_definitions():
    r = np.random.default_rng(1)
    z = r.standard_normal((9, 11)) * 30
    ls, sm = O.log_softmax_rows(z)
    assert np.allclose(ls, z - logsumexp(z, axis=1, keepdims=True), rtol=1e-13, atol=1e-13)
    assert np.allclose(sm.sum(1), 1.0, rtol=1e-14)
    # head forward against explicit triple loops
    X, Wg, Wu = r.standard_normal((3, 4)), r.standard_normal((4, 5)), r.standard_normal((4, 5))
    Wd, Wo = r.standard_normal((5, 4)), r.standard_normal((4, 6))
    u, v, s, su, a, y, z = O.head_forward(X, Wg, Wu, Wd, Wo)
    for m in range(3):
        a_ref = np.zeros(5)
        for j in range(5):
            uu = sum(X[m, i] * Wg[i, j] for i in range(4))
            vv = sum(X[m, i] * Wu[i, j] for i in range(4))
            a_ref[j] = uu / (1 + np.exp(-uu)) * vv
        y_ref = [sum(a_ref[j] * Wd[j, i] for j in range(5)) for i in range(4)]
        z_ref = [sum(y_ref[i] * Wo[i, b] for i in range(4)) for b in range(6)]
        assert np.allclose(z[m], z_ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("perturb", [0.0, 0.15])
def test_gradients_match_finite_differences(perturb):
    # central differences of the scalar loss in fp64; with perturb = 0 the ratio is 1 everywhere,
    # with perturb > 0 some rows sit on the flat (clipped) side and must contribute nothing
    p = _problem(seed=2)
    r = np.random.default_rng(5)
    old = {k: p[k] + perturb * r.standard_normal(p[k].shape) for k in ("Wg", "Wu", "Wd", "Wo")}
    logp_old = _logp_all(p, old)
    kept = np.array([0, 3, 4, 7, 11, 12, 18, 19])
    kw = dict(eps_low=0.2, eps_high=0.3, loss_scale=0.25)
    ref = _call(p, kept, logp_old, **kw)
    if perturb > 0:
        flows_frac = 1 - ref["stats"][0]
        assert 0.05 < flows_frac < 0.95                   # both branches of the clip are exercised
    h = 1e-6
    for name in ("Wg", "Wu", "Wd", "Wo", "hidden"):
        W = p[name]
        g = ref["d" + name] if name != "hidden" else None
        for _ in range(6):
            if name == "hidden":
                kr = int(r.integers(0, len(ref["rows"])))
                idx = (int(ref["rows"][kr]), int(r.integers(0, W.shape[1])))
                analytic = ref["dX"][kr, idx[1]]
            else:
                idx = tuple(int(r.integers(0, s)) for s in W.shape)
                analytic = g[idx]
            keep = W[idx]
            W[idx] = keep + h
            lp = _call(p, kept, logp_old, want_grads=False, **kw)["loss"]
            W[idx] = keep - h
            lm = _call(p, kept, logp_old, want_grads=False, **kw)["loss"]
            W[idx] = keep
            fd = (lp - lm) / (2 * h)
            assert abs(fd - analytic) <= 1e-6 * max(1.0, abs(analytic)) + 1e-8, (name, idx, fd, analytic)


def _torch_head(p, Wt, rows):
    import torch
    import torch.nn.functional as F
    X = torch.tensor(p["hidden"][rows], dtype=torch.float64)
    z = ((F.silu(X @ Wt["Wg"]) * (X @ Wt["Wu"])) @ Wt["Wd"]) @ Wt["Wo"]
    return X, z


@pytest.mark.parametrize("perturb", [0.0, 0.2])
def test_gradients_match_library_autograd(perturb):
    """The clipped surrogate written with a library's primitives (silu, matmul, log_softmax, clamp,
    minimum) and differentiated by its reverse-mode autodiff, fp64 on the CPU: every weight gradient
    and the loss.  At perturb = 0 the ratio is 1 and the objective is advantage-weighted cross-entropy,
    which is evaluated with the library's own cross_entropy routine."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    p = _problem(seed=6)
    r = np.random.default_rng(8)
    old = {k: p[k] + perturb * r.standard_normal(p[k].shape) for k in ("Wg", "Wu", "Wd", "Wo")}
    logp_old = _logp_all(p, old)
    kept = np.array([1, 2, 5, 8, 9, 13, 17])
    eps_low, eps_high, scale = 0.2, 0.4, 0.125
    ref = _call(p, kept, logp_old, eps_low=eps_low, eps_high=eps_high, loss_scale=scale)
    rows = (kept[:, None] * p["A"] + np.arange(p["A"])[None, :]).reshape(-1)
    assert np.array_equal(rows, ref["rows"])
    Wt = {k: torch.tensor(p[k], dtype=torch.float64, requires_grad=True) for k in ("Wg", "Wu", "Wd", "Wo")}
    _, z = _torch_head(p, Wt, rows)
    tok = torch.tensor(p["tokens"][rows], dtype=torch.long)
    adv_row = torch.tensor(p["adv"][kept // p["N"]].repeat(p["A"]), dtype=torch.float64)
    if perturb == 0.0:
        loss = scale * (adv_row * F.cross_entropy(z, tok, reduction="none")).sum()
        # value of the surrogate at rho = 1 is -scale * sum A; only its gradient is that of the cross-entropy
        value = -scale * float(adv_row.sum())
    else:
        logp = F.log_softmax(z, dim=1).gather(1, tok[:, None])[:, 0]
        rho = torch.exp(logp - torch.tensor(logp_old[rows]))
        loss = -scale * torch.minimum(rho * adv_row, torch.clamp(rho, 1 - eps_low, 1 + eps_high) * adv_row).sum()
        value = float(loss.detach())
        assert 0.05 < ref["stats"][0] < 0.95                # some rows clipped, some not
    loss.backward()
    assert np.isclose(ref["loss"], value, rtol=1e-12, atol=1e-12)
    for k in ("Wg", "Wu", "Wd", "Wo"):
        g = Wt[k].grad.numpy()
        assert np.allclose(ref["d" + k], g, rtol=1e-10, atol=1e-12 * max(1.0, np.abs(g).max())), k


@pytest.mark.parametrize("kw", [dict(entropy_coef=0.05), dict(token_mean=True), dict(chunk_ratio=True),
                                dict(chunk_weight=True), dict(token_mean=True, entropy_coef=0.02, chunk_ratio=True,
                                                              chunk_weight=True)])
def test_variant_gradients_match_library_autograd(kw):
    """The loss variants written with library primitives (entropy through torch.special.entr, one
    ratio per chunk through a sum of log-probabilities) and differentiated by reverse-mode autodiff."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    p = _problem(seed=9)
    r = np.random.default_rng(10)
    old = {k: p[k] + 0.1 * r.standard_normal(p[k].shape) for k in ("Wg", "Wu", "Wd", "Wo")}
    logp_old = _logp_all(p, old)
    kept = np.array([0, 2, 6, 7, 10, 14, 15, 19])
    A = p["A"]
    eps_low, eps_high, scale0 = 0.2, 0.4, 0.5
    kw = dict(kw)
    cw = r.uniform(0.5, 3.0, size=len(kept)) if kw.pop("chunk_weight", False) else None
    ref = _call(p, kept, logp_old, eps_low=eps_low, eps_high=eps_high, loss_scale=scale0, chunk_weight=cw, **kw)
    rows = ref["rows"]
    Wt = {k: torch.tensor(p[k], dtype=torch.float64, requires_grad=True) for k in ("Wg", "Wu", "Wd", "Wo")}
    _, z = _torch_head(p, Wt, rows)
    tok = torch.tensor(p["tokens"][rows], dtype=torch.long)
    adv_chunk = torch.tensor(p["adv"][kept // p["N"]], dtype=torch.float64)
    w_chunk = torch.ones(len(kept), dtype=torch.float64) if cw is None else torch.tensor(cw)
    delta = F.log_softmax(z, dim=1).gather(1, tok[:, None])[:, 0] - torch.tensor(logp_old[rows])
    scale = scale0 / len(rows) if kw.get("token_mean") else scale0
    if kw.get("chunk_ratio"):
        rho = torch.exp(delta.reshape(-1, A).sum(1))                       # one ratio, one term per chunk
        terms = w_chunk * torch.minimum(rho * adv_chunk, torch.clamp(rho, 1 - eps_low, 1 + eps_high) * adv_chunk)
    else:
        rho = torch.exp(delta)
        a_row, w_row = adv_chunk.repeat_interleave(A), w_chunk.repeat_interleave(A)
        terms = w_row * torch.minimum(rho * a_row, torch.clamp(rho, 1 - eps_low, 1 + eps_high) * a_row)
    entropy = torch.special.entr(F.softmax(z, dim=1)).sum()
    loss = -scale * terms.sum() - kw.get("entropy_coef", 0.0) * scale * entropy
    loss.backward()
    assert np.isclose(ref["loss"], float(loss.detach()), rtol=1e-12, atol=1e-12)
    for k in ("Wg", "Wu", "Wd", "Wo"):
        g = Wt[k].grad.numpy()
        assert np.allclose(ref["d" + k], g, rtol=1e-10, atol=1e-12 * max(1.0, np.abs(g).max())), (k, kw)


def test_all_kept_equals_unmasked_objective():
    # Eq. 11 with K_i = all chunks is Eq. 2: loss = -(1/T) sum_i A_i sum_k log pi(chunk), at rho = 1
    p = _problem(seed=3)
    lp_all = _logp_all(p)
    kept = np.arange(p["T"] * p["N"])
    out = _call(p, kept, lp_all, loss_scale=1.0 / p["T"])
    chunk_logp = lp_all.reshape(p["T"], p["N"], p["A"]).sum(-1)
    # value of the surrogate at rho = 1 is -(1/T) sum A_i * N_i * A  (each token term equals A_i)
    assert np.isclose(out["loss"], -(p["adv"] * p["N"] * p["A"]).sum() / p["T"], rtol=1e-12, atol=1e-12)
    # its gradient is that of -(1/T) sum_i A_i sum_k log pi(a_ik | s_ik): check through Wo by differences
    h = 1e-6
    r = np.random.default_rng(0)
    for _ in range(5):
        idx = (int(r.integers(0, p["Wo"].shape[0])), int(r.integers(0, p["Wo"].shape[1])))
        keep = p["Wo"][idx]
        p["Wo"][idx] = keep + h
        fp = -(p["adv"][:, None] * _logp_all(p).reshape(p["T"], p["N"], p["A"]).sum(-1)).sum() / p["T"]
        p["Wo"][idx] = keep - h
        fm = -(p["adv"][:, None] * _logp_all(p).reshape(p["T"], p["N"], p["A"]).sum(-1)).sum() / p["T"]
        p["Wo"][idx] = keep
        assert abs((fp - fm) / (2 * h) - out["dWo"][idx]) < 1e-7
    assert chunk_logp.shape == (p["T"], p["N"])
    # a mask that keeps everything, given in sampler form, is bit-identical
    kept2, _, _ = O.sample_chunks(np.ones(2), np.zeros((p["T"], p["N"]), dtype=np.uint8), None, None,
                                  p["N"], seed=0, step=0)
    out2 = _call(p, kept2, lp_all, loss_scale=1.0 / p["T"])
    for k in ("loss", "dWg", "dWu", "dWd", "dWo", "dX"):
        assert np.array_equal(out[k], out2[k])


def test_uniform_rewards_give_zero_gradient():
    p = _problem(seed=4)
    p["adv"], _ = O.advantages(np.ones(p["T"], dtype=np.uint8), 4)
    out = _call(p, np.arange(0, 20, 3), _logp_all(p) + 0.05)
    for k in ("dWg", "dWu", "dWd", "dWo", "dX"):
        assert not out[k].any()
    assert out["loss"] == 0.0


def test_dz_rows_sum_to_zero_and_clipped_rows_vanish():
    p = _problem(seed=5)
    lp = _logp_all(p)
    r = np.random.default_rng(9)
    logp_old = lp + r.uniform(-0.6, 0.6, size=lp.shape)    # ratios spread over [0.55, 1.8]
    kept = np.arange(p["T"] * p["N"])
    out = _call(p, kept, logp_old, eps_low=0.2, eps_high=0.2)
    assert np.allclose(out["dz"].sum(1), 0, atol=1e-14)
    adv_row = np.repeat(p["adv"][kept // p["N"]], p["A"])
    rho = out["ratio"]
    dead = ((adv_row > 0) & (rho > 1.2)) | ((adv_row < 0) & (rho < 0.8))
    assert dead.any() and (~dead).any()
    assert not out["dz"][dead].any() and not out["dX"][dead].any()
    assert np.abs(out["dz"][~dead]).sum(1).min() > 0
    assert np.isclose(out["stats"][0], dead.mean())
    assert np.isclose(out["stats"][1], rho.mean())


def test_gradient_additive_over_groups_and_linear_in_advantage():
    p = _problem(seed=6, T=8)
    lp = _logp_all(p) + 0.01
    kept = np.arange(p["T"] * p["N"])[::2]
    whole = _call(p, kept, lp)
    first = _call(p, kept[kept // p["N"] < 4], lp)
    second = _call(p, kept[kept // p["N"] >= 4], lp)
    for k in ("dWg", "dWu", "dWd", "dWo"):
        assert np.allclose(whole[k], first[k] + second[k], rtol=1e-12, atol=1e-14)
    assert np.allclose(whole["dX"], np.concatenate([first["dX"], second["dX"]]), rtol=1e-13, atol=0)
    p2 = dict(p, adv=3.0 * p["adv"])
    tripled = _call(p2, kept, lp)
    assert np.allclose(tripled["dWd"], 3.0 * whole["dWd"], rtol=1e-12, atol=1e-14)


def test_dropping_zero_advantage_trajectories_changes_nothing():
    # compaction drops trajectories of collapsed groups; their terms are exactly zero
    p = _problem(seed=7, T=8)
    reward = np.array([1, 0, 0, 1, 1, 1, 1, 1], dtype=np.uint8)
    p["adv"], active = O.advantages(reward, 4)
    lp = _logp_all(p) - 0.02
    kept_all = np.arange(p["T"] * p["N"])
    kept_act = kept_all[active[kept_all // p["N"]] == 1]
    a, b = _call(p, kept_all, lp), _call(p, kept_act, lp)
    assert a["loss"] == b["loss"]
    for k in ("dWg", "dWu", "dWd", "dWo"):
        assert np.allclose(a[k], b[k], rtol=1e-13, atol=1e-16)


# ---- variants of the training loss (App. D: entropy bonus, token mean; per-chunk ratio; chunk weights) ----

def _fd_check(p, kept, logp_old, kw, r, names=("Wg", "Wd", "Wo", "hidden"), n=4):
    ref = _call(p, kept, logp_old, **kw)
    h = 1e-6
    for name in names:
        W = p[name]
        for _ in range(n):
            if name == "hidden":
                kr = int(r.integers(0, len(ref["rows"])))
                idx = (int(ref["rows"][kr]), int(r.integers(0, W.shape[1])))
                analytic = ref["dX"][kr, idx[1]]
            else:
                idx = tuple(int(r.integers(0, s)) for s in W.shape)
                analytic = ref["d" + name][idx]
            keep = W[idx]
            W[idx] = keep + h
            lp = _call(p, kept, logp_old, want_grads=False, **kw)["loss"]
            W[idx] = keep - h
            lm = _call(p, kept, logp_old, want_grads=False, **kw)["loss"]
            W[idx] = keep
            fd = (lp - lm) / (2 * h)
            assert abs(fd - analytic) <= 2e-6 * max(1.0, abs(analytic)) + 1e-8, (name, idx, fd, analytic)
    return ref


@pytest.mark.parametrize("kw", [
    dict(entropy_coef=0.05),
    dict(token_mean=True),
    dict(chunk_ratio=True),
    dict(chunk_weight="random"),
    dict(entropy_coef=1e-3, token_mean=True, chunk_ratio=True, chunk_weight="random", eps_low=0.2, eps_high=0.4),
])
def test_variant_gradients_match_finite_differences(kw):
    p = _problem(seed=11)
    r = np.random.default_rng(12)
    old = {k: p[k] + 0.05 * r.standard_normal(p[k].shape) for k in ("Wg", "Wu", "Wd", "Wo")}
    logp_old = _logp_all(p, old)
    kept = np.array([1, 2, 5, 8, 9, 13, 17, 19])
    kw = dict(kw)
    if isinstance(kw.get("chunk_weight"), str):
        kw["chunk_weight"] = r.uniform(0.5, 4.0, size=len(kept))
    kw.setdefault("loss_scale", 0.25)
    ref = _fd_check(p, kept, logp_old, kw, r)
    if kw.get("chunk_ratio"):
        flows_frac = 1 - ref["stats"][0]
        assert 0.05 < flows_frac < 0.95                   # per-chunk ratios do reach both clip branches here


def test_entropy_of_uniform_logits_is_log_V_and_enters_with_a_minus_sign():
    p = _problem(seed=13)
    p["Wo"] = np.zeros_like(p["Wo"])                       # z = 0: uniform distribution over V bins
    V = p["Wo"].shape[1]
    kept = np.array([0, 4, 6])
    lp_all = _logp_all(p)
    assert np.allclose(lp_all, -np.log(V))
    base = _call(p, kept, lp_all, loss_scale=0.5, want_grads=False)
    ent = _call(p, kept, lp_all, loss_scale=0.5, entropy_coef=0.1, want_grads=False)
    M = len(kept) * p["A"]
    assert np.allclose(ent["entropy"], np.log(V), rtol=1e-14)
    assert np.isclose(base["loss"] - ent["loss"], 0.1 * 0.5 * M * np.log(V), rtol=1e-13)
    assert np.isclose(ent["stats"][4], np.log(V), rtol=1e-14)
    # entropy is maximal at the uniform distribution: its gradient in the logits vanishes there
    full = _call(p, kept, lp_all, loss_scale=0.5, entropy_coef=0.1)
    plain = _call(p, kept, lp_all, loss_scale=0.5)
    assert np.allclose(full["dz"], plain["dz"], atol=1e-16)


def test_entropy_matches_scipy_on_random_logits():
    from scipy.stats import entropy as scipy_entropy
    p = _problem(seed=14)
    kept = np.array([2, 3, 10])
    out = _call(p, kept, _logp_all(p), entropy_coef=1.0, want_grads=False)
    rows = out["rows"]
    *_, z = O.head_forward(p["hidden"][rows], p["Wg"], p["Wu"], p["Wd"], p["Wo"])
    pr = np.exp(z - logsumexp(z, axis=1, keepdims=True))
    assert np.allclose(out["entropy"], scipy_entropy(pr, axis=1), rtol=1e-12)


def test_token_mean_is_the_sum_divided_by_the_number_of_kept_rows():
    p = _problem(seed=15)
    r = np.random.default_rng(16)
    logp_old = _logp_all(p) + 0.1 * r.standard_normal(p["hidden"].shape[0])
    kept = np.array([0, 1, 7, 12, 13])
    M = len(kept) * p["A"]
    a = _call(p, kept, logp_old, loss_scale=2.0, token_mean=True, entropy_coef=0.01)
    b = _call(p, kept, logp_old, loss_scale=2.0 / M, entropy_coef=0.01)
    assert np.isclose(a["loss"], b["loss"], rtol=1e-14)
    for k in ("dWg", "dWo", "dX"):
        assert np.allclose(a[k], b[k], rtol=1e-13, atol=1e-18)
    empty = _call(p, np.array([], dtype=np.int64), logp_old, token_mean=True)
    assert empty["loss"] == 0.0


def test_chunk_ratio_is_the_ratio_of_chunk_probabilities():
    p = _problem(seed=17)
    r = np.random.default_rng(18)
    logp_old = _logp_all(p) + 0.05 * r.standard_normal(p["hidden"].shape[0])
    kept = np.array([3, 4, 9, 15])
    A = p["A"]
    out = _call(p, kept, logp_old, chunk_ratio=True, eps_low=0.2, eps_high=0.4, loss_scale=1.0)
    lp = _logp_all(p)
    total = 0.0
    for j, c in enumerate(kept):
        rows = np.arange(c * A, (c + 1) * A)
        ratio = np.exp(lp[rows].sum()) / np.exp(logp_old[rows].sum())     # pi(chunk) / pi_old(chunk)
        assert np.allclose(out["ratio"][j * A:(j + 1) * A], ratio, rtol=1e-12)
        adv = p["adv"][c // p["N"]]
        total += min(ratio * adv, np.clip(ratio, 0.8, 1.4) * adv)
    assert np.isclose(out["loss"], -total, rtol=1e-12)
    # with one token per chunk the two forms coincide
    q = _problem(seed=19, A=1)
    lo = _logp_all(q) + 0.1 * r.standard_normal(q["hidden"].shape[0])
    k1 = np.array([0, 2, 5, 11])
    a = _call(q, k1, lo, chunk_ratio=True)
    b = _call(q, k1, lo)
    assert np.isclose(a["loss"], b["loss"], rtol=1e-14) and np.allclose(a["dWo"], b["dWo"], rtol=1e-13, atol=1e-18)


def test_chunk_weights_reweight_each_chunks_contribution():
    p = _problem(seed=20)
    r = np.random.default_rng(21)
    logp_old = _logp_all(p) + 0.05 * r.standard_normal(p["hidden"].shape[0])
    kept = np.array([1, 6, 14])
    ones = _call(p, kept, logp_old, chunk_weight=np.ones(3))
    none = _call(p, kept, logp_old)
    assert ones["loss"] == none["loss"] and np.array_equal(ones["dWg"], none["dWg"])
    # the weighted objective is the weighted sum of the single-chunk objectives
    w = np.array([0.5, 2.0, 3.5])
    whole = _call(p, kept, logp_old, chunk_weight=w)
    parts = [_call(p, kept[j:j + 1], logp_old) for j in range(3)]
    assert np.isclose(whole["loss"], sum(wj * pj["loss"] for wj, pj in zip(w, parts)), rtol=1e-13)
    assert np.allclose(whole["dWd"], sum(wj * pj["dWd"] for wj, pj in zip(w, parts)), rtol=1e-12, atol=1e-16)
