"""GPU parity of grpo_masked_actor_step_ex (loss variants of App. D and App. C) against the checker.

fp32 path: relative 1e-5 as for the plain step; with a per-chunk ratio the chunk's log-ratio is a sum
of A = 56 fp32 row values, so the ratio itself carries A times the rounding of one row and the bound
used is 5e-5.
bf16 path: relative Frobenius 2e-2 as for the plain step, the per-chunk ratio included, at chunk lengths 4, 16
and 56 (with a per-chunk ratio the library carries the activations as value + remainder through the down and
the logit product, so that the sum of a chunk's log-probabilities is accurate to 1e-3).
Inputs are conditioned so that no ratio sits within the stated margin of a clip threshold: the clip
decision is a discrete one and both sides must take the same branch.
"""
import numpy as np
import pytest
import torch

from oracle import pcm_oracle as O
from workloads import CONFIGS, make_rollouts

from test_gpu_actor import BF16_TOL, check, composed, make_problem, run_both  # noqa: E402,F401

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pcm():
    import paper_2605_16154_amd as m
    m.lib()
    return m


def condition_chunks(pr, eps, margin):
    """Shift logp_old of the first row of chunks whose log chunk-ratio is within `margin` of a threshold."""
    cfg, W = pr["cfg"], pr["W"]
    cur = O.actor_step(pr["hidden"], pr["tokens"], pr["logp_old"], pr["adv"], pr["kept"], cfg.N, cfg.A,
                       W["Wg"], W["Wu"], W["Wd"], W["Wo"], want_grads=False)
    delta = (cur["logp"] - pr["logp_old"][cur["rows"]].astype(np.float64)).reshape(-1, cfg.A).sum(axis=1)
    lo = pr["logp_old"].astype(np.float64)
    for thr in (np.log1p(-eps[0]), np.log1p(eps[1])):
        near = np.abs(delta - thr) < margin
        first_rows = cur["rows"].reshape(-1, cfg.A)[near, 0]
        lo[first_rows] -= np.where(delta[near] >= thr, 2 * margin, -2 * margin)
    pr["logp_old"] = lo.astype(np.float32)
    return pr


def weights_for(pr, seed):
    return np.random.default_rng(seed).uniform(0.5, 4.0, size=len(pr["kept"]))


VARIANTS = [
    ("entropy", dict(entropy_coef=0.05)),
    ("token_mean", dict(token_mean=True)),
    ("chunk_weight", dict(chunk_weight="random")),
    ("paper_defaults", dict(entropy_coef=1e-3, token_mean=True)),
]


@pytest.mark.parametrize("name,variants", VARIANTS)
def test_fp32_cfg1_variants(pcm, name, variants):
    pr = make_problem(CONFIGS["cfg1"], margin=1e-3, eps=(0.2, 0.4))
    variants = dict(variants)
    if isinstance(variants.get("chunk_weight"), str):
        variants["chunk_weight"] = weights_for(pr, 3)
    scale = 3.0 if variants.get("token_mean") else None
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), scale=scale, variants=variants)
    check(ref, got, 1e-5, len(ref["rows"]), n_stats=5)


def test_fp32_chunk_ratio_alone_and_with_everything(pcm, composed):
    cfg = CONFIGS["cfg1"]
    pr = make_problem(cfg, wstd=0.05, old_rel=0.1, eps=(0.2, 0.4))
    pr = condition_chunks(pr, (0.2, 0.4), 1e-3)
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), variants=dict(chunk_ratio=True))
    assert 0.05 < ref["stats"][0] < 0.95                      # chunk ratios fall on both sides of the clip
    check(ref, got, 5e-5, len(ref["rows"]), stats_tol=5e-5, n_stats=5)
    everything = dict(chunk_ratio=True, token_mean=True, entropy_coef=1e-3, chunk_weight=weights_for(pr, 4))
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), scale=2.0, variants=everything, max_kept=len(pr["kept"]) + 3,
                        composed_head=composed)
    check(ref, got, 5e-5, len(ref["rows"]), stats_tol=5e-5, n_stats=5)


def test_fp32_ragged_shapes_with_everything(pcm):
    cfg = CONFIGS["cfg1"].with_(n_groups=3, G=4, N=9, K=3, B=4, d=72, ff=200, V=101, L=3, D=5, seed=8)
    pr = make_problem(cfg, wstd=0.12, eps=(0.2, 0.4), old_rel=0.05)
    pr = condition_chunks(pr, (0.2, 0.4), 1e-3)
    everything = dict(chunk_ratio=True, token_mean=True, entropy_coef=0.02, chunk_weight=weights_for(pr, 5))
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), variants=everything, max_kept=len(pr["kept"]) + 5)
    check(ref, got, 5e-5, len(ref["rows"]), stats_tol=5e-5, n_stats=5)
    # forward only and empty kept list
    _, fwd = run_both(pcm, pr, eps=(0.2, 0.4), variants=everything, max_kept=len(pr["kept"]) + 5,
                      want_grads=False, want_dX=False)
    assert fwd["loss"][0] == got["loss"][0]
    pr0 = dict(pr, kept=pr["kept"][:0])
    ref0, got0 = run_both(pcm, pr0, eps=(0.2, 0.4), variants=dict(chunk_ratio=True, token_mean=True, entropy_coef=0.02),
                          max_kept=4)
    assert got0["loss"][0] == 0.0 and not got0["dWg"].any() and not got0["dX"].any()


def _bf16_problem(A_dims=None, seed=21, n_kept=37):
    kw = dict(n_groups=2, G=4, N=16, K=4, B=5, d=512, ff=768, seed=seed)
    if A_dims:
        kw.update(L=A_dims[0], D=A_dims[1])
    cfg = CONFIGS["cfg2"].with_(**kw)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, seed, 0)
    return cfg, kept[:n_kept]


def test_bf16_token_level_variants(pcm, composed):
    cfg, kept = _bf16_problem()
    pr = make_problem(cfg, wstd=0.05, margin=0.08, kept=kept, old_rel=0.1, eps=(0.2, 0.4))
    variants = dict(entropy_coef=0.05, token_mean=True, chunk_weight=weights_for(pr, 6))
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), scale=50.0, torch_dtype=torch.bfloat16, max_kept=40, variants=variants,
                        composed_head=composed)
    assert 0.05 < ref["stats"][0] < 0.95
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2, n_stats=5)
    # the entropy term alone (zero advantages): gradients come from the entropy bonus only
    pr["adv"] = np.zeros(cfg.T)
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), scale=50.0, torch_dtype=torch.bfloat16, max_kept=40,
                        variants=dict(entropy_coef=0.05, token_mean=True))
    assert np.abs(ref["dWo"]).max() > 0
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2, n_stats=5)


@pytest.mark.parametrize("A_dims,n_kept", [((2, 2), 40), ((4, 4), 40), ((8, 7), 37)])
def test_bf16_chunk_ratio_matches_checker_at_any_chunk_length(pcm, A_dims, n_kept):
    # A = 4, 16 and the paper's 56 tokens per chunk (Sec. 5.1), all at the bound of the per-token form: with one
    # ratio per chunk the library carries a and y as value + remainder through the down and the logit product
    cfg, kept = _bf16_problem(A_dims=A_dims, seed=22, n_kept=n_kept)
    assert cfg.A == A_dims[0] * A_dims[1]
    pr = make_problem(cfg, wstd=0.05, kept=kept, old_rel=0.1 if cfg.A < 56 else 0.03, eps=(0.2, 0.4))
    pr = condition_chunks(pr, (0.2, 0.4), 0.02)
    variants = dict(chunk_ratio=True, entropy_coef=0.02, token_mean=True, chunk_weight=weights_for(pr, 7))
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), scale=20.0, torch_dtype=torch.bfloat16, max_kept=n_kept + 8,
                        variants=variants)
    assert 0.05 < ref["stats"][0] < 0.95
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=2e-2, n_stats=5)
    # the log-ratio of a chunk is a sum of A log-probabilities: its error must stay far below the clip margin
    n = len(ref["rows"])
    chunk_err = np.abs((got["logp"][:n] - ref["logp"]).reshape(-1, cfg.A).sum(axis=1))
    assert chunk_err.max() < 5e-3, chunk_err.max()
    # forward only: same loss, no gradient buffers
    _, fwd = run_both(pcm, pr, eps=(0.2, 0.4), scale=20.0, torch_dtype=torch.bfloat16, max_kept=n_kept + 8,
                      variants=variants, want_grads=False, want_dX=False)
    assert fwd["loss"][0] == got["loss"][0] and np.array_equal(fwd["logp"], got["logp"])


def test_bf16_chunk_ratio_with_the_composed_head_is_refused(pcm):
    # the value + remainder forward pass exists for the head as written; the combination says so instead of
    # returning gradients outside the bound
    cfg, kept = _bf16_problem(A_dims=(2, 2), seed=22, n_kept=8)
    pr = make_problem(cfg, wstd=0.05, kept=kept, old_rel=0.1)
    with pytest.raises(pcm.PcmError, match="unsupported"):
        run_both(pcm, pr, torch_dtype=torch.bfloat16, variants=dict(chunk_ratio=True), composed_head=True)


def test_bf16_chunk_ratio_of_one_has_the_token_forms_gradient(pcm):
    # logp_old taken from the library's own forward pass of the same form: every ratio is exactly 1 at either
    # level.  The derivative of a chunk's term in each of its rows' log-probabilities is then A_i, as in the
    # per-token form, so the per-chunk path (separate ratio kernel + row scaling) must reproduce the gradients of
    # the fused per-token path; the loss value has one term per chunk instead of one per row.
    cfg, kept = _bf16_problem(seed=23)
    pr = make_problem(cfg, wstd=0.05, kept=kept, old_rel=0.1)
    rows = (pr["kept"].astype(np.int64)[:, None] * cfg.A + np.arange(cfg.A)[None, :]).reshape(-1)
    out = {}
    for form, variants in (("tok", {}), ("chk", dict(chunk_ratio=True))):
        _, fwd = run_both(pcm, pr, torch_dtype=torch.bfloat16, want_grads=False, want_dX=False, variants=variants)
        own = dict(pr, logp_old=pr["logp_old"].copy())
        own["logp_old"][rows] = fwd["logp"][:len(rows)]
        _, out[form] = run_both(pcm, own, torch_dtype=torch.bfloat16, variants=dict(variants, entropy_coef=0.01))
        _, out[form + "0"] = run_both(pcm, own, torch_dtype=torch.bfloat16, want_grads=False, want_dX=False,
                                      variants=variants)
        assert np.allclose(out[form]["stats"][:2], [0.0, 1.0], atol=1e-6), form
    for k in ("dWg", "dWu", "dWd", "dWo", "dX"):
        den = np.linalg.norm(out["tok"][k])
        assert np.linalg.norm(out["tok"][k] - out["chk"][k]) <= 1e-2 * den, k     # two bf16 roundings of dz instead of one
    assert abs(out["tok0"]["loss"][0] - cfg.A * out["chk0"]["loss"][0]) <= 1e-5 * max(1.0, abs(out["tok0"]["loss"][0]))
