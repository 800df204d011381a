"""GPU parity of grpo_masked_actor_step (Eq. 11 / Eq. 2 with PPO clipping) against the CPU checker.

Tolerances: fp32 path relative 1e-5; bf16 path relative Frobenius 2e-2 on gradients (the GPU
rounds intermediates to bf16, the checker works in fp64 on the same bf16-valued inputs).  Beside the
per-tensor norms every row is checked on its own, so that a single wrong row cannot hide in the norm of
thousands: |logp - ref| <= tol * max(1, |ref|) for every row, and the row of dX within ROW_FACTOR * tol of
the reference row in relative 2-norm (a row's error is not averaged over anything, hence the factor); rows
whose reference gradient is exactly zero (clipped away) must be exactly zero.

The clip decision is discrete: a row whose ratio sits on a threshold flips its whole gradient
under the smallest perturbation.  Inputs are therefore conditioned so that no row's reference
ratio lies within the path's accuracy of a threshold (logp_old of such rows is moved away by a
fixed amount); both sides then take the same decisions and the comparison is well-posed.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pcm_oracle as O
from workloads import (CONFIGS, make_head_numpy, make_head_torch, make_hidden_numpy, make_hidden_torch,
                       make_rollouts, perturb_numpy, perturb_torch)

pytestmark = pytest.mark.gpu
GRADS = ("dWg", "dWu", "dWd", "dWo")


@pytest.fixture(scope="module")
def pcm():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_16154_amd as pcm
    pcm.lib()
    return pcm


@pytest.fixture(params=[False, True], ids=["as_written", "composed"])
def composed(request):
    """Both evaluations of the head: projections applied one after the other, or as the one matrix Wd Wo."""
    return request.param


def dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t if dtype is None else t.to(dtype)


def rel(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / den if den > 0 else np.linalg.norm(got)


def condition_logp_old(logp_old, logp_ref_rows, rows, eps_low, eps_high, margin):
    """Move logp_old of rows whose reference log-ratio is within `margin` of a clip threshold."""
    logp_old = logp_old.copy()
    lr = logp_ref_rows - logp_old[rows]
    for thr in (np.log1p(-eps_low), np.log1p(eps_high)):
        near = np.abs(lr - thr) < margin
        # push the ratio to the far side it is already on
        logp_old[rows[near]] -= np.where(lr[near] >= thr, 2 * margin, -2 * margin)
    return logp_old


def make_problem(cfg, wstd=0.02, margin=0.0, kept=None, seed_step=0, eps=(0.2, 0.2), old_rel=0.5):
    """Inputs of one actor step; old-policy weights = current + N(0, old_rel * wstd)."""
    ro = make_rollouts(cfg, seed_step)
    W = make_head_numpy(cfg, std=wstd)
    W_old = perturb_numpy(cfg, W, std=wstd * old_rel)
    hidden = make_hidden_numpy(cfg, seed_step)
    tokens = (ro["tokens"].reshape(-1).astype(np.int64) % cfg.V).astype(np.uint8)
    adv, active = O.advantages(ro["reward"], cfg.G)
    if kept is None:
        p = np.maximum(0.1, np.linspace(1.0, 0.05, cfg.K))
        kept, _, _ = O.sample_chunks(p, ro["phase"], ro["n_chunks"], active, cfg.B, cfg.seed, seed_step)
    zeros = np.zeros(hidden.shape[0])
    old = O.actor_step(hidden, tokens, zeros, adv, kept, cfg.N, cfg.A, W_old["Wg"], W_old["Wu"], W_old["Wd"],
                       W_old["Wo"], want_grads=False)
    logp_old = np.zeros(hidden.shape[0])
    logp_old[old["rows"]] = old["logp"]
    if margin > 0:
        cur = O.actor_step(hidden, tokens, zeros, adv, kept, cfg.N, cfg.A, W["Wg"], W["Wu"], W["Wd"], W["Wo"],
                           want_grads=False)
        logp_old = condition_logp_old(logp_old, cur["logp"], cur["rows"], eps[0], eps[1], margin)
    logp_old = logp_old.astype(np.float32)
    return dict(cfg=cfg, hidden=hidden, tokens=tokens, adv=adv, kept=kept.astype(np.int32), W=W, logp_old=logp_old)


def run_both(pcm, pr, eps=(0.2, 0.2), scale=None, torch_dtype=torch.float32, max_kept=None, variants=None, **kw):
    """The same step through the checker and through the library.  `variants`: loss options given to both
    (token_mean, entropy_coef, chunk_ratio, chunk_weight as a numpy array over the kept chunks)."""
    cfg, W = pr["cfg"], pr["W"]
    scale = 1.0 / cfg.T if scale is None else scale
    variants = dict(variants or {})
    ref = O.actor_step(pr["hidden"], pr["tokens"], pr["logp_old"], pr["adv"], pr["kept"], cfg.N, cfg.A,
                       W["Wg"], W["Wu"], W["Wd"], W["Wo"], eps[0], eps[1], scale, **variants)
    kept = pr["kept"]
    max_kept = len(kept) if max_kept is None else max_kept
    kept_buf = np.full(max_kept, -7, dtype=np.int32)       # tail entries are garbage on purpose
    kept_buf[:len(kept)] = kept
    if variants.get("chunk_weight") is not None:
        wbuf = np.full(max_kept, 1e30, dtype=np.float32)   # so are the weights beyond the kept count
        wbuf[:len(kept)] = variants["chunk_weight"]
        variants["chunk_weight"] = dev(wbuf)
    kw.update(variants)
    out = pcm.grpo_masked_actor_step(
        dev(pr["hidden"], torch_dtype), dev(pr["tokens"]), dev(pr["logp_old"]), dev(pr["adv"].astype(np.float32)),
        dev(kept_buf), dev(np.array([len(kept)], np.int32)), cfg.T, cfg.N, cfg.A,
        *(dev(W[k], torch_dtype) for k in ("Wg", "Wu", "Wd", "Wo")), eps[0], eps[1], scale,
        max_kept_chunks=max_kept, **kw)
    torch.cuda.synchronize()
    return ref, {k: (v.double() if v.dtype == torch.float64 else v.float()).cpu().numpy() for k, v in out.items()}


ROW_FACTOR = 2.5


def check_rows(logp, dX, ref_logp, ref_dX, tol):
    """Row-by-row bounds on the per-row outputs (every row, not a norm over rows)."""
    logp, ref_logp = np.asarray(logp, np.float64), np.asarray(ref_logp, np.float64)
    bad = np.abs(logp - ref_logp) > tol * np.maximum(1.0, np.abs(ref_logp))
    assert not bad.any(), ("logp rows", np.flatnonzero(bad)[:8], np.abs(logp - ref_logp).max())
    if dX is None:
        return
    dX, ref_dX = np.asarray(dX, np.float64), np.asarray(ref_dX, np.float64)
    ref_norm = np.linalg.norm(ref_dX, axis=1)
    err = np.linalg.norm(dX - ref_dX, axis=1)
    zero = ref_norm == 0.0
    assert not err[zero].any(), ("rows with zero reference gradient", np.flatnonzero(zero & (err > 0))[:8])
    # rows whose gradient is more than six orders below the largest carry no weight in any sum: bounded absolutely
    scale = np.maximum(ref_norm, 1e-6 * ref_norm.max() if ref_norm.size else 0.0)
    bad = err > ROW_FACTOR * tol * scale
    assert not bad.any(), ("dX rows", np.flatnonzero(bad)[:8], (err / np.maximum(scale, 1e-300)).max())


def check(ref, got, tol, n_rows, stats_tol=None, n_stats=4):
    stats_tol = max(tol, 1e-5) if stats_tol is None else stats_tol
    assert abs(got["loss"][0] - ref["loss"]) <= tol * max(1.0, abs(ref["loss"])), (got["loss"], ref["loss"])
    assert rel(got["logp"][:n_rows], ref["logp"]) <= tol
    for k in GRADS:
        assert rel(got[k], ref[k]) <= tol, (k, rel(got[k], ref[k]))
    assert rel(got["dX"][:n_rows], ref["dX"]) <= tol, rel(got["dX"][:n_rows], ref["dX"])
    check_rows(got["logp"][:n_rows], got["dX"][:n_rows], ref["logp"], ref["dX"], tol)
    assert np.allclose(got["stats"][:n_stats], ref["stats"][:n_stats], rtol=stats_tol, atol=stats_tol), \
        (got["stats"], ref["stats"])


# ------------------------------------------------------------------------------------------ fp32

def test_fp32_cfg1_matches_checker(pcm, composed):
    pr = make_problem(CONFIGS["cfg1"])
    ref, got = run_both(pcm, pr, composed_head=composed)
    lr = np.log(ref["ratio"])
    assert np.min(np.abs(lr - np.log(0.8))) > 1e-4 and np.min(np.abs(lr - np.log(1.2))) > 1e-4
    check(ref, got, 1e-5, len(ref["rows"]))


def test_fp32_ragged_shapes_clipping_and_padding(pcm, composed):
    # sizes that are not multiples of any tile, asymmetric clip, kept list shorter than its buffer
    cfg = CONFIGS["cfg1"].with_(n_groups=3, G=4, N=9, K=3, B=4, d=72, ff=200, V=101, L=3, D=5, seed=8)
    # weights N(0, 0.2) against an old policy half a standard deviation away: logits of order 30, ratios up to
    # 1e35 on the rows the clip lets through.  (At N(0, 0.3) the largest ratio is 2e188, which no fp32 value
    # holds: the library's loss is inf there by construction of the arithmetic, so that scale is no parity case.)
    pr = make_problem(cfg, wstd=0.2, margin=1e-3, eps=(0.2, 0.4))
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), max_kept=len(pr["kept"]) + 5, composed_head=composed)
    assert 0.02 < ref["stats"][0] < 0.98                      # both sides of the clip occur
    check(ref, got, 1e-5, len(ref["rows"]))
    # the same shapes in the regime the method runs in (ratios of order one)
    pr = make_problem(cfg, wstd=0.12, margin=1e-3, eps=(0.2, 0.4), old_rel=0.3)
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), max_kept=len(pr["kept"]) + 5, composed_head=composed)
    assert 0.02 < ref["stats"][0] < 0.98
    check(ref, got, 1e-5, len(ref["rows"]))


def test_fp32_all_kept_equals_unmasked_and_forward_only(pcm):
    cfg = CONFIGS["cfg1"].with_(n_groups=1, N=8, B=8, d=64, ff=128)
    kept = np.arange(cfg.T * cfg.N)
    pr = make_problem(cfg, wstd=0.2, kept=kept, margin=1e-3)
    ref, got = run_both(pcm, pr)
    check(ref, got, 1e-5, len(ref["rows"]))
    # kept ids produced by the sampler with B >= N are the same list: identical output
    k2, _, nk = pcm.pcm_sample_chunks(dev(np.ones(cfg.K)), dev(np.zeros((cfg.T, cfg.N), np.uint8)), None, None,
                                      cfg.N, 0, 0)
    assert np.array_equal(k2.cpu().numpy(), kept)
    # forward only: loss and logp without any gradient buffer
    _, fwd = run_both(pcm, pr, want_grads=False, want_dX=False)
    assert fwd["loss"][0] == got["loss"][0] and np.array_equal(fwd["logp"], got["logp"])
    assert "dWg" not in fwd and "dX" not in fwd


def test_fp32_uniform_rewards_and_empty_kept_list(pcm):
    cfg = CONFIGS["cfg1"].with_(n_groups=1, N=8, B=3, d=64, ff=128)
    pr = make_problem(cfg, wstd=0.2, kept=np.array([1, 5, 9, 20]))
    pr["adv"] = np.zeros(cfg.T)                               # a collapsed group: every advantage is zero
    ref, got = run_both(pcm, pr)
    for k in GRADS + ("dX",):
        assert not got[k].any()
    assert got["loss"][0] == 0.0
    pr["kept"] = np.zeros(0, np.int32)                        # nothing kept at all
    pr["adv"] = np.ones(cfg.T)
    _, got = run_both(pcm, pr, max_kept=4)
    assert got["loss"][0] == 0.0 and got["stats"][3] == 0.0
    for k in GRADS:
        assert not got[k].any()


# ------------------------------------------------------------------------------------------ bf16

BF16_TOL = 2e-2


def test_bf16_small_head_matches_checker(pcm, composed):
    # several 256-row tiles plus a ragged tail (37 chunks * 56 = 2072 rows), 2 x 3 x 1 weight tiles
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=4, N=16, K=4, B=5, d=512, ff=768, seed=12)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, 12, 0)
    kept = kept[:37]
    pr = make_problem(cfg, wstd=0.05, margin=0.08, kept=kept, old_rel=0.1)
    ref, got = run_both(pcm, pr, torch_dtype=torch.bfloat16, max_kept=40, composed_head=composed)
    assert 0.05 < ref["stats"][0] < 0.95
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2)


@pytest.mark.parametrize("d,ff,n_kept,A_dims", [
    (256, 256, 3, (8, 7)),        # a single row tile, mostly padding; one tile in every weight dimension
    (768, 1280, 23, (8, 7)),      # 3 x 5 weight tiles, 1288 rows = 5 row tiles + ragged tail
    (512, 256, 64, (2, 2)),       # short chunks: 256 rows, exactly one full row tile
    (256, 1024, 40, (4, 4)),      # 640 rows: the row count is a multiple of 64 but not of 256
])
def test_bf16_shape_sweep(pcm, d, ff, n_kept, A_dims, composed):
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=4, N=16, K=4, B=8, d=d, ff=ff, L=A_dims[0], D=A_dims[1], seed=40 + n_kept)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, cfg.seed, 0)
    assert len(kept) >= n_kept
    # weight scale chosen so that logits stay O(1): the bf16 error of a log-probability grows with the logit scale
    pr = make_problem(cfg, wstd=0.04, margin=0.08, kept=kept[:n_kept], old_rel=0.2, eps=(0.2, 0.4))
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), torch_dtype=torch.bfloat16, max_kept=n_kept + 2, composed_head=composed)
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2)


def test_bf16_all_kept_and_forward_only(pcm, composed):
    cfg = CONFIGS["cfg2"].with_(n_groups=1, G=4, N=6, K=3, B=6, d=256, ff=256, seed=13)
    pr = make_problem(cfg, wstd=0.08, margin=0.08, kept=np.arange(cfg.T * cfg.N), old_rel=0.1)
    ref, got = run_both(pcm, pr, torch_dtype=torch.bfloat16, composed_head=composed)
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2)
    _, fwd = run_both(pcm, pr, torch_dtype=torch.bfloat16, want_grads=False, want_dX=False, composed_head=composed)
    assert fwd["loss"][0] == got["loss"][0] and np.array_equal(fwd["logp"], got["logp"])
    pr["adv"] = np.zeros(cfg.T)
    _, zero = run_both(pcm, pr, torch_dtype=torch.bfloat16, composed_head=composed)
    for k in GRADS + ("dX",):
        assert not zero[k].any()


def test_bf16_packed_weights_give_the_same_step(pcm):
    """The operand layouts of the weights written once by pcm_pack_head_weights and handed to the step: the same
    kernels read the same bytes, so every output is bit for bit what the step computes when it lays the weights out
    itself; stale layouts (weights changed, not re-packed) are the caller's responsibility and do change the result."""
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=4, N=16, K=4, B=5, d=512, ff=768, seed=12)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, 12, 0)
    pr = make_problem(cfg, wstd=0.05, margin=0.08, kept=kept[:37], old_rel=0.1)
    ref, own = run_both(pcm, pr, torch_dtype=torch.bfloat16, max_kept=40)
    W = {k: dev(v, torch.bfloat16) for k, v in pr["W"].items()}
    packed = pcm.pcm_pack_head_weights(W["Wg"], W["Wu"], W["Wd"], W["Wo"])
    _, given = run_both(pcm, pr, torch_dtype=torch.bfloat16, max_kept=40, packed_weights=packed)
    n = len(ref["rows"])                                        # rows beyond the kept ones are left untouched
    for k in GRADS + ("loss",):
        assert np.array_equal(given[k], own[k]), k
    assert np.array_equal(given["stats"][:4], own["stats"][:4])     # the extended entry point also fills stats[4]
    assert np.array_equal(given["logp"][:n], own["logp"][:n]) and np.array_equal(given["dX"][:n], own["dX"][:n])
    check(ref, given, BF16_TOL, n, stats_tol=5e-2)
    stale = pcm.pcm_pack_head_weights(W["Wg"] * 2, W["Wu"], W["Wd"], W["Wo"])
    _, other = run_both(pcm, pr, torch_dtype=torch.bfloat16, max_kept=40, packed_weights=stale)
    assert not np.array_equal(other["logp"][:n], own["logp"][:n])
    with pytest.raises(pcm.PcmError, match="unsupported"):
        run_both(pcm, pr, torch_dtype=torch.bfloat16, max_kept=40, packed_weights=packed, composed_head=True)


def test_bf16_short_kept_list_after_a_long_one(pcm, composed):
    """The kept count lives on the device: a call that keeps few chunks after one that kept many (same
    buffers, same workspace) must not see anything the earlier call left behind in the skipped row tiles."""
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=4, N=16, K=4, B=10, d=256, ff=512, seed=14)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept_long, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, 14, 0)
    assert len(kept_long) == 80                                  # 4480 rows = 18 row tiles
    pr_long = make_problem(cfg, wstd=0.07, margin=0.08, kept=kept_long, old_rel=0.1)
    ref_long, got_long = run_both(pcm, pr_long, torch_dtype=torch.bfloat16, max_kept=80, composed_head=composed)
    check(ref_long, got_long, BF16_TOL, len(ref_long["rows"]), stats_tol=5e-2)
    for n_short in (37, 5, 0):                                   # 9 tiles with a ragged tail, 2 tiles, none
        pr = dict(pr_long, kept=kept_long[::2][:n_short].astype(np.int32))
        ref, got = run_both(pcm, pr, torch_dtype=torch.bfloat16, max_kept=80, composed_head=composed)
        if n_short:
            check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2)
        else:
            assert got["loss"][0] == 0.0 and not any(got[k].any() for k in GRADS)


def chunk_rows(chunks, A):
    """Row indices (into the [T*N*A] arrays) of the A tokens of each chunk id, in order."""
    return (np.asarray(chunks, np.int64)[:, None] * A + np.arange(A)[None, :]).reshape(-1)


def conditioned_logp_old(hidden_rows, tokens_rows, lp_old_rows, adv_chunks, A, Wn, eps, margin):
    """logp_old of the given rows moved away from the clip thresholds of the checker's ratios (see the module text)."""
    cur = O.actor_step(hidden_rows, tokens_rows, lp_old_rows, adv_chunks, np.arange(len(adv_chunks)), 1, A,
                       Wn["Wg"], Wn["Wu"], Wn["Wd"], Wn["Wo"], want_grads=False)
    return condition_logp_old(lp_old_rows, cur["logp"], np.arange(len(lp_old_rows)), eps[0], eps[1], margin)


@pytest.mark.parametrize("n_kept,variants", [(120, {}), (101, dict(chunk_ratio=True, entropy_coef=0.01, token_mean=True))])
def test_bf16_row_panels_add_up_to_the_whole_batch(pcm, n_kept, variants):
    """A batch worked through in row panels (here: panels of 1792 rows = 32 chunks, so 120 kept chunks are three full
    panels and a ragged fourth, 101 chunks end inside the fourth): every panel adds its weight gradients to the
    earlier ones', per-row outputs land at the panel's offset, the loss is reduced once over all rows.  Against the
    checker on the whole batch, and bit for bit against itself with a different kept count below the capacity."""
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=8, N=16, K=4, B=8, d=512, ff=768, seed=31)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, cfg.seed, 0)
    assert len(kept) == 128
    pr = make_problem(cfg, wstd=0.05, margin=0.08, kept=kept[:n_kept], old_rel=0.1, eps=(0.2, 0.4))
    if variants.get("chunk_ratio"):
        from test_gpu_actor_variants import condition_chunks
        pr = condition_chunks(pr, (0.2, 0.4), 0.02)
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), torch_dtype=torch.bfloat16, max_kept=128, variants=variants, panel_rows=1792)
    assert 0.05 < ref["stats"][0] < 0.95
    check(ref, got, BF16_TOL, len(ref["rows"]), stats_tol=5e-2)
    # one panel for everything (the default height) gives the same rows bit for bit; the weight gradients differ only
    # by the order of fp32 additions
    _, whole = run_both(pcm, pr, eps=(0.2, 0.4), torch_dtype=torch.bfloat16, max_kept=128, variants=variants)
    n = len(ref["rows"])
    assert np.array_equal(whole["logp"][:n], got["logp"][:n]) and np.array_equal(whole["dX"][:n], got["dX"][:n])
    for k in GRADS:
        assert rel(got[k], whole[k]) <= 1e-5, k


@pytest.mark.parametrize("n_kept,old_rel,variants,listed", [
    (120, 0.5, {}, True),                        # many clipped rows, four panels (the last one ragged)
    (101, 0.5, dict(chunk_ratio=True), True),    # one ratio per chunk: whole chunks drop out
    (120, 0.01, {}, False),                      # fewer than one row in sixteen clipped: all rows stay
    (120, 0.01, dict(chunk_weight="some_zero"), True),   # rows drop out through a zero chunk weight
])
def test_bf16_backward_over_the_rows_with_a_gradient(pcm, n_kept, old_rel, variants, listed):
    """Rows whose ratio the clip cuts have a zero row of dz: the backward products run over the other rows only
    (when enough drop out).  Against the checker, and against the library's own backward pass over all rows
    (dense_backward): per-row outputs bit for bit, weight gradients up to the order of the fp32 sums; also with
    only dX or only the weight gradients asked for."""
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=8, N=16, K=4, B=8, d=512, ff=768, seed=37)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, cfg.seed, 0)
    pr = make_problem(cfg, wstd=0.05, margin=0.08, kept=kept[:n_kept], old_rel=old_rel, eps=(0.2, 0.4))
    if variants.get("chunk_ratio"):
        from test_gpu_actor_variants import condition_chunks
        pr = condition_chunks(pr, (0.2, 0.4), 0.02)
    if variants.get("chunk_weight") is not None:
        rng = np.random.default_rng(5)
        variants = dict(chunk_weight=np.where(rng.random(n_kept) < 0.3, 0.0, rng.uniform(0.5, 4.0, n_kept)))
    kw = dict(eps=(0.2, 0.4), torch_dtype=torch.bfloat16, max_kept=128, variants=variants, panel_rows=1792)
    ref, got = run_both(pcm, pr, **kw)
    if "chunk_weight" not in variants:
        assert (ref["stats"][0] >= 1 / 8) if listed else (ref["stats"][0] < 1 / 32), ref["stats"]
    n = len(ref["rows"])
    check(ref, got, BF16_TOL, n, stats_tol=5e-2)
    _, dense = run_both(pcm, pr, dense_backward=True, **kw)
    assert np.array_equal(got["loss"], dense["loss"]) and np.array_equal(got["logp"][:n], dense["logp"][:n])
    assert np.array_equal(got["dX"][:n], dense["dX"][:n])
    for k in GRADS:
        assert rel(got[k], dense[k]) <= 1e-5, (k, rel(got[k], dense[k]))
    # the sum of the squares of the four weight gradients, gathered where their final values are written
    _, with_sq = run_both(pcm, pr, grad_sumsq=True, **kw)
    want = sum(float((with_sq[k].astype(np.float64) ** 2).sum()) for k in GRADS)
    assert abs(float(with_sq["grad_sumsq"][0]) - want) <= 2e-5 * want, (with_sq["grad_sumsq"], want)
    want_checker = sum(float((ref[k] ** 2).sum()) for k in GRADS)      # the checker's own gradients, squared norm
    assert abs(float(with_sq["grad_sumsq"][0]) - want_checker) <= 2.5 * BF16_TOL * want_checker
    for k in GRADS:
        assert np.array_equal(with_sq[k], got[k]), k
    _, only_dx = run_both(pcm, pr, want_grads=False, **kw)
    assert np.array_equal(only_dx["dX"][:n], got["dX"][:n])
    _, only_dw = run_both(pcm, pr, want_dX=False, **kw)
    for k in GRADS:
        assert np.array_equal(only_dw[k], got[k]), k


def test_bf16_every_row_clipped(pcm):
    """No row carries a gradient (every ratio far beyond its threshold on the clipped side): the backward products
    run over nothing, on every panel; gradients, dX and the sum of squared gradients are exactly zero, the loss is
    the sum of the clipped terms."""
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=8, N=16, K=4, B=8, d=512, ff=768, seed=41)
    ro = make_rollouts(cfg, 0)
    _, active = O.advantages(ro["reward"], cfg.G)
    kept, _, _ = O.sample_chunks(np.array([1.0, 0.3, 0.1, 0.6]), ro["phase"], None, active, cfg.B, cfg.seed, 0)
    pr = make_problem(cfg, wstd=0.05, kept=kept[:100], old_rel=0.1, eps=(0.2, 0.4))
    adv_rows = np.repeat(pr["adv"], cfg.N * cfg.A)
    pr["logp_old"] = np.where(adv_rows > 0, -40.0, 30.0).astype(np.float32)
    ref, got = run_both(pcm, pr, eps=(0.2, 0.4), torch_dtype=torch.bfloat16, max_kept=128, panel_rows=1792, grad_sumsq=True)
    assert ref["stats"][0] == 1.0 and got["stats"][0] == 1.0
    assert abs(got["loss"][0] - ref["loss"]) <= BF16_TOL * abs(ref["loss"])
    for k in GRADS:
        assert not got[k].any(), k
    assert not got["dX"][:len(ref["rows"])].any()
    assert got["grad_sumsq"][0] == 0.0


@pytest.mark.timeout(1200)
def test_bf16_full_size_head_whole_batch_against_checker(pcm, composed):
    """LIBERO-shaped head (d = 4096, ff = 11008) in the launch configuration the benchmark times: the whole
    batch (64 trajectories x 12 kept chunks = 43,008 rows) in one call, every output against the checker run on
    the same rows: loss, statistics, logp and dX row by row, and all four weight gradients.  The checker's inputs
    come from the generators and from a forward-only library call with the old weights (logp_old is an input of
    the step); nothing it is compared with is used to build them.  Additivity of Eq. 11 over groups (sum of
    per-group calls = one call) is kept as a property check of the library against itself."""
    cfg = CONFIGS["cfg2"]
    dv = torch.device("cuda")
    ro = make_rollouts(cfg, 0)
    adv, active = O.advantages(ro["reward"], cfg.G)
    C, valid = O.phase_scores(ro["actions"], ro["phase"], ro["reward"], None, cfg.n_groups, cfg.G, cfg.K)
    p = O.KeepProbState(cfg.K).update(C, valid)
    kept, off, nk = O.sample_chunks(p, ro["phase"], None, active, cfg.B, cfg.seed, 0)
    hidden = make_hidden_torch(cfg, dv)
    W = make_head_torch(cfg, dv)
    W_old = perturb_torch(cfg, W, std=0.002)
    tokens = dev(ro["tokens"].reshape(-1))
    adv_t = dev(adv.astype(np.float32))
    kept_t, nk_t = dev(kept), dev(np.array([nk], np.int32))
    zeros = torch.zeros(hidden.shape[0], device=dv)
    scale = 1.0 / cfg.T
    args = (cfg.T, cfg.N, cfg.A)

    old = pcm.grpo_masked_actor_step(hidden, tokens, zeros, adv_t, kept_t, nk_t, *args, W_old["Wg"], W_old["Wu"],
                                     W_old["Wd"], W_old["Wo"], want_grads=False, want_dX=False, composed_head=composed)
    rows = chunk_rows(kept, cfg.A)
    rows_t = torch.from_numpy(rows).to(dv)
    Wn = {k: v.float().cpu().numpy() for k, v in W.items()}
    hid_rows = hidden[rows_t].float().cpu().numpy()
    tok_rows = ro["tokens"].reshape(-1)[rows]
    adv_chunks = adv[kept // cfg.N]
    lp_old = conditioned_logp_old(hid_rows, tok_rows, old["logp"].double().cpu().numpy(), adv_chunks, cfg.A, Wn,
                                  (0.2, 0.2), 0.08).astype(np.float32)
    logp_old = torch.zeros(hidden.shape[0], device=dv)
    logp_old[rows_t] = torch.from_numpy(lp_old).to(dv)

    full = pcm.grpo_masked_actor_step(hidden, tokens, logp_old, adv_t, kept_t, nk_t, *args, W["Wg"], W["Wu"], W["Wd"],
                                      W["Wo"], 0.2, 0.2, scale, composed_head=composed, grad_sumsq=not composed)
    torch.cuda.synchronize()
    if not composed:     # sum of the squares of the weight gradients, written by the launches that finish them
        want = sum(float((full[k].double() ** 2).sum().item()) for k in GRADS)
        assert abs(float(full.pop("grad_sumsq").item()) - want) <= 2e-5 * want
    ref = O.actor_step(hid_rows, tok_rows, lp_old.astype(np.float64), adv_chunks, np.arange(len(kept)), 1, cfg.A,
                       Wn["Wg"], Wn["Wu"], Wn["Wd"], Wn["Wo"], 0.2, 0.2, scale)
    assert 0.02 < ref["stats"][0] < 0.98                          # clipped and unclipped rows both occur
    check(ref, {k: v.float().cpu().numpy() for k, v in full.items()}, BF16_TOL, len(rows), stats_tol=5e-2)

    # additivity over groups, library against library
    acc = {k: torch.zeros_like(full[k]) for k in GRADS}
    loss_sum = 0.0
    for g in range(cfg.n_groups):
        kg = kept[(kept // cfg.N) // cfg.G == g]
        part = pcm.grpo_masked_actor_step(hidden, tokens, logp_old, adv_t, dev(kg), dev(np.array([len(kg)], np.int32)),
                                          *args, W["Wg"], W["Wu"], W["Wd"], W["Wo"], 0.2, 0.2, scale, want_dX=False,
                                          composed_head=composed)
        for k in GRADS:
            acc[k] += part[k]
        loss_sum += part["loss"].item()
    # as written the only difference is the order of fp32 accumulation; composed, every call rounds its own
    # G = a^T dz to bf16 (2^-9 relative per element) before dWd and dWo are formed from it
    additivity_tol = 5e-3 if composed else 2e-3
    for k in GRADS:
        assert rel(acc[k].cpu().numpy(), full[k].cpu().numpy()) <= additivity_tol, k
    assert abs(loss_sum - full["loss"].item()) <= 1e-4 * max(1.0, abs(loss_sum))


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_bf16_large_configs_chained_selection_and_sampled_rows(pcm, name):
    """Unmasked (B = N), larger-batch and skewed long-horizon instances at full size: the four calls chained
    on the GPU, selection compared bit for bit, per-row outputs (logp, dX) of sampled kept chunks against the
    checker.  With B = N the kept list is every chunk in order (the all-kept mask is unmasked GRPO, Eq. 2); in
    the skewed instance a quarter of the groups have uniform rewards and are dropped at compaction."""
    cfg = CONFIGS[name]
    dv = torch.device("cuda")
    ro = make_rollouts(cfg, 0)
    adv_o, act_o = O.advantages(ro["reward"], cfg.G)
    C_o, valid_o = O.phase_scores(ro["actions"], ro["phase"], ro["reward"], None, cfg.n_groups, cfg.G, cfg.K)
    p_o = O.KeepProbState(cfg.K).update(C_o, valid_o)
    kept_o, off_o, nk_o = O.sample_chunks(p_o, ro["phase"], None, act_o, cfg.B, cfg.seed, 0)
    if name == "cfg5":
        assert nk_o == (cfg.n_groups - cfg.n_groups // 4) * cfg.G * cfg.B     # collapsed groups keep nothing
    if name == "cfg3":
        assert np.array_equal(kept_o, np.arange(cfg.T * cfg.N))               # nothing is masked

    phase = dev(ro["phase"])
    C, valid, adv, act = pcm.pcm_score_phases(dev(ro["actions"]), phase, dev(ro["reward"]), None, cfg.n_groups,
                                              cfg.G, cfg.K, 1e-6)
    state = pcm.pcm_state_init(cfg.K, dv)
    p = pcm.pcm_update_keep_probs(state, C, valid)
    kept, off, nk = pcm.pcm_sample_chunks(p, phase, None, act, cfg.B, cfg.seed, 0)
    torch.cuda.synchronize()
    assert int(nk.item()) == nk_o and np.array_equal(kept.cpu().numpy()[:nk_o], kept_o)
    assert np.array_equal(off.cpu().numpy(), off_o)

    hidden = make_hidden_torch(cfg, dv)
    W = make_head_torch(cfg, dv)
    W_old = perturb_torch(cfg, W, std=0.002)
    tokens = dev(ro["tokens"].reshape(-1))
    args = (cfg.T, cfg.N, cfg.A)
    zeros = torch.zeros(hidden.shape[0], device=dv)
    old = pcm.grpo_masked_actor_step(hidden, tokens, zeros, adv, kept, nk, *args, W_old["Wg"], W_old["Wu"],
                                     W_old["Wd"], W_old["Wo"], want_grads=False, want_dX=False)
    rows_kept = (torch.from_numpy(kept_o.astype(np.int64))[:, None] * cfg.A + torch.arange(cfg.A)[None, :]).reshape(-1).to(dv)
    logp_old = zeros
    logp_old[rows_kept] = old["logp"][:nk_o * cfg.A]
    del old

    # sampled kept chunks, spread over the batch, for the checker
    pick_pos = np.linspace(0, nk_o - 1, 8).astype(np.int64)
    pick = kept_o[pick_pos]
    rows_pick = (pick[:, None].astype(np.int64) * cfg.A + np.arange(cfg.A)[None, :]).reshape(-1)
    ridx = torch.from_numpy(rows_pick).to(dv)
    Wn = {k: v.float().cpu().numpy() for k, v in W.items()}
    sub_hidden = hidden[ridx].float().cpu().numpy()
    sub_tokens = ro["tokens"].reshape(-1)[rows_pick]
    sub_adv = adv_o[pick // cfg.N]
    lp_old = logp_old[ridx].cpu().numpy().astype(np.float64)
    cur = O.actor_step(sub_hidden, sub_tokens, lp_old, sub_adv, np.arange(len(pick)), 1, cfg.A, Wn["Wg"], Wn["Wu"],
                       Wn["Wd"], Wn["Wo"], want_grads=False)
    lp_old = condition_logp_old(lp_old, cur["logp"], np.arange(len(rows_pick)), 0.2, 0.2, 0.08)
    logp_old[ridx] = torch.from_numpy(lp_old.astype(np.float32)).to(dv)
    lp_old = logp_old[ridx].cpu().numpy().astype(np.float64)

    scale = 1.0 / cfg.T
    out = pcm.grpo_masked_actor_step(hidden, tokens, logp_old, adv, kept, nk, *args, W["Wg"], W["Wu"], W["Wd"], W["Wo"],
                                     0.2, 0.2, scale, grad_sumsq=True)
    torch.cuda.synchronize()
    # the final panel (wherever the kept rows end) leaves the sum of the squares of the accumulated gradients
    want = sum(float((out[k].double() ** 2).sum().item()) for k in GRADS)
    assert abs(float(out["grad_sumsq"].item()) - want) <= 2e-5 * want, (out["grad_sumsq"], want)
    ref = O.actor_step(sub_hidden, sub_tokens, lp_old, sub_adv, np.arange(len(pick)), 1, cfg.A, Wn["Wg"], Wn["Wu"],
                       Wn["Wd"], Wn["Wo"], 0.2, 0.2, scale)
    sel = np.concatenate([np.arange(q * cfg.A, (q + 1) * cfg.A) for q in pick_pos])
    sel_t = torch.from_numpy(sel).to(dv)
    assert rel(out["logp"][sel_t].cpu().numpy(), ref["logp"]) <= BF16_TOL
    assert rel(out["dX"][sel_t].float().cpu().numpy(), ref["dX"]) <= BF16_TOL
    assert out["stats"][3].item() == nk_o * cfg.A
    for k in GRADS:
        g = out[k]
        assert torch.isfinite(g).all() and g.abs().max().item() > 0
    del out

    # A sub-batch through the same launch: the kept list, its capacity and every buffer stay those of the whole
    # batch, only the device-side kept count says that fewer chunks are live (the first groups' chunks), so the
    # row-tile skipping, the re-dealing of live tiles over the XCDs and the cut-off of the weight-gradient
    # reductions all run at full head size.  Everything against the checker: loss, logp and dX row by row, and the
    # four weight gradients (Eq. 11 restricted to those groups).
    per_traj = min(cfg.B, cfg.N)
    n_sub = {"cfg3": 1, "cfg4": 2, "cfg5": 2}[name] * cfg.G * per_traj
    assert n_sub < nk_o and np.all(np.diff(kept_o[:n_sub] // cfg.N) >= 0)
    sub = kept_o[:n_sub]
    rows_sub = chunk_rows(sub, cfg.A)
    rsub_t = torch.from_numpy(rows_sub).to(dv)
    hid_sub = hidden[rsub_t].float().cpu().numpy()
    tok_sub = ro["tokens"].reshape(-1)[rows_sub]
    adv_sub = adv_o[sub // cfg.N]
    assert np.abs(adv_sub).min() > 0                              # live groups only
    lp_sub = conditioned_logp_old(hid_sub, tok_sub, logp_old[rsub_t].double().cpu().numpy(), adv_sub, cfg.A, Wn,
                                  (0.2, 0.2), 0.08).astype(np.float32)
    logp_old[rsub_t] = torch.from_numpy(lp_sub).to(dv)
    nk_sub = dev(np.array([n_sub], np.int32))
    got = pcm.grpo_masked_actor_step(hidden, tokens, logp_old, adv, kept, nk_sub, *args, W["Wg"], W["Wu"], W["Wd"],
                                     W["Wo"], 0.2, 0.2, scale)
    torch.cuda.synchronize()
    ref = O.actor_step(hid_sub, tok_sub, lp_sub.astype(np.float64), adv_sub, np.arange(n_sub), 1, cfg.A, Wn["Wg"],
                       Wn["Wu"], Wn["Wd"], Wn["Wo"], 0.2, 0.2, scale)
    n_rows = n_sub * cfg.A
    got_np = {k: got[k].float().cpu().numpy() for k in GRADS + ("loss", "stats")}
    got_np["logp"] = got["logp"][:n_rows].cpu().numpy()
    got_np["dX"] = got["dX"][:n_rows].float().cpu().numpy()
    check(ref, got_np, BF16_TOL, n_rows, stats_tol=5e-2)
