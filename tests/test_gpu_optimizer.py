"""GPU parity of pcm_adamw_clip_step (through the C boundary) against the fp64 checker.

Tolerances: the kernel does the update in fp32 on fp32 state, the checker in fp64.  v is a sum of
positive fp32 terms (relative 2e-6); m is a sum of two terms that may cancel, so its error is bounded
relative to the magnitude of the terms, beta1 |m| + (1 - beta1) |g|, not of the result; the gradient
norm is accumulated in fp64 from fp32 squares (relative 1e-6); a new weight differs from the
checker's by at most a few fp32 roundings of the weight itself plus a relative 1e-5 of the size of
the step (again measured with the terms of m taken in absolute value).
"""
import numpy as np
import pytest
import torch

from oracle import pcm_oracle as O

pytestmark = pytest.mark.gpu


def _case(seed, shapes, gscale, wscale=0.02):
    rng = np.random.default_rng(seed)
    w = [(rng.standard_normal(s) * wscale).astype(np.float32) for s in shapes]
    g = [(rng.standard_normal(s) * gscale).astype(np.float32) for s in shapes]
    m = [(rng.standard_normal(s) * gscale * 0.1).astype(np.float32) for s in shapes]
    v = [(rng.random(s) * gscale * gscale * 1e-3).astype(np.float32) for s in shapes]
    return w, g, m, v


def _run(w, g, m, v, step, want_bf16=True, **hp):
    import paper_2605_16154_amd as pcm
    dev = torch.device("cuda:0")
    t = lambda xs: [torch.from_numpy(x.copy()).to(dev).reshape(-1) for x in xs]
    dw, dg, dm, dv = t(w), t(g), t(m), t(v)
    lowp = [torch.zeros(x.numel(), dtype=torch.bfloat16, device=dev) for x in dw] if want_bf16 else None
    norm = pcm.pcm_adamw_clip_step(dg, dw, dm, dv, step, weights_bf16=lowp, **hp)
    torch.cuda.synchronize()
    back = lambda xs, ref: [x.cpu().numpy().reshape(r.shape) for x, r in zip(xs, ref)]
    return back(dw, w), back(dm, m), back(dv, v), float(norm.item()), lowp, dw, back(dg, g)


def _check(w, g, m, v, step, **hp):
    got_w, got_m, got_v, got_norm, lowp, dw, got_g = _run(w, g, m, v, step, **hp)
    okw = dict(lr=hp.get("lr", 1e-5), beta1=hp.get("beta1", 0.9), beta2=hp.get("beta2", 0.999), eps=hp.get("eps", 1e-8),
               weight_decay=hp.get("weight_decay", 0.0), max_grad_norm=hp.get("max_grad_norm", 2.0))
    ref_w, ref_m, ref_v, ref_norm = O.adamw_step(w, g, m, v, step, **okw)
    assert abs(got_norm - ref_norm) <= 1e-6 * ref_norm + 1e-30
    for a, b in zip(got_g, g):
        np.testing.assert_array_equal(a, b)            # gradients are read only
    scale = min(1.0, okw["max_grad_norm"] / (ref_norm + 1e-6))
    b1, b2 = okw["beta1"], okw["beta2"]
    m_terms = [b1 * np.abs(mi.astype(np.float64)) + (1 - b1) * np.abs(gi.astype(np.float64)) * scale for mi, gi in zip(m, g)]
    for gm, rm, mt in zip(got_m, ref_m, m_terms):
        assert np.all(np.abs(gm - rm) <= 2e-6 * mt + 1e-30)
    for gv, rv in zip(got_v, ref_v):
        np.testing.assert_allclose(gv, rv, rtol=2e-6, atol=1e-35)
    step_size = okw["lr"] / (1 - b1 ** step)
    for gw, rw, w0, mt, rv in zip(got_w, ref_w, w, m_terms, ref_v):
        step_bound = step_size * mt / (np.sqrt(rv / (1 - b2 ** step)) + okw["eps"])
        tol = 3 * np.spacing(np.abs(w0).astype(np.float32)).astype(np.float64) + 1e-5 * step_bound + 1e-30
        assert np.all(np.abs(gw.astype(np.float64) - rw) <= tol), float(np.max(np.abs(gw - rw) / tol))
    if lowp is not None:
        for lp, x in zip(lowp, dw):
            assert torch.equal(lp, x.to(torch.bfloat16))   # round-to-nearest-even copy of the new fp32 weights
    return got_norm


def test_head_shaped_tensors_clipped_and_unclipped():
    shapes = ((256, 1024), (256, 1024), (1024, 256), (256, 256))     # the head's four matrices, small
    w, g, m, v = _case(0, shapes, 1e-3)
    n1 = _check(w, g, m, v, 1)
    assert n1 < 2.0
    w, g, m, v = _case(1, shapes, 0.5)
    n2 = _check(w, g, m, v, 7)
    assert n2 > 2.0


def test_ragged_sizes_and_single_tensor():
    # sizes that are not multiples of 4 or of the 4096-element chunk, including a 1-element tensor
    w, g, m, v = _case(2, ((4097,), (1,), (3, 5), (8191,), (4096,), (12289,)), 0.05)
    _check(w, g, m, v, 3, want_bf16=True)
    w, g, m, v = _case(3, ((70001,),), 0.2)
    _check(w, g, m, v, 1, want_bf16=False)


def test_weight_decay_and_other_hyperparameters():
    w, g, m, v = _case(4, ((513, 129), (1000,)), 0.3)
    _check(w, g, m, v, 12, lr=3e-4, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1, max_grad_norm=0.7)


def test_zero_gradient_leaves_weights_with_zero_decay():
    w, g, m, v = _case(5, ((2048,), (100,)), 0.1)
    g = [np.zeros_like(x) for x in g]
    m = [np.zeros_like(x) for x in m]
    v = [np.zeros_like(x) for x in v]
    got_w, got_m, got_v, norm, _, _, _ = _run(w, g, m, v, 1)
    assert norm == 0.0
    for a, b in zip(got_w, w):
        np.testing.assert_array_equal(a, b)
    for a in got_m + got_v:
        assert not a.any()


def test_several_steps_track_the_checker():
    shapes = ((300, 70), (4100,))
    w, g, m, v = _case(6, shapes, 0.1)
    import paper_2605_16154_amd as pcm
    dev = torch.device("cuda:0")
    dw = [torch.from_numpy(x.copy()).to(dev).reshape(-1) for x in w]
    dm = [torch.zeros_like(x) for x in dw]
    dv = [torch.zeros_like(x) for x in dw]
    rw = [x.astype(np.float64) for x in w]
    rm = [np.zeros_like(x) for x in rw]
    rv = [np.zeros_like(x) for x in rw]
    rng = np.random.default_rng(60)
    for t in range(1, 6):
        g = [(rng.standard_normal(s) * 0.3).astype(np.float32) for s in shapes]
        dg = [torch.from_numpy(x).to(dev).reshape(-1) for x in g]
        pcm.pcm_adamw_clip_step(dg, dw, dm, dv, t, lr=1e-3)
        rw, rm, rv, _ = O.adamw_step(rw, g, rm, rv, t, lr=1e-3)
    torch.cuda.synchronize()
    for a, b, w0 in zip(dw, rw, w):
        moved = np.abs(b - w0.reshape(b.shape))
        err = np.abs(a.cpu().numpy().reshape(b.shape).astype(np.float64) - b)
        assert np.all(err <= 1e-4 * moved + 8 * np.spacing(np.abs(w0).astype(np.float32))), float(err.max())


def test_given_sum_of_squares_replaces_the_norm_pass():
    """pcm_adamw_clip_step_ex with the sum of the squares of the gradients handed in (as the actor step leaves it):
    the same norm and the same update as the call that sums them itself."""
    import paper_2605_16154_amd as pcm
    dev = torch.device("cuda:0")
    shapes = ((256, 1024), (256, 1024), (1024, 256), (256, 256))
    for seed, gscale, step in ((11, 1e-3, 1), (12, 0.5, 4)):
        w, g, m, v = _case(seed, shapes, gscale)
        ref_w, ref_m, ref_v, ref_norm, _, _, _ = _run(w, g, m, v, step)
        t = lambda xs: [torch.from_numpy(x.copy()).to(dev).reshape(-1) for x in xs]
        dw, dg, dm, dv = t(w), t(g), t(m), t(v)
        sumsq = torch.tensor([sum(float((x.astype(np.float64) ** 2).sum()) for x in g)], dtype=torch.float64, device=dev)
        norm = pcm.pcm_adamw_clip_step(dg, dw, dm, dv, step, grad_sumsq=sumsq)
        torch.cuda.synchronize()
        assert abs(float(norm.item()) - ref_norm) <= 1e-6 * ref_norm
        for got, ref in zip(dw + dm + dv, ref_w + ref_m + ref_v):
            np.testing.assert_allclose(got.cpu().numpy().reshape(ref.shape), ref, rtol=2e-6, atol=1e-30)


def test_bad_arguments_are_rejected():
    import paper_2605_16154_amd as pcm
    dev = torch.device("cuda:0")
    x = [torch.zeros(16, device=dev)]
    with pytest.raises(pcm.PcmError):
        pcm.pcm_adamw_clip_step(x, x, x, x, 0)                      # steps count from 1
    with pytest.raises(pcm.PcmError):
        pcm.pcm_adamw_clip_step(x, x, x, x, 1, beta1=1.0)
    with pytest.raises(pcm.PcmError):
        pcm.pcm_adamw_clip_step(x * 9, x * 9, x * 9, x * 9, 1)      # more than PCM_MAX_OPT_TENSORS
