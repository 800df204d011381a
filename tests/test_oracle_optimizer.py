"""Pins of the checker's optimizer step (App. D of the paper: AdamW, lr 1e-5, betas (0.9, 0.999),
weight decay 0, gradient clipping at 2.0) against closed forms and against PyTorch's own
implementation run in fp64 on the CPU."""
import numpy as np
import pytest
import torch

from oracle import pcm_oracle as O


def _tensors(seed, shapes=((7, 5), (3,), (4, 6)), scale=1.0):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal(s) * scale for s in shapes]


def test_clip_leaves_small_gradients_alone():
    g = _tensors(0, scale=1e-3)
    out, norm = O.clip_grad_norm(g, 2.0)
    assert norm < 2.0
    for a, b in zip(g, out):
        np.testing.assert_array_equal(a, b)
    assert np.isclose(norm, np.sqrt(sum((x * x).sum() for x in g)), rtol=1e-15)


def test_clip_scales_the_joint_norm_to_the_threshold():
    g = _tensors(1, scale=10.0)
    out, norm = O.clip_grad_norm(g, 2.0)
    after = np.sqrt(sum((x * x).sum() for x in out))
    assert norm > 2.0
    assert np.isclose(after, 2.0 * norm / (norm + 1e-6), rtol=1e-14)
    # one common factor for every tensor (the norm is joint, not per tensor)
    ratios = np.concatenate([(b / a).ravel() for a, b in zip(g, out)])
    assert np.allclose(ratios, ratios[0], rtol=1e-14)


def test_first_step_moves_each_weight_by_lr_times_sign():
    # t = 1, m = v = 0: m_hat = g, v_hat = g^2, so the step is lr * g / (|g| + eps)
    p, g = _tensors(2), _tensors(3, scale=1e-2)
    zeros = [np.zeros_like(x) for x in p]
    new_p, m, v, _ = O.adamw_step(p, g, zeros, zeros, 1, lr=1e-5, max_grad_norm=1e9)
    for a, b, gi in zip(p, new_p, g):
        np.testing.assert_allclose(a - b, 1e-5 * gi / (np.abs(gi) + 1e-8), rtol=1e-9, atol=0)
    for mi, vi, gi in zip(m, v, g):
        np.testing.assert_allclose(mi, 0.1 * gi, rtol=1e-12)
        np.testing.assert_allclose(vi, 0.001 * gi * gi, rtol=1e-12)


def test_decay_is_decoupled_from_the_gradient():
    p = _tensors(4)
    zeros = [np.zeros_like(x) for x in p]
    new_p, m, v, norm = O.adamw_step(p, zeros, zeros, zeros, 1, lr=1e-2, weight_decay=0.5)
    assert norm == 0.0
    for a, b in zip(p, new_p):
        np.testing.assert_allclose(b, a * (1 - 1e-2 * 0.5), rtol=1e-15)


@pytest.mark.parametrize("wd,max_norm,gscale", [(0.0, 2.0, 0.05), (0.0, 2.0, 5.0), (0.01, 0.5, 1.0)])
def test_matches_pytorch_adamw_over_several_steps(wd, max_norm, gscale):
    shapes = ((6, 4), (5,), (3, 7))
    p0 = _tensors(10, shapes)
    tp = [torch.nn.Parameter(torch.tensor(x, dtype=torch.float64)) for x in p0]
    opt = torch.optim.AdamW(tp, lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
    p = [x.copy() for x in p0]
    m = [np.zeros_like(x) for x in p0]
    v = [np.zeros_like(x) for x in p0]
    for t in range(1, 7):
        g = _tensors(100 + t, shapes, scale=gscale)
        for q, gi in zip(tp, g):
            q.grad = torch.tensor(gi, dtype=torch.float64)
        tnorm = torch.nn.utils.clip_grad_norm_(tp, max_norm)
        opt.step()
        p, m, v, norm = O.adamw_step(p, g, m, v, t, lr=1e-3, weight_decay=wd, max_grad_norm=max_norm)
        assert np.isclose(norm, float(tnorm), rtol=1e-13)
        for a, q in zip(p, tp):
            np.testing.assert_allclose(a, q.detach().numpy(), rtol=1e-11, atol=1e-14)
