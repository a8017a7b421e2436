"""Pins for the oracle's gated average + AdamW (the optimizer of the paper's LLM runs, App. "Hyperparameters
for LLM Architecture": beta1 = 0.9, beta2 = 0.95, weight decay 0.1), applied to covered rows only."""
import numpy as np
import pytest
import torch

HP = dict(lr=4e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def test_matches_torch_adamw_over_several_steps(orc):
    # library routine as the reference: torch.optim.AdamW on fp64 CPU tensors, every row covered by all
    # workers, so the gated average is the plain mean
    K, R, D = 3, 7, 5
    theta0 = _rand((R, D), 1, 0.02)
    p = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"], weight_decay=HP["weight_decay"])
    th, m, v = theta0.copy(), np.zeros((R, D)), np.zeros((R, D))
    mask = np.ones((K, R), dtype=np.uint8)
    for step in range(1, 6):
        gs = [_rand((R, D), 10 * step + k, 1e-3) for k in range(K)]
        p.grad = torch.from_numpy(np.mean(gs, axis=0))
        opt.step()
        th, m, v, cov = orc.avg_adamw(gs, mask, th, m, v, step=step, **HP)
        assert (cov == K).all()
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-15)
        st = opt.state[p]
        np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-24)


def test_first_step_closed_form(orc):
    # m = v = 0 and t = 1: mhat = g, vhat = g^2, so theta_1 = theta_0 (1 - lr wd) - lr g / (|g| + eps)
    R, D = 4, 6
    theta0, g = _rand((R, D), 3, 0.02), _rand((R, D), 4, 1e-3)
    th, m, v, _ = orc.avg_adamw([g], np.ones((1, R), np.uint8), theta0, np.zeros((R, D)), np.zeros((R, D)), step=1, **HP)
    want = theta0 * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g / (np.abs(g) + HP["eps"])
    np.testing.assert_allclose(th, want, rtol=1e-12)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 0.05 * g * g, rtol=1e-12)


def test_uncovered_rows_are_untouched_and_covered_rows_use_their_own_count(orc):
    K, R, D = 3, 5, 4
    mask = np.array([[1, 0, 1, 0, 1], [1, 0, 0, 0, 1], [0, 0, 1, 0, 1]], dtype=np.uint8)  # loads 2, 0, 2, 0, 3
    gs = [_rand((R, D), 20 + k, 1e-3) for k in range(K)]
    for k in range(K):
        gs[k][mask[k] == 0] = np.nan  # what a worker does not cover is never read
    theta0, m0, v0 = _rand((R, D), 5, 0.02), _rand((R, D), 6, 1e-4), np.abs(_rand((R, D), 7, 1e-7))
    th, m, v, cov = orc.avg_adamw(gs, mask, theta0, m0, v0, step=3, **HP)
    assert cov.tolist() == [2, 0, 2, 0, 3]
    for r in (1, 3):
        assert (th[r] == theta0[r]).all() and (m[r] == m0[r]).all() and (v[r] == v0[r]).all()
    assert np.isfinite(th).all()
    # row by row against the single-worker routine fed with that row's mean gradient
    for r in (0, 2, 4):
        gbar = np.mean([gs[k][r] for k in range(K) if mask[k, r]], axis=0)[None]
        t1, m1, v1, _ = orc.avg_adamw([gbar], np.ones((1, 1), np.uint8), theta0[r][None], m0[r][None], v0[r][None], step=3, **HP)
        np.testing.assert_allclose(th[r], t1[0], rtol=1e-13)
        np.testing.assert_allclose(m[r], m1[0], rtol=1e-13)
        np.testing.assert_allclose(v[r], v1[0], rtol=1e-13)


def test_grad_scale_is_a_scale_of_the_gradient_and_lr_zero_freezes_theta(orc):
    R, D = 3, 8
    g, theta0 = _rand((R, D), 8, 1e-3), _rand((R, D), 9, 0.02)
    z = np.zeros((R, D))
    one = np.ones((1, R), np.uint8)
    a = orc.avg_adamw([g], one, theta0, z, z, step=2, grad_scale=0.25, **HP)
    b = orc.avg_adamw([0.25 * g], one, theta0, z, z, step=2, **HP)
    for x, y in zip(a[:3], b[:3]):
        np.testing.assert_allclose(x, y, rtol=1e-13)
    hp0 = dict(HP, lr=0.0)
    th, m, v, _ = orc.avg_adamw([g], one, theta0, z, z, step=2, **hp0)
    assert (th == theta0).all() and (m != 0).any() and (v != 0).any()


def test_bf16_inputs_are_widened_exactly(orc):
    R, D = 2, 8
    g32 = torch.from_numpy(_rand((R, D), 11, 1e-3)).to(torch.bfloat16)
    bits = g32.view(torch.int16).numpy().view(np.uint16)
    theta0 = _rand((R, D), 12, 0.02)
    z = np.zeros((R, D))
    one = np.ones((1, R), np.uint8)
    a = orc.avg_adamw([bits], one, theta0, z, z, step=1, **HP)
    b = orc.avg_adamw([g32.to(torch.float64).numpy()], one, theta0, z, z, step=1, **HP)
    for x, y in zip(a[:3], b[:3]):
        assert (x == y).all()


def test_clip_coefficient_matches_the_library_routine(orc):
    """orc_clip_scale against torch.nn.utils.clip_grad_norm_ on two parameter groups, above and below the
    threshold (the paper states the threshold, 1.0; the form of the coefficient is the usual one)."""
    rng = np.random.default_rng(31)
    for scale in (5.0, 1e-3):
        ga, gb = rng.standard_normal((7, 5)) * scale, rng.standard_normal((3, 11)) * scale
        pa, pb = torch.zeros((7, 5), dtype=torch.float64, requires_grad=True), torch.zeros((3, 11), dtype=torch.float64, requires_grad=True)
        pa.grad, pb.grad = torch.from_numpy(ga.copy()), torch.from_numpy(gb.copy())
        total = torch.nn.utils.clip_grad_norm_([pa, pb], max_norm=1.0)
        coef = orc.clip_scale([(ga ** 2).sum(), (gb ** 2).sum()], 1.0)
        assert abs(float(total) ** 2 - ((ga ** 2).sum() + (gb ** 2).sum())) <= 1e-12 * float(total) ** 2
        np.testing.assert_allclose(pa.grad.numpy(), coef * ga, rtol=1e-12, atol=0)
        np.testing.assert_allclose(pb.grad.numpy(), coef * gb, rtol=1e-12, atol=0)
        assert (coef == 1.0) == (scale < 1.0)
    assert orc.clip_scale([0.0], 1.0) == 1.0  # a zero gradient is left alone
    assert abs(orc.clip_scale([4.0, 12.0], 2.0) - 2.0 / (4.0 + 1e-6)) < 1e-15
