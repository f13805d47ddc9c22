"""Pins of the oracle's Adam step and cosine learning-rate schedule (the optimiser the paper trains
with) against the library implementation (torch.optim.Adam / CosineAnnealingLR in fp64) and closed forms."""
import math

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(7)


@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_adam_matches_torch_fp64_over_steps(wd):
    p0 = RNG.normal(size=257)
    p = p0.copy(); m = np.zeros_like(p); v = np.zeros_like(p)
    pt = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([pt], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
    for t in range(1, 8):
        g = RNG.normal(size=p.shape) * (1.0 + t)
        oracle.adam_step(p, g, m, v, 3e-3, t, weight_decay=wd)
        pt.grad = torch.tensor(g)
        opt.step()
        assert np.allclose(p, pt.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adam_first_step_is_lr_times_sign():
    # t = 1, m = v = 0: m_hat / sqrt(v_hat) = g / |g|, so every parameter moves by lr against its gradient's sign
    g = np.array([3.0, -0.25, 1e-3, -7.0]); p = np.zeros(4); m = np.zeros(4); v = np.zeros(4)
    oracle.adam_step(p, g, m, v, 0.1, 1, eps=0.0)
    assert np.allclose(p, -0.1 * np.sign(g), rtol=1e-14)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_cosine_schedule_closed_forms_and_torch():
    assert oracle.cosine_lr(0.01, 0.0, 0, 100) == 0.01
    assert abs(oracle.cosine_lr(0.01, 0.001, 100, 100) - 0.001) < 1e-18
    assert abs(oracle.cosine_lr(0.01, 0.0, 50, 100) - 0.005) < 1e-18
    pt = torch.zeros(1, requires_grad=True)
    opt = torch.optim.SGD([pt], lr=0.02)
    sch = torch.optim.lr_scheduler.CosineAnnealingLR(opt, T_max=40, eta_min=0.002)
    for t in range(41):
        assert abs(opt.param_groups[0]["lr"] - oracle.cosine_lr(0.02, 0.002, t, 40)) < 1e-12
        opt.step(); sch.step()
