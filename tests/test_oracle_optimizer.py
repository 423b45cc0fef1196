"""Pins for the oracle of the PS-side optimizer step (Adam as published):
closed forms of the algorithm, a hand-computed step, and the library optimizer
in float64 as the textbook routine."""
import numpy as np
import pytest
import torch

from oracle import optimizer as oo

H = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)


def test_first_step_moves_every_weight_by_lr_against_the_gradient_sign():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(100)
    g = rng.standard_normal(100) * 10.0 ** rng.integers(-3, 4, 100)
    w1, m1, v1 = oo.adam_step(w, np.zeros(100), np.zeros(100), g, step=1, **H)
    # mhat = g, vhat = g^2 exactly at t = 1
    assert np.allclose(w - w1, H["lr"] * g / (np.abs(g) + H["eps"]), rtol=1e-12, atol=0)
    assert np.allclose(m1, 0.1 * g, rtol=1e-15) and np.allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_constant_gradient_gives_the_closed_form_trajectory():
    g = np.array([0.5, -2.0, 3e-4])
    w = np.array([1.0, 1.0, 1.0])
    m = np.zeros(3)
    v = np.zeros(3)
    for t in range(1, 21):
        w, m, v = oo.adam_step(w, m, v, g, step=t, **H)
        # bias-corrected moments equal g and g^2 at every step
        assert np.allclose(m / (1 - 0.9 ** t), g, rtol=1e-12)
        assert np.allclose(v / (1 - 0.999 ** t), g * g, rtol=1e-10)
    assert np.allclose(w, 1.0 - 20 * H["lr"] * g / (np.abs(g) + H["eps"]), rtol=1e-12)


def test_hand_computed_step():
    # w=1, m=0.2, v=0.04, g=-0.1, t=3, lr=0.01, b1=0.5, b2=0.75, eps=0, wd=0.1
    w, m, v = oo.adam_step([1.0], [0.2], [0.04], [-0.1], 0.01, 0.5, 0.75, 0.0, 0.1, 3)
    m_e = 0.5 * 0.2 + 0.5 * -0.1            # 0.05
    v_e = 0.75 * 0.04 + 0.25 * 0.01         # 0.0325
    mh = m_e / (1 - 0.125)
    vh = v_e / (1 - 0.421875)
    w_e = 1.0 - 0.01 * (mh / vh ** 0.5 + 0.1 * 1.0)
    assert abs(m[0] - 0.05) < 1e-16 and abs(v[0] - 0.0325) < 1e-16 and abs(w[0] - w_e) < 1e-15


def test_zero_gradient_only_decays_the_moments():
    w, m, v = oo.adam_step([2.0], [0.0], [0.0], [0.0], step=5, **H)
    assert w[0] == 2.0 and m[0] == 0.0 and v[0] == 0.0
    w, m, v = oo.adam_step([2.0], [1.0], [1.0], [0.0], step=5, **H)
    assert m[0] == 0.9 and v[0] == 0.999 and w[0] < 2.0


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_matches_the_library_optimizer_in_float64(wd):
    torch.manual_seed(0)
    p = torch.randn(64, 48, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.8, 0.95), eps=1e-7, weight_decay=wd)
    w = p.detach().numpy().copy()
    m = np.zeros_like(w)
    v = np.zeros_like(w)
    for t in range(1, 6):
        g = torch.randn(64, 48, dtype=torch.float64)
        p.grad = g.clone()
        opt.step()
        w, m, v = oo.adam_step(w, m, v, g.numpy(), 3e-3, 0.8, 0.95, 1e-7, wd, t)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -3.1415927, 1e-20], dtype=np.float32)
    r = oo.bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0            # tie to even (mantissa 0)
    assert r[2] == np.float32(1.0 + 2 ** -7)
    assert r[3] == np.float32(1.0 + 2 ** -6)      # tie to even (up)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
