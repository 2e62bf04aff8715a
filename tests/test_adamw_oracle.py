"""Pins of the AdamW oracle (CPU): a closed form, a library implementation, invariants."""
import numpy as np
import pytest
import torch

from oracle import optim

HP = dict(lr=3e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def test_first_step_closed_form():
    """From zero moments, step 1: m_hat = g and v_hat = g^2 exactly, so the update is
    p (1 - lr wd) - lr g / (|g| + eps): every entry moves by about lr against the sign of g."""
    rng = np.random.default_rng(0)
    p, g = rng.normal(size=1000), rng.normal(size=1000)
    z = np.zeros_like(p)
    pn, m, v = optim.adamw_step(p, g, z, z, step=1, **HP)
    lr, wd, eps = HP["lr"], HP["weight_decay"], HP["eps"]
    assert np.allclose(pn, p * (1 - lr * wd) - lr * g / (np.abs(g) + eps), rtol=1e-13, atol=0)
    assert np.allclose(m, 0.1 * g, rtol=1e-13) and np.allclose(v, 0.001 * g * g, rtol=1e-12)


def test_zero_gradient_only_decays():
    p = np.linspace(-2, 2, 11)
    z = np.zeros_like(p)
    pn, m, v = optim.adamw_step(p, z, z, z, step=7, **HP)
    assert np.array_equal(m, z) and np.array_equal(v, z)
    assert np.allclose(pn, p * (1 - HP["lr"] * HP["weight_decay"]), rtol=1e-15)


def test_decay_is_decoupled_from_the_moments():
    """Weight decay must not leak into m and v (that would be Adam with L2 regularisation)."""
    rng = np.random.default_rng(1)
    p, g, m0, v0 = rng.normal(size=64), rng.normal(size=64), rng.normal(size=64), rng.uniform(size=64)
    a = optim.adamw_step(p, g, m0, v0, step=3, **HP)
    b = optim.adamw_step(p, g, m0, v0, step=3, **dict(HP, weight_decay=0.0))
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    assert np.allclose(a[0] - b[0], -HP["lr"] * HP["weight_decay"] * p, rtol=1e-9, atol=1e-18)


@pytest.mark.parametrize("wd", [0.0, 0.01, 0.1])
def test_against_torch_adamw_over_several_steps(wd):
    """torch.optim.AdamW in float64 on the CPU is an independent implementation of the same rule."""
    rng = np.random.default_rng(2)
    n, steps = 257, 6
    p0 = rng.normal(size=n)
    grads = rng.normal(size=(steps, n)) * np.logspace(-3, 1, n)
    hp = dict(HP, weight_decay=wd)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.AdamW([tp], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"], weight_decay=wd)
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, steps + 1):
        tp.grad = torch.from_numpy(grads[t - 1].copy())
        opt.step()
        p, m, v = optim.adamw_step(p, grads[t - 1], m, v, step=t, **hp)
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15), t
    st = opt.state[tp]
    assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
    assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)


def test_planted_mistakes_are_caught():
    """Variants with one plausible mistake each must differ from the oracle by far more than
    the tolerances used above."""
    rng = np.random.default_rng(3)
    p, g, m0, v0 = rng.normal(size=50), rng.normal(size=50), 0.1 * rng.normal(size=50), rng.uniform(size=50) * 0.01
    ref = optim.adamw_step(p, g, m0, v0, step=4, **HP)[0]
    lr, b1, b2, eps, wd = HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"]
    m = b1 * m0 + (1 - b1) * g
    v = b2 * v0 + (1 - b2) * g * g
    no_bias_correction = p - lr * wd * p - lr * m / (np.sqrt(v) + eps)
    coupled_decay_g = g + wd * p
    mc = b1 * m0 + (1 - b1) * coupled_decay_g
    vc = b2 * v0 + (1 - b2) * coupled_decay_g ** 2
    coupled = p - lr * (mc / (1 - b1 ** 4)) / (np.sqrt(vc / (1 - b2 ** 4)) + eps)
    wrong_sign = p - lr * wd * p + lr * (m / (1 - b1 ** 4)) / (np.sqrt(v / (1 - b2 ** 4)) + eps)
    for bad in (no_bias_correction, coupled, wrong_sign):
        assert np.max(np.abs(bad - ref)) > 1e-6
