"""GPU parity of the fused AdamW step (C ABI) against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import optim
from paper_2309_16119_amd import binding as b

pytestmark = pytest.mark.gpu

HP = dict(lr=3e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def run_steps(n, steps, hp, seed):
    # the C ABI takes the hyper-parameters as float32: give the oracle those same values
    hp = {k: float(np.float32(x)) for k, x in hp.items()}
    rng = np.random.default_rng(seed)
    p0 = rng.normal(size=n).astype(np.float32) * 0.02
    grads = (rng.normal(size=(steps, n)) * np.logspace(-4, 1, n)).astype(np.float32)
    dev = lambda a: torch.from_numpy(a.copy()).cuda()
    p, m, v = dev(p0), torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    pr, mr, vr, m_abs = p0.astype(np.float64), np.zeros(n), np.zeros(n), np.zeros(n)
    for t in range(1, steps + 1):
        g = dev(grads[t - 1])
        b.modulora_adamw(p, g, m, v, step=t, **hp)
        # the terms of m may cancel: its rounding error scales with the same recursion over |g|
        m_abs = hp["beta1"] * m_abs + (1 - hp["beta1"]) * np.abs(grads[t - 1].astype(np.float64))
        pr_new, mr, vr = optim.adamw_step(pr, grads[t - 1], mr, vr, step=t, **hp)
        # Every step moves a parameter by at most about lr: fp32 rounding of the update is
        # bounded by a few ulp of lr (times a ratio m_hat / sqrt(v_hat) of order one) plus an ulp of the parameter itself.  The moments are a
        # handful of fp32 operations: a few ulp.
        got = p.cpu().numpy().astype(np.float64)
        # (the GPU's own parameter is the running fp32 value: two roundings of p per step)
        tol = t * 2.0 ** -23 * np.abs(pr_new) + 32 * 2.0 ** -24 * hp["lr"] * t
        assert np.all(np.abs(got - pr_new) <= tol), (t, np.max(np.abs(got - pr_new) - tol))
        assert np.all(np.abs(m.cpu().numpy() - mr) <= 4e-7 * t * m_abs)
        assert np.allclose(v.cpu().numpy(), vr, rtol=4e-7 * t, atol=1e-38)
        pr = pr_new
    return p


@pytest.mark.parametrize("n", [1, 3, 4, 1023, 1024, 1025, 8 * (8192 + 22016) + 2])
def test_adamw_against_oracle(n):
    run_steps(n, 4, HP, seed=n)


def test_adamw_without_decay_and_other_betas():
    run_steps(5000, 3, dict(lr=1e-2, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.0), seed=1)


def test_adamw_leaves_the_neighbours_alone():
    """The ragged end must not touch memory past n."""
    n = 1021
    buf = [torch.full((n + 16,), 7.0, device="cuda") for _ in range(4)]
    p, g, m, v = (t[:n] for t in buf)
    b.modulora_adamw(p, g, m, v, step=1, **HP)
    for t in buf:
        assert torch.all(t[n:] == 7.0)
    assert torch.all(buf[1] == 7.0)          # the gradient is read only
