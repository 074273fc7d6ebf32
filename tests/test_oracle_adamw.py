"""Pins for oracle/adamw.py: a library routine (torch.optim.AdamW in fp64 on the CPU) and
two closed forms.  CPU only."""
import numpy as np
import torch

from oracle.adamw import adamw_step


def test_against_torch_adamw_fp64():
    rng = np.random.default_rng(0)
    n = 257
    p0 = rng.normal(0, 0.02, n)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([tp], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"], amsgrad=False, foreach=False)
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        g = rng.normal(0, 1e-3, n) * (10.0 ** rng.integers(-6, 2, n))
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = adamw_step(p, m, v, g, t, **hp)
        st = opt.state[tp]
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-12, atol=1e-15)
        assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=0)
        assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=0)


def test_first_step_closed_form_without_decay():
    """t = 1, m = v = 0: m_hat = g, v_hat = g*g, so p1 = p0 - lr * g / (|g| + eps)."""
    g = np.array([1e-3, -2e-5, 3.0, 1e-9, 0.0])
    p0 = np.array([0.1, -0.2, 0.3, 0.4, 0.5])
    p, m, v = adamw_step(p0, np.zeros(5), np.zeros(5), g, 1, 1e-3, 0.9, 0.95, 1e-8, 0.0)
    assert np.allclose(p, p0 - 1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-13, atol=0)
    assert np.allclose(m, 0.1 * g, rtol=1e-13) and np.allclose(v, 0.05 * g * g, rtol=1e-13)


def test_zero_gradient_is_pure_decay():
    p0 = np.array([0.5, -1.0])
    p, m, v = adamw_step(p0, np.zeros(2), np.zeros(2), np.zeros(2), 3, 1e-2, 0.9, 0.95, 1e-8, 0.1)
    assert np.allclose(p, p0 * (1 - 1e-3), rtol=1e-15) and not m.any() and not v.any()


def test_decay_is_decoupled_from_the_moments():
    """Weight decay must not enter m or v (the difference from Adam with L2)."""
    g = np.array([1e-3, 2e-3])
    a = adamw_step(np.array([1.0, 2.0]), np.zeros(2), np.zeros(2), g, 1, 1e-3, 0.9, 0.95, 1e-8, 0.0)
    b = adamw_step(np.array([1.0, 2.0]), np.zeros(2), np.zeros(2), g, 1, 1e-3, 0.9, 0.95, 1e-8, 0.5)
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    assert np.allclose(a[0] - b[0], 1e-3 * 0.5 * np.array([1.0, 2.0]), rtol=1e-12)
