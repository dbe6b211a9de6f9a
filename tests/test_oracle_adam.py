"""Pins for the oracle's Adam step on the scale parameters (Sec. 3.2: Adam on the log-scales
only; Kingma & Ba 2015, Algorithm 1)."""
import numpy as np


def test_first_step_closed_form(oracle):
    """With m = v = 0 the first step is theta - lr * g / (|g| + eps) up to float32 rounding:
    m_hat = g and v_hat = g^2 exactly in real arithmetic."""
    g = np.array([0.3, -2.0, 1e-3, 50.0, 0.0], np.float32)
    th = np.array([0.5, -1.0, 2.0, 0.0, 0.7], np.float32)
    z = np.zeros(5, np.float32)
    out, m, v = oracle.adam(g, z, z, th, 1e-2, 0.9, 0.999, 1e-8, 1)
    want = th.astype(np.float64) - 1e-2 * g.astype(np.float64) / (np.abs(g.astype(np.float64)) + 1e-8)
    np.testing.assert_allclose(out, want, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-6)
    np.testing.assert_allclose(v, 0.001 * g.astype(np.float64) ** 2, rtol=1e-5)
    assert out[4] == th[4] and m[4] == 0 and v[4] == 0          # zero gradient, zero state: no move


def test_against_torch_adam_over_steps(oracle):
    import torch
    rng = np.random.default_rng(2)
    c, steps = 16, 12
    th0 = rng.standard_normal(c).astype(np.float32)
    grads = (rng.standard_normal((steps, c)) * np.exp(rng.uniform(-6, 3, (steps, 1)))).astype(np.float32)
    p = torch.tensor(th0.copy(), requires_grad=True)
    opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.999), eps=1e-8)
    th, m, v = th0.copy(), np.zeros(c, np.float32), np.zeros(c, np.float32)
    for t in range(steps):
        p.grad = torch.tensor(grads[t])
        opt.step()
        th, m, v = oracle.adam(grads[t], m, v, th, 3e-3, 0.9, 0.999, 1e-8, t + 1)
        # the library orders its float32 operations differently: a few ulp per step
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=2e-6, atol=2e-7)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-5, atol=1e-12)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-20)


def test_non_finite_gradient_is_skipped(oracle):
    g = np.array([np.nan, np.inf, -np.inf, 1.0], np.float32)
    th = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    m0 = np.array([0.1, 0.2, 0.3, 0.4], np.float32)
    v0 = np.array([0.01, 0.02, 0.03, 0.04], np.float32)
    out, m, v = oracle.adam(g, m0, v0, th, 1e-2, 0.9, 0.999, 1e-8, 3)
    assert np.array_equal(out[:3], th[:3]) and np.array_equal(m[:3], m0[:3]) and np.array_equal(v[:3], v0[:3])
    assert out[3] != th[3] and m[3] != m0[3]


def test_descent_direction_and_step_bound(oracle):
    """Adam's step is bounded by about lr in magnitude and opposes the sign of a steady gradient."""
    g = np.array([0.7, -0.7], np.float32)
    th, m, v = np.zeros(2, np.float32), np.zeros(2, np.float32), np.zeros(2, np.float32)
    for t in range(1, 30):
        new, m, v = oracle.adam(g, m, v, th, 1e-2, 0.9, 0.999, 1e-8, t)
        assert np.all(np.abs(new - th) <= 1e-2 * 1.0001)
        assert new[0] < th[0] and new[1] > th[1]
        th = new
