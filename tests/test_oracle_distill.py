"""Pins for the oracle's distillation loss (Eq. (7), one student/teacher pair): autograd of the
library routines in float64, and closed forms."""
import numpy as np
import pytest


def _torch_ref(a, b, lam, eps, upstream):
    import torch
    import torch.nn.functional as F
    ta = torch.tensor(a.astype(np.float64), requires_grad=True)
    tb = torch.tensor(b.astype(np.float64))
    cos = F.cosine_similarity(ta, tb, dim=1, eps=eps)            # [N, M]
    mse = F.mse_loss(ta, tb)
    loss = mse + lam * (1.0 - cos.mean())
    (loss * upstream).backward()
    return float(mse.detach()), float(cos.mean().detach()), float(loss.detach()), ta.grad.numpy()


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_against_torch_autograd(oracle, dtype):
    rng = np.random.default_rng(4)
    n, c, m = 3, 17, 29
    a = (rng.standard_normal((n, c, m)) * 1.5).astype(dtype)
    b = (a.astype(np.float64) * 0.8 + rng.standard_normal((n, c, m)) * 0.4).astype(dtype)
    mse, cosim, loss, ga = oracle.distill(a, b, lam=0.37, eps=1e-8, upstream=1.7)
    r_mse, r_cos, r_loss, r_g = _torch_ref(a, b, 0.37, 1e-8, 1.7)
    assert abs(mse - r_mse) <= 1e-12 * r_mse and abs(cosim - r_cos) <= 1e-12 and abs(loss - r_loss) <= 1e-12 * r_loss
    # ga is rounded once to the I/O dtype: half an ulp, and half a subnormal step (2^-25) for binary16
    rtol, atol = (1e-6, 1e-12) if dtype == np.float32 else (2.0 ** -11, 2.0 ** -25)
    np.testing.assert_allclose(ga.astype(np.float64), r_g, rtol=rtol * 1.001, atol=atol * 1.001)


def test_closed_forms(oracle):
    rng = np.random.default_rng(6)
    a = rng.standard_normal((2, 8, 11)).astype(np.float32)
    # identical: mse 0, cos 1, loss 0, gradient 0
    mse, cosim, loss, ga = oracle.distill(a, a, lam=0.5)
    assert mse == 0.0 and abs(cosim - 1.0) < 1e-12 and abs(loss) < 1e-12 and np.abs(ga).max() < 1e-7
    # opposite: cos -1
    _, cosim, loss, _ = oracle.distill(a, -a, lam=0.5)
    assert abs(cosim + 1.0) < 1e-12
    # cosine ignores a positive rescaling of the student, the MSE does not
    b = rng.standard_normal(a.shape).astype(np.float32)
    m1, c1, _, _ = oracle.distill(a, b, lam=1.0)
    m2, c2, _, _ = oracle.distill(np.float32(2.0) * a, b, lam=1.0)
    assert abs(c1 - c2) < 1e-9 and abs(m1 - m2) > 1e-3
    # orthogonal channel vectors: cos 0; single channel: cos = sign(a*b)
    e = np.zeros((1, 2, 4), np.float32); f = np.zeros((1, 2, 4), np.float32)
    e[0, 0] = 1.0; f[0, 1] = 3.0
    _, cosim, _, _ = oracle.distill(e, f, lam=1.0)
    assert cosim == 0.0
    s = np.array([[[1.0, -2.0, 3.0, -4.0]]], np.float32); t = np.array([[[2.0, 2.0, -1.0, -1.0]]], np.float32)
    _, cosim, _, _ = oracle.distill(s, t, lam=1.0)
    assert cosim == 0.0                                          # (+1 -1 -1 +1) / 4
    mse, _, _, _ = oracle.distill(s, t, lam=0.0)
    assert mse == (1 + 16 + 16 + 9) / 4


def test_axis_and_layout(oracle):
    """The cosine runs over the channel axis of [N, C, M]: permuting channels changes nothing,
    permuting positions changes nothing, but swapping the roles of C and M does."""
    rng = np.random.default_rng(8)
    a = rng.standard_normal((2, 5, 7)).astype(np.float32)
    b = rng.standard_normal((2, 5, 7)).astype(np.float32)
    base = oracle.distill(a, b, lam=0.3)[:3]
    pc, pm = rng.permutation(5), rng.permutation(7)
    np.testing.assert_allclose(oracle.distill(a[:, pc], b[:, pc], lam=0.3)[:3], base, rtol=1e-12)
    np.testing.assert_allclose(oracle.distill(a[:, :, pm], b[:, :, pm], lam=0.3)[:3], base, rtol=1e-12)
    swapped = oracle.distill(np.ascontiguousarray(a.transpose(0, 2, 1)), np.ascontiguousarray(b.transpose(0, 2, 1)),
                             lam=0.3)
    assert abs(swapped[1] - base[1]) > 1e-3 and abs(swapped[0] - base[0]) < 1e-12


def test_zero_student_norm_is_clamped(oracle):
    a = np.zeros((1, 3, 2), np.float32)
    b = np.ones((1, 3, 2), np.float32)
    mse, cosim, loss, ga = oracle.distill(a, b, lam=1.0, eps=1e-8)
    r = _torch_ref(a, b, 1.0, 1e-8, 1.0)
    assert cosim == 0.0 and mse == 1.0
    np.testing.assert_allclose(ga.astype(np.float64), r[3], rtol=1e-6)


def test_nan_poisons_its_position_only(oracle):
    """A NaN in one channel of one position: that position's cosine, hence every channel of its
    gradient, and the three scalars are NaN (the library routines do the same); nothing else is."""
    rng = np.random.default_rng(10)
    a = rng.standard_normal((1, 6, 9)).astype(np.float32)
    b = rng.standard_normal((1, 6, 9)).astype(np.float32)
    a[0, 2, 4] = np.nan
    mse, cosim, loss, ga = oracle.distill(a, b, lam=0.5)
    r = _torch_ref(a, b, 0.5, 1e-8, 1.0)
    assert np.isnan(mse) and np.isnan(cosim) and np.isnan(loss)
    assert np.array_equal(np.isnan(ga), np.isnan(r[3]))
    assert np.isnan(ga[0, :, 4]).all() and not np.isnan(np.delete(ga, 4, axis=2)).any()
    np.testing.assert_allclose(np.delete(ga, 4, axis=2), np.delete(r[3], 4, axis=2), rtol=1e-6)


def test_clamped_norms(oracle):
    """Norms below eps on either side.  Values and, away from a clamped student norm, gradients are
    pinned to the library routines; a zero teacher vector keeps the division finite.  Where the
    student's own norm is clamped the gradient is the derivative of the function as defined
    (max(||a||, eps) is locally the constant eps), pinned by central differences of the oracle's
    own loss, which are exact there up to rounding: with the norm clamped cos is linear in a and
    the MSE is quadratic.  (Autograd of the library's cosine differs at such positions: it uses
    the clamped value of the norm but still differentiates the unclamped norm.)"""
    rng = np.random.default_rng(12)
    a = rng.standard_normal((2, 5, 8)).astype(np.float32)
    b = rng.standard_normal((2, 5, 8)).astype(np.float32)
    unit = np.float32(2.0 ** -30)
    a[0, :, 1] = rng.integers(-16, 17, 5).astype(np.float32) * unit     # ||a|| ~ 2e-8 < eps
    a[1, :, 3] = rng.integers(-16, 17, 5).astype(np.float32) * unit
    b[0, :, 5] = 0.0
    b[1, :, 3] *= np.float32(1e-7)                                       # both below eps at (1, 3)
    eps, lam = 1e-6, 0.8
    mse, cosim, loss, ga = oracle.distill(a, b, lam=lam, eps=eps)
    r_mse, r_cos, r_loss, r_g = _torch_ref(a, b, lam, eps, 1.0)
    assert np.isfinite(ga).all()
    assert abs(mse - r_mse) <= 1e-12 * r_mse and abs(cosim - r_cos) <= 1e-12 and abs(loss - r_loss) <= 1e-12 * r_loss
    clamped = np.zeros(a.shape, bool)
    clamped[0, :, 1] = clamped[1, :, 3] = True
    na = np.sqrt((a.astype(np.float64) ** 2).sum(axis=1))
    assert na[0, 1] < eps and na[1, 3] < eps and (np.delete(na.reshape(-1), [1, 11]) > 0.1).all()
    np.testing.assert_allclose(ga[~clamped].astype(np.float64), r_g[~clamped], rtol=2e-6, atol=1e-12)
    h = np.float32(2.0 ** -34)                    # a +- h is exact for the multiples of 2^-30 above
    for n_, m_ in ((0, 1), (1, 3)):
        for c_ in range(5):
            ap, am = a.copy(), a.copy()
            ap[n_, c_, m_] += h
            am[n_, c_, m_] -= h
            fd = (oracle.distill(ap, b, lam, eps, want_grad=False)[2] -
                  oracle.distill(am, b, lam, eps, want_grad=False)[2]) / (2.0 * float(h))
            assert abs(float(ga[n_, c_, m_]) - fd) <= 2e-6 * abs(fd) + 1e-9, (n_, c_, m_, ga[n_, c_, m_], fd)
    assert np.abs(ga[0, :, 1]).max() > 1e3        # the regime where the clamp matters: cos is far from 0
