"""Pins of the oracle's DDPM tables against closed forms (no GPU)."""
import numpy as np
import pytest

from oracle.ddpm import Schedule


@pytest.mark.parametrize("T,kind", [(10, 0), (100, 1), (100, 0), (1000, 1)])
def test_tables_closed_forms(T, kind):
    s = Schedule(T, kind, 1e-4, 0.02, round_fp32=False)
    beta, abar = s.beta, s.abar
    assert np.all(beta > 0) and np.all(beta < 1)
    assert np.all(np.diff(abar) < 0)                                  # abar strictly decreasing
    abar_prev = np.concatenate([[1.0], abar[:-1]])
    assert s.sigma[0] == 0.0                                          # no noise at the last step
    assert np.all(s.sigma[1:] > 0)
    assert np.all(s.sigma ** 2 <= beta + 1e-15)                       # posterior variance <= beta_t
    # noise-free consistency: a state built from x0 with eps = 0 maps to sqrt(abar_{t-1}) x0
    np.testing.assert_allclose(s.c0 + s.cx * np.sqrt(abar), np.sqrt(abar_prev), rtol=1e-12)
    # x0-form of the posterior mean == eps-form (x - beta/sqrt(1-abar) eps)/sqrt(alpha)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((T, 5)); e = rng.standard_normal((T, 5)); t = np.arange(T)
    mu = s.posterior_mean(x, e, t)
    ref = (x - (beta / np.sqrt(1 - abar))[:, None] * e) / np.sqrt(1 - beta)[:, None]
    np.testing.assert_allclose(mu, ref, rtol=1e-9, atol=1e-12)
    # sigma_t^2 = beta_t (1 - abar_{t-1}) / (1 - abar_t), written from scratch
    np.testing.assert_allclose(s.sigma ** 2, beta * (1 - abar_prev) / (1 - abar), rtol=1e-12)


def test_linear_schedule_values():
    s = Schedule(10, 0, 1e-4, 0.02, round_fp32=False)
    assert s.beta[0] == pytest.approx(1e-4) and s.beta[-1] == pytest.approx(0.02)
    np.testing.assert_allclose(np.diff(s.beta), (0.02 - 1e-4) / 9, rtol=1e-12)
    assert s.abar[0] == pytest.approx(1 - 1e-4)


def test_squared_cosine_closed_form():
    T = 100
    s = Schedule(T, 1, round_fp32=False)
    f = lambda i: np.cos(((i / T) + 0.008) / 1.008 * np.pi / 2) ** 2
    uncapped = 1 - f(np.arange(1, T + 1)) / f(np.arange(T)) < 0.999
    n = int(np.argmin(uncapped)) if not uncapped.all() else T        # first capped index
    np.testing.assert_allclose(s.abar[:n], f(np.arange(1, n + 1)) / f(0), rtol=1e-12)
    assert s.beta.max() <= 0.999
    assert s.beta[-1] == 0.999                                        # the final step hits the cap


def test_fp32_rounding_is_small_and_clip_only_touches_x0():
    a, b = Schedule(100, 1, round_fp32=False), Schedule(100, 1, round_fp32=True)
    for k in ("sqrt_abar", "sqrt_1m", "c0", "cx", "sigma"):
        np.testing.assert_allclose(getattr(a, k), getattr(b, k), rtol=6e-8, atol=0)
    x = np.full((1, 3), 5.0); e = np.zeros((1, 3)); t = np.array([50])
    x0 = x / b.sqrt_abar[50]
    np.testing.assert_allclose(b.posterior_mean(x, e, t, clip=1.0), b.c0[50] * 1.0 + b.cx[50] * x)
    assert np.all(x0 > 1.0)


def test_ddim_tables():
    T = 100
    for kind in (0, 1):
        d = Schedule(T, kind, 1e-4, 0.02, round_fp32=False)
        i = Schedule(T, kind, 1e-4, 0.02, round_fp32=False, sampler=1, eta=1.0)
        # eta = 1: the DDIM transition is the DDPM posterior (same variance, same mean when x0 is not clamped)
        np.testing.assert_allclose(i.sigma, d.sigma, rtol=1e-12, atol=1e-15)
        rng = np.random.default_rng(1)
        x = rng.standard_normal((T, 4)); e = rng.standard_normal((T, 4)); t = np.arange(T)
        np.testing.assert_allclose(i.posterior_mean(x, e, t), d.posterior_mean(x, e, t), rtol=1e-9, atol=1e-12)
        # any eta: marginal consistency  abar_{t-1} = c0^2 abar-free form:  c0 = sqrt(abar_{t-1}),  ce^2 + sigma^2 = 1 - abar_{t-1}
        h = Schedule(T, kind, 1e-4, 0.02, round_fp32=False, sampler=1, eta=0.4)
        abar_prev = np.concatenate([[1.0], h.abar[:-1]])
        np.testing.assert_allclose(h.c0, np.sqrt(abar_prev), rtol=1e-12)
        np.testing.assert_allclose(h.ce ** 2 + h.sigma ** 2, 1 - abar_prev, rtol=1e-9, atol=1e-15)
        np.testing.assert_allclose(h.sigma, 0.4 * d.sigma, rtol=1e-12, atol=1e-15)
        assert h.sigma[0] == 0 and np.all(h.cx == 0) and h.ce[0] == 0       # last step returns x0_hat
        # a state built from (x0, eps) maps to sqrt(abar_{t-1}) x0 + ce eps: the noise direction is kept
        x0 = rng.standard_normal((T, 4)); eps = rng.standard_normal((T, 4))
        xt = h.sqrt_abar[:, None] * x0 + h.sqrt_1m[:, None] * eps
        np.testing.assert_allclose(h.posterior_mean(xt, eps, t), np.sqrt(abar_prev)[:, None] * x0 + h.ce[:, None] * eps,
                                   rtol=1e-9, atol=1e-12)
    with pytest.raises(ValueError):
        Schedule(T, 0, sampler=1, eta=0.0)
