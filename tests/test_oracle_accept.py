"""Pins of the oracle's acceptance arithmetic against closed forms and laws (no GPU)."""
import itertools

import numpy as np
from scipy import stats

from oracle import philox, spec_round as sr


def test_log_ratio_equals_gaussian_log_density_difference():
    # log alpha = log N(x; mu_q, s^2 I) - log N(x; mu_p, s^2 I) at x = mu_p + s xi  (Section 3.1 ratio
    # vs Section 3.2 closed form): the densities come from scipy, not from the oracle's formula.
    rng = np.random.default_rng(1)
    for D in (2, 32, 160):
        mu_p = rng.standard_normal((6, D)); mu_q = mu_p + 0.3 * rng.standard_normal((6, D))
        sig = rng.uniform(0.05, 2.0, 6); xi = rng.standard_normal((6, D))
        l, dd, dx = sr.log_ratio(mu_p, mu_q, sig, xi)
        for r in range(6):
            x = mu_p[r] + sig[r] * xi[r]
            ref = stats.norm.logpdf(x, mu_q[r], sig[r]).sum() - stats.norm.logpdf(x, mu_p[r], sig[r]).sum()
            assert abs(l[r] - ref) < 1e-9 * max(1.0, abs(ref))
            assert dd[r] >= 0


def test_acceptance_probability_is_one_minus_total_variation():
    # E[accept] = 1 - TV(N(mu_p), N(mu_q)) = 2 Phi(-|d|/2) for equal isotropic covariances.
    n, D = 120_000, 8
    env = np.arange(n) % 4096; t = 1 + np.arange(n) // 4096
    xi = philox.normal(11, env, t, D)
    logu = np.log(philox.uniform(11, env, t))
    rng = np.random.default_rng(2)
    for delta in (0.0, 0.1, 0.5, 1.0, 2.0, 4.0):
        dirn = rng.standard_normal(D); dirn /= np.linalg.norm(dirn)
        sig = 0.7
        mu_q = np.zeros((n, D)); mu_p = mu_q + delta * sig * dirn
        l, _, _ = sr.log_ratio(mu_p, mu_q, np.full(n, sig), xi)
        rate = np.mean(logu <= l)
        p = 2 * stats.norm.cdf(-delta / 2)
        assert abs(rate - p) <= 4 * np.sqrt(max(p * (1 - p), 1e-12) / n) + 1e-12, (delta, rate, p)


def test_first_rejection_brute_force():
    for K in range(0, 9):
        for pat in itertools.product([0, 1], repeat=K):
            j = sr.first_rejection(pat)
            rej = [i + 1 for i, a in enumerate(pat) if a == 0]
            assert j == (min(rej) if rej else K + 1)
            assert all(pat[i] == 1 for i in range(j - 1))            # the committed prefix is all accepted


def test_reflection_is_an_isometry_that_flips_only_the_mean_difference_axis():
    rng = np.random.default_rng(3)
    for D in (2, 7, 160):
        mu_p = rng.standard_normal(D); mu_q = rng.standard_normal(D); xi = rng.standard_normal(D); sig = 0.37
        x = sr.reflect(mu_p, mu_q, sig, xi)
        e = (mu_p - mu_q) / np.linalg.norm(mu_p - mu_q)
        a, b = x - mu_q, sig * xi                                     # corrected and drafted offsets
        assert abs(np.linalg.norm(a) - np.linalg.norm(b)) < 1e-12
        assert abs(a @ e + b @ e) < 1e-12                             # component along e changes sign
        np.testing.assert_allclose(a - (a @ e) * e, b - (b @ e) * e, atol=1e-12)   # the rest is kept
        np.testing.assert_allclose(sr.reflect(mu_p, mu_q, sig, (x - mu_q) / sig),  # an involution
                                   mu_q + sig * xi, atol=1e-12)


def _one_step_outputs(n, mu_p, mu_q, sig, seed):
    D = len(mu_p)
    env = np.arange(n) % 8192; t = 1 + np.arange(n) // 8192
    xi = philox.normal(seed, env, t, D)
    logu = np.log(philox.uniform(seed, env, t))
    MP = np.broadcast_to(mu_p, (n, D)); MQ = np.broadcast_to(mu_q, (n, D))
    l, _, _ = sr.log_ratio(MP, MQ, np.full(n, sig), xi)
    acc = logu <= l
    out = MP + sig * xi
    for i in np.nonzero(~acc)[0]:
        out[i] = sr.reflect(mu_p, mu_q, sig, xi[i])
    return out, acc


def test_accept_or_reflect_output_follows_the_target_law():
    # Marginal of (accepted draft) U (reflected draft) is exactly N(mu_q, sig^2 I)  (Section 3.1).
    n = 100_000
    mu_p = np.array([0.4, -0.2]); mu_q = np.array([-0.1, 0.3]); sig = 0.5
    out, acc = _one_step_outputs(n, mu_p, mu_q, sig, seed=21)
    assert 0.2 < acc.mean() < 0.8                                     # both branches are exercised
    z = (out - mu_q) / sig
    for a in range(2):
        assert stats.kstest(z[:, a], "norm").pvalue > 1e-3
        assert abs(z[:, a].mean()) < 4 / np.sqrt(n)
        assert abs(z[:, a].var() - 1) < 4 * np.sqrt(2 / n)
    assert abs(np.corrcoef(z.T)[0, 1]) < 4 / np.sqrt(n)
    # along the mean-difference axis too (the axis the reflection acts on)
    e = (mu_p - mu_q) / np.linalg.norm(mu_p - mu_q)
    assert stats.kstest(z @ e, "norm").pvalue > 1e-3
    # the drafted samples themselves follow the draft law, not the target: the test can tell
    zp = (out[acc] - mu_q) / sig
    assert stats.kstest(zp @ e, "norm").pvalue < 1e-6


def test_threshold_rule_is_deterministic_monotone_and_matches_its_definition():
    # Section 3.2: accept iff p = min(1, exp(log alpha)) >= lambda.  Pins: no dependence on the seed, acceptance is
    # non-increasing in lambda, lambda = 1 accepts exactly the rows with log alpha >= 0, a tiny lambda accepts all,
    # and the committed prefix / reflected row follow the same scan as the stochastic rule.
    from oracle.ddpm import Schedule
    rng = np.random.default_rng(8)
    sched = Schedule(100, 1)
    B, K, D = 40, 6, 12
    row_ptr = np.arange(B + 1) * K
    t0 = rng.integers(K, 100, B)
    row_t = (t0[:, None] - np.arange(K)[None]).ravel()
    states = rng.standard_normal((B * K, D)); eps_p = 0.3 * rng.standard_normal((B * K, D))
    eps_q = eps_p + 0.2 * rng.standard_normal((B * K, D)); xi = rng.standard_normal((B * K, D))
    y_last = rng.standard_normal((B, D)); s = np.ones(B)
    prev = None
    for lam in (1e-12, 0.05, 0.3, 0.7, 1.0):
        a = sr.accept(sched, row_ptr, row_t, s, None, 1, states, eps_p, eps_q, xi, y_last, lam=np.full(B, lam))
        b = sr.accept(sched, row_ptr, row_t, s, None, 999, states, eps_p, eps_q, xi, y_last, lam=np.full(B, lam))
        np.testing.assert_array_equal(a["flags"], b["flags"])                      # no random number is consumed
        np.testing.assert_array_equal(a["flags"], (np.minimum(1, np.exp(a["logratio"])) >= lam).astype(np.uint8))
        if prev is not None:
            assert np.all(a["flags"] <= prev)                                       # monotone in lambda
        prev = a["flags"]
        for e in range(B):
            f = a["flags"][e * K:(e + 1) * K]
            assert a["n_accept"][e] == sr.first_rejection(f) - 1
    assert sr.accept(sched, row_ptr, row_t, s, None, 1, states, eps_p, eps_q, xi, y_last, lam=1e-12)["flags"].all()
    one = sr.accept(sched, row_ptr, row_t, s, None, 1, states, eps_p, eps_q, xi, y_last, lam=1.0)
    np.testing.assert_array_equal(one["flags"], (one["logratio"] >= 0).astype(np.uint8))


def test_distillation_loss_closed_forms():
    # eps_hat = eps + c  =>  L_pred = D c^2 and, without clipping, mu_hat - mu = -(beta_t/(sqrt(alpha_t) sqrt(1-abar_t))) c
    # (textbook eps-form of the posterior mean), so L_norm = D c^2 mean_t (beta_t/(sqrt(alpha_t) sqrt(1-abar_t) sigma_t))^2.
    from oracle.ddpm import Schedule
    T, R, D, c = 100, 64, 12, 0.3
    sched = Schedule(T, 1, round_fp32=False)
    rng = np.random.default_rng(9)
    row_t = rng.integers(1, T, R)
    states = rng.standard_normal((R, D)); eps_q = rng.standard_normal((R, D)); eps_p = eps_q + c
    lp, ln, l = sr.distill_loss(sched, row_t, states, eps_p, eps_q, 0.7, 0.2)
    beta, abar = sched.beta, sched.abar
    abar_prev = np.concatenate([[1.0], abar[:-1]])
    with np.errstate(divide="ignore"):                                 # entry t = 0 (sigma_0 = 0) is never indexed
        kap = beta / (np.sqrt(1 - beta) * np.sqrt(1 - abar)) / np.sqrt(beta * (1 - abar_prev) / (1 - abar))
    assert abs(lp - D * c * c) < 1e-12
    assert abs(ln - D * c * c * np.mean(kap[row_t] ** 2)) < 1e-9 * ln
    assert abs(l - (0.7 * lp + 0.2 * ln)) < 1e-12
    # identical networks give zero; t = 0 rows contribute to L_pred only
    assert sr.distill_loss(sched, row_t, states, eps_q, eps_q, 1, 1) == (0.0, 0.0, 0.0)
    lp0, ln0, _ = sr.distill_loss(sched, np.zeros(R, int), states, eps_p, eps_q, 1, 1)
    assert abs(lp0 - D * c * c) < 1e-12 and ln0 == 0.0
    # the normalised term is the mean |d|^2 of the acceptance ratio at sigma scale 1
    mu_p = sched.posterior_mean(states, eps_p, row_t); mu_q = sched.posterior_mean(states, eps_q, row_t)
    _, dd, _ = sr.log_ratio(mu_p, mu_q, sched.sigma[row_t], np.zeros((R, D)))
    assert abs(ln - dd.mean()) < 1e-9 * ln
