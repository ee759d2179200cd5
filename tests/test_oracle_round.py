"""Pins of the oracle's round: identity-drafter invariant and whole-chain law (no GPU)."""
import numpy as np
from scipy import stats

import tsdp_inputs as ti
from oracle import spec_round as sr
from oracle.ddpm import Schedule
from oracle.denoiser import Denoiser


class LinearEps:
    """Toy denoiser eps(x, t) = a_t x + b_t: makes the base chain linear-Gaussian."""

    def __init__(self, a, b):
        self.a, self.b = np.asarray(a, float), np.asarray(b, float)

    def __call__(self, x, t, cond):
        sh = (-1,) + (1,) * (x.ndim - 1)
        return self.a[t].reshape(sh) * x + self.b[t].reshape(sh)


def _closed_form_chain_ddim(T, kind, a, b, s, eta, beta0=1e-4, beta1=0.02):
    """Final mean / variance of the base DDIM(eta) chain for eps(x,t) = a_t x + b_t, from the textbook update
    x' = sqrt(abar') (x - sqrt(1-abar) eps)/sqrt(abar) + sqrt(1-abar'-sig^2) eps + s sig z."""
    if kind == 0:
        beta = np.linspace(beta0, beta1, T)
    else:
        f = lambda i: np.cos(((i / T) + 0.008) / 1.008 * np.pi / 2) ** 2
        beta = np.minimum(1 - f(np.arange(1, T + 1)) / f(np.arange(T)), 0.999)
    abar = np.cumprod(1 - beta); abar_prev = np.concatenate([[1.0], abar[:-1]])
    m, v = 0.0, 1.0
    for t in range(T - 1, -1, -1):
        sig = eta * np.sqrt((1 - abar_prev[t]) / (1 - abar[t])) * np.sqrt(1 - abar[t] / abar_prev[t])
        r = np.sqrt(abar_prev[t] / abar[t]); ce = np.sqrt(max(1 - abar_prev[t] - sig ** 2, 0.0))
        A = r + (ce - r * np.sqrt(1 - abar[t])) * a[t]; Bc = (ce - r * np.sqrt(1 - abar[t])) * b[t]
        m, v = A * m + Bc, A * A * v + (s * sig) ** 2
    return m, v


def _closed_form_chain(T, kind, a, b, s, beta0=1e-4, beta1=0.02):
    """Mean and variance of x_{-1} for x_{T-1} ~ N(0,1) under the base chain, from the textbook
    posterior written in its eps-form: x' = (x - beta/sqrt(1-abar) eps)/sqrt(alpha) + s sigma z."""
    if kind == 0:
        beta = np.linspace(beta0, beta1, T)
    else:
        f = lambda i: np.cos(((i / T) + 0.008) / 1.008 * np.pi / 2) ** 2
        beta = np.minimum(1 - f(np.arange(1, T + 1)) / f(np.arange(T)), 0.999)
    abar = np.cumprod(1 - beta); abar_prev = np.concatenate([[1.0], abar[:-1]])
    m, v = 0.0, 1.0
    for t in range(T - 1, -1, -1):
        ce = beta[t] / np.sqrt(1 - abar[t]); ra = 1 / np.sqrt(1 - beta[t])
        A = ra * (1 - ce * a[t]); Bc = -ra * ce * b[t]
        var = beta[t] * (1 - abar_prev[t]) / (1 - abar[t]) if t > 0 else 0.0
        m, v = A * m + Bc, A * A * v + s * s * var
    return m, v


def _run_chains(base, drafter, sched, n, K, s, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, 1, 2))
    t = np.full(n, sched.T - 1)
    cond = np.zeros((n, 1))
    tot_acc = tot_draft = rounds = 0
    while np.any(t >= 0):
        r = sr.spec_round(base, drafter, sched, x, t, np.full(n, K), np.full(n, s), None, seed, cond)
        tot_acc += int(r["n_accept"].sum()); tot_draft += int(r["draft"]["K_eff"].sum())
        assert np.all(r["n_adv"][t >= 0] >= 1)                        # every live env advances
        x, t = r["x_out"], r["t_next"]
        rounds += 1
        assert rounds <= sched.T + 1
    return x.reshape(n, 2), tot_acc / max(tot_draft, 1), rounds


def _check_law(x, m, v):
    n = x.shape[0]
    z = (x - m) / np.sqrt(v)
    for a in range(2):
        assert stats.kstest(z[:, a], "norm").pvalue > 1e-3
        assert abs(z[:, a].mean()) < 4 / np.sqrt(n)
        assert abs(z[:, a].var() - 1) < 4.5 * np.sqrt(2 / n)
    assert abs(np.corrcoef(z.T)[0, 1]) < 4 / np.sqrt(n)


def test_chain_with_imperfect_drafter_keeps_the_base_law():
    # Lossless speculation: full chains driven by repeated rounds with a perturbed drafter end in the
    # same law as the base DDPM chain, whose final mean / variance are known in closed form.
    T, n = 10, 100_000
    rng = np.random.default_rng(5)
    a = rng.uniform(0.2, 0.8, T); b = rng.uniform(-0.5, 0.5, T)
    base = LinearEps(a, b)
    drafter = LinearEps(a + rng.uniform(-0.25, 0.25, T), b + rng.uniform(-0.6, 0.6, T))
    sched = Schedule(T, 0, 1e-4, 0.02, round_fp32=False)
    x, rate, rounds = _run_chains(base, drafter, sched, n, K=4, s=1.0, seed=77)
    assert 0.3 < rate < 0.97 and rounds < T                           # rejections happen, and drafts help
    m, v = _closed_form_chain(T, 0, a, b, 1.0)
    _check_law(x, m, v)
    # sanity of the detector: the drafter's own chain has a different law
    md, vd = _closed_form_chain(T, 0, drafter.a, drafter.b, 1.0)
    assert abs(md - m) / np.sqrt(v) > 0.05


def test_chain_with_sigma_scale_matches_the_variance_inflated_base_chain():
    T, n = 10, 60_000
    rng = np.random.default_rng(6)
    a = rng.uniform(0.2, 0.8, T); b = rng.uniform(-0.5, 0.5, T)
    base = LinearEps(a, b)
    drafter = LinearEps(a + rng.uniform(-0.05, 0.05, T), b + rng.uniform(-0.1, 0.1, T))
    sched = Schedule(T, 1, round_fp32=False)
    x, rate, _ = _run_chains(base, drafter, sched, n, K=3, s=1.3, seed=78)
    assert 0.2 < rate < 0.98
    m, v = _closed_form_chain(T, 1, a, b, 1.3)
    _check_law(x, m, v)


def _tiny_nets(bf16=False):
    wl = ti.small_variant(ti.C1)
    wb = ti.make_weights(wl, "base", b_std=0.02)
    base = Denoiser(wb, wl.base.layers, wl.base.heads, wl.cond_mode, bf16)
    return wl, base


def test_identity_drafter_accepts_everything_and_reproduces_the_base_chain():
    # drafter == base  =>  d = 0  =>  log alpha = 0 >= log U: all K_eff drafts accepted, and since the
    # noise is a function of (env, t) the output equals K_eff plain base DDPM steps.
    wl, base = _tiny_nets()
    sched = Schedule(wl.T, wl.schedule, wl.beta0, wl.beta1)
    B = 5
    x = ti.make_latents(wl, B); cond = ti.make_cond(wl, B)
    t0 = np.array([9, 7, 2, 0, -1]); K = np.array([4, 4, 4, 4, 4]); s = np.array([1.0, 1.2, 1.0, 1.0, 1.0])
    env = np.array([10, 11, 12, 13, 14])
    r = sr.spec_round(base, base, sched, x, t0, K, s, env, 0, cond)
    np.testing.assert_array_equal(r["draft"]["K_eff"], [4, 4, 2, 0, 0])
    np.testing.assert_array_equal(r["n_accept"], [4, 4, 2, 0, 0])
    np.testing.assert_array_equal(r["n_adv"], [4, 4, 2, 1, 0])
    np.testing.assert_array_equal(r["t_next"], [5, 3, 0, -1, -1])
    np.testing.assert_allclose(r["logratio"], 0.0, atol=1e-12)   # batched vs row-wise matmul rounding only
    ref = np.asarray(x, float).copy()
    for b in range(B):
        xb, tb = ref[b:b + 1], t0[b]
        for _ in range(r["n_adv"][b]):
            xb = sr.base_chain_step(base, sched, xb, np.array([tb]), s[b:b + 1], env[b:b + 1], 0, cond[b:b + 1])
            tb -= 1
        ref[b] = xb[0]
    np.testing.assert_allclose(r["x_out"], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_array_equal(r["x_out"][4], np.asarray(x[4], float))      # finished env untouched


def test_round_is_independent_of_batch_composition_and_row_table_is_consistent():
    wl, base = _tiny_nets()
    wd = ti.make_weights(wl, "draft", b_std=0.02)
    drafter = Denoiser(wd, wl.draft.layers, wl.draft.heads, wl.cond_mode)
    sched = Schedule(wl.T, wl.schedule, wl.beta0, wl.beta1)
    B = 6
    x = ti.make_latents(wl, B); cond = ti.make_cond(wl, B)
    t0 = np.array([9, 5, 3, 1, 0, 8]); K = np.array([4, 2, 4, 4, 3, 1]); s = np.linspace(1, 1.5, B)
    env = np.arange(B) + 100
    full = sr.spec_round(base, drafter, sched, x, t0, K, s, env, 3, cond)
    d = full["draft"]
    np.testing.assert_array_equal(d["K_eff"], [4, 2, 3, 1, 0, 1])
    np.testing.assert_array_equal(np.diff(d["row_ptr"]), [4, 2, 3, 1, 1, 1])
    for b in range(B):
        rows = slice(d["row_ptr"][b], d["row_ptr"][b + 1])
        np.testing.assert_array_equal(d["row_env"][rows], b)
        np.testing.assert_array_equal(d["row_t"][rows], t0[b] - np.arange(rows.stop - rows.start))
        one = sr.spec_round(base, drafter, sched, x[b:b + 1], t0[b:b + 1], K[b:b + 1], s[b:b + 1],
                            env[b:b + 1], 3, cond[b:b + 1])
        np.testing.assert_allclose(one["x_out"][0], full["x_out"][b], rtol=1e-9, atol=1e-12)
        assert one["n_accept"][0] == full["n_accept"][b] and one["t_next"][0] == full["t_next"][b]
        np.testing.assert_array_equal(one["flags"], full["flags"][rows])
    # each drafted state is the draft sample of the previous row: y_k = mu_p + s sigma xi
    for b in range(B):
        for k in range(1, d["K_eff"][b]):
            r0 = d["row_ptr"][b] + k - 1
            t = d["row_t"][r0]
            mu = sched.posterior_mean(d["states"][r0][None], d["eps_p"][r0][None], np.array([t]))[0]
            np.testing.assert_allclose(d["states"][r0 + 1], mu + s[b] * sched.sigma[t] * d["xi"][r0], rtol=1e-12)
    # with random independent nets some draft is rejected somewhere and the reflected output differs from y
    assert (full["n_accept"] < d["K_eff"]).any()


def test_ddim_chain_with_imperfect_drafter_keeps_the_base_law():
    T, n = 10, 60_000
    rng = np.random.default_rng(12)
    a = rng.uniform(0.2, 0.8, T); b = rng.uniform(-0.5, 0.5, T)
    base = LinearEps(a, b)
    drafter = LinearEps(a + rng.uniform(-0.1, 0.1, T), b + rng.uniform(-0.2, 0.2, T))
    sched = Schedule(T, 0, 1e-4, 0.02, round_fp32=False, sampler=1, eta=0.7)
    x, rate, rounds = _run_chains(base, drafter, sched, n, K=4, s=1.0, seed=91)
    assert 0.2 < rate < 0.98
    m, v = _closed_form_chain_ddim(T, 0, a, b, 1.0, 0.7)
    _check_law(x, m, v)


def test_bonus_row_identity_drafter_advances_one_extra_exact_base_step():
    # K+1 candidate set: with drafter == base every draft passes and the round must equal K_eff + 1 plain base steps
    wl, base = _tiny_nets()
    sched = Schedule(wl.T, wl.schedule, wl.beta0, wl.beta1)
    B = 6
    x = ti.make_latents(wl, B); cond = ti.make_cond(wl, B)
    t0 = np.array([9, 4, 2, 0, -1, 6]); K = np.array([4, 4, 4, 4, 4, 0]); s = np.array([1.0, 1.2, 1.0, 1.0, 1.0, 1.1])
    env = np.arange(B) + 20
    r = sr.spec_round(base, base, sched, x, t0, K, s, env, 0, cond, bonus=True)
    d = r["draft"]
    np.testing.assert_array_equal(d["K_eff"], [4, 4, 2, 0, 0, 0])
    np.testing.assert_array_equal(np.diff(d["row_ptr"]), [5, 5, 3, 1, 0, 1])
    np.testing.assert_array_equal(r["n_accept"], [4, 4, 2, 0, 0, 0])
    np.testing.assert_array_equal(r["n_adv"], [5, 5, 3, 1, 0, 1])
    np.testing.assert_array_equal(r["t_next"], [4, -1, -1, -1, -1, 5])
    for b in range(B):                                                     # row timesteps run down to t0 - K_eff
        rows = slice(d["row_ptr"][b], d["row_ptr"][b + 1])
        np.testing.assert_array_equal(d["row_t"][rows], t0[b] - np.arange(rows.stop - rows.start))
    ref = np.asarray(x, float).copy()
    for b in range(B):
        xb, tb = ref[b:b + 1], t0[b]
        for _ in range(r["n_adv"][b]):
            xb = sr.base_chain_step(base, sched, xb, np.array([tb]), s[b:b + 1], env[b:b + 1], 0, cond[b:b + 1])
            tb -= 1
        ref[b] = xb[0]
    np.testing.assert_allclose(r["x_out"], ref, rtol=1e-10, atol=1e-12)
    # without the bonus row K = 0 is refused
    try:
        sr.plan_rows(np.array([5]), np.array([0]))
        raise AssertionError("K = 0 accepted without the bonus row")
    except ValueError:
        pass


def test_bonus_row_chain_keeps_the_base_law_and_needs_fewer_rounds():
    T, n = 10, 100_000
    rng = np.random.default_rng(15)
    a = rng.uniform(0.2, 0.8, T); b = rng.uniform(-0.5, 0.5, T)
    base = LinearEps(a, b)
    drafter = LinearEps(a + rng.uniform(-0.25, 0.25, T), b + rng.uniform(-0.6, 0.6, T))
    sched = Schedule(T, 0, 1e-4, 0.02, round_fp32=False)
    x0 = np.random.default_rng(79).standard_normal((n, 1, 2))
    cond = np.zeros((n, 1))
    t0 = np.full(n, T - 1)
    plain = sr.chain(base, drafter, sched, x0, t0, np.full(n, 3), np.ones(n), None, 79, cond)
    bonus = sr.chain(base, drafter, sched, x0, t0, np.full(n, 3), np.ones(n), None, 79, cond, bonus=True)
    m, v = _closed_form_chain(T, 0, a, b, 1.0)
    _check_law(bonus["x"].reshape(n, 2), m, v)
    _check_law(plain["x"].reshape(n, 2), m, v)
    assert (bonus["t"] == -1).all() and (plain["t"] == -1).all()
    assert bonus["totals"]["rounds"].mean() < plain["totals"]["rounds"].mean()
    # steps advanced add up to the chain length: accepted + one corrected or base step per round ran, at most
    assert ((bonus["totals"]["accept"] + bonus["totals"]["rounds"]) >= T).all()


def test_stage_tables_select_by_timestep_and_reduce_to_the_plain_chain():
    # selection: brute force over every timestep
    tab = np.array([[1, 5, 2], [3, 4, 6]])
    for t in range(-1, 12):
        got = sr.stage_select(np.array([t, t]), 8, 3, tab)
        want = tab[:, 0] if t >= 8 else (tab[:, 1] if t >= 3 else tab[:, 2])
        np.testing.assert_array_equal(got, want)
    wl, base = _tiny_nets()
    sched = Schedule(wl.T, wl.schedule, wl.beta0, wl.beta1)
    B = 4
    x = ti.make_latents(wl, B); cond = ti.make_cond(wl, B)
    t0 = np.array([9, 9, 5, 2])
    # constant tables == the plain chain
    K = np.array([3, 2, 4, 1]); s = np.array([1.0, 1.1, 1.0, 1.2])
    wd = ti.make_weights(wl, "draft", b_std=0.02)
    drafter = Denoiser(wd, wl.draft.layers, wl.draft.heads, wl.cond_mode)
    a = sr.chain(base, drafter, sched, x, t0, K, s, None, 4, cond)
    b = sr.chain(base, drafter, sched, x, t0, np.repeat(K[:, None], 3, 1), np.repeat(s[:, None], 3, 1), None, 4, cond,
                 stages=(7, 3))
    np.testing.assert_array_equal(a["x"], b["x"])
    assert a["rounds"] == b["rounds"]
    # identity drafter: every draft passes, so the round count follows from the K table alone
    Kt = np.array([[1, 4, 2]] * B); st = np.ones((B, 3))
    c = sr.chain(base, base, sched, x, t0, Kt, st, None, 4, cond, stages=(7, 3))
    want = []
    for t in t0:
        n = 0
        while t >= 0:
            k = 1 if t >= 7 else (4 if t >= 3 else 2)
            t -= max(min(k, t), 1); n += 1
        want.append(n)
    np.testing.assert_array_equal(c["totals"]["rounds"], want)
    np.testing.assert_array_equal(c["totals"]["accept"], c["totals"]["drafts"])
