"""One speculative draft-then-verify denoising round (oracle, fp64).

Follows Section 3.1 (likelihood-ratio test, first-rejection index,
reflection-maximal coupling) and Section 3.2 (drafter rollout with retained
means / noises, batched verification, log acceptance ratio, chronological
commit) of the paper.  Readings taken where the text is silent or garbled:

* A round verifies K_eff = min(K, t0) drafted transitions per environment,
  at the K_eff input states y_0 .. y_{K_eff-1} (y_0 = the current latent);
  the drafted transition k goes from timestep t_k = t0 - k + 1 to t_k - 1.
* Networks are always evaluated at the noise level of their input state.
* The step at t = 0 adds no noise, so it is never drafted: an environment at
  t0 = 0 takes one deterministic base step (K_eff = 0, one verify row).
* The scheduler's sigma scale s multiplies sigma_t identically in the draft
  sample, in the acceptance ratio and in the target law, so the coupling is
  exact with respect to N(mu_q, (s sigma_t)^2 I).
* Acceptance is the stochastic test U <= min(1, q/p), taken as
  log U <= log alpha with equality accepting.
* Environments with t0 < 0 are finished: no rows, latent unchanged.
* Bonus-row variant (the paper's candidate set has K+1 members): the state y_{K_eff} reached by the
  last draft is verified too, at its own timestep t0 - K_eff >= 0; when every draft is accepted the
  base model's prediction there gives one more, exact base step, so the round advances K_eff + 1
  steps.  The lone row of a t0 = 0 environment is the K_eff = 0 case of the same rule.  With the
  bonus row K = 0 is allowed (a plain base step); without it K >= 1.
* Stage tables (the scheduler's action holds one draft count / sigma scale / threshold for each of
  three denoising stages, whose boundaries the paper does not give): stage 0 while t >= t_hi, stage 1
  while t_lo <= t < t_hi, stage 2 below t_lo; the stage is taken at the start of a round.

Rows are stored environment-major, k ascending: row_ptr[b] + (k - 1).
"""
import numpy as np

from . import philox


def plan_rows(t0, K, bonus=False):
    """K_eff and the ragged row table (row_ptr [B+1], row_env [R], row_t [R])."""
    t0 = np.asarray(t0, dtype=np.int64)
    K = np.asarray(K, dtype=np.int64)
    if (K < (0 if bonus else 1)).any():
        raise ValueError("K must be >= 1 (>= 0 with the bonus row)")
    live = t0 >= 0
    K_eff = np.where(live, np.minimum(K, t0), 0)
    nrows = np.where(live, K_eff + 1 if bonus else np.maximum(K_eff, 1), 0)
    row_ptr = np.concatenate([[0], np.cumsum(nrows)]).astype(np.int64)
    R = int(row_ptr[-1])
    row_env = np.zeros(R, dtype=np.int64)
    row_t = np.zeros(R, dtype=np.int64)
    for b in range(len(t0)):
        for j in range(int(nrows[b])):
            row_env[row_ptr[b] + j] = b
            row_t[row_ptr[b] + j] = t0[b] - j
    return K_eff, row_ptr, row_env, row_t


def draft(drafter, sched, x, t0, K, sigma_scale, env_id, seed, cond, clip=None, bonus=False):
    """Drafter rollout (Section 3.2, Draft Generation Procedure).

    For k = 1..K_eff:  eps_p = Mhat(y_{k-1}; t_k),  mu_p = posterior mean,
    y_k = mu_p + s sigma_{t_k} xi_{env,t_k}.  Keeps the input states, the
    drafter outputs and the noise realisations for the acceptance stage.
    """
    x = np.asarray(x, dtype=np.float64)
    B = x.shape[0]
    D = int(np.prod(x.shape[1:]))
    s = np.asarray(sigma_scale, dtype=np.float64)
    t0 = np.asarray(t0, dtype=np.int64)
    env_id = np.arange(B) if env_id is None else np.asarray(env_id, dtype=np.int64)
    K_eff, row_ptr, row_env, row_t = plan_rows(t0, K, bonus)
    R = int(row_ptr[-1])
    states = np.zeros((R,) + x.shape[1:])
    eps_p = np.zeros_like(states)
    xi = np.zeros_like(states)
    y = x.copy()
    for b in np.nonzero((t0 == 0))[0]:              # lone base step: the row carries the latent itself
        states[row_ptr[b]] = x[b]
    for k in range(1, int(K_eff.max(initial=0)) + 1):
        act = np.nonzero(K_eff >= k)[0]
        rows = row_ptr[act] + (k - 1)
        t_k = t0[act] - k + 1
        states[rows] = y[act]
        e = drafter(y[act], t_k, cond[act])
        mu = sched.posterior_mean(y[act], e, t_k, clip)
        z = philox.normal(seed, env_id[act], t_k, D).reshape(mu.shape)
        sig = (s[act] * sched.sigma[t_k]).reshape((-1,) + (1,) * (x.ndim - 1))
        y[act] = mu + sig * z
        eps_p[rows] = e
        xi[rows] = z
    if bonus:                                        # the state after the last draft and the noise of a base step from it
        for b in np.nonzero(t0 >= 0)[0]:
            r, tb = row_ptr[b] + K_eff[b], int(t0[b] - K_eff[b])
            states[r] = y[b]
            if tb > 0:
                xi[r] = philox.normal(seed, env_id[b:b + 1], np.array([tb]), D).reshape(x.shape[1:])
    return dict(K_eff=K_eff, row_ptr=row_ptr, row_env=row_env, row_t=row_t,
                states=states, eps_p=eps_p, xi=xi, y_last=y)


def verify(base, row_env, row_t, states, cond):
    """Batched verification (Section 3.2, Verification of Speculative Drafts):
    the frozen base network scores every candidate row in one batch."""
    if len(row_t) == 0:
        return np.zeros_like(np.asarray(states, dtype=np.float64))
    return base(states, row_t, cond[row_env])


def log_ratio(mu_p, mu_q, sig, xi):
    """log alpha = -1/2 |d|^2 - <d, xi>,  d = (mu_p - mu_q)/sigma  (Section 3.2, log acceptance ratio).

    Rows along axis 0; the remaining axes are reduced.  Returns (log alpha, |d|^2, <d, xi>).
    """
    R = mu_p.shape[0]
    d = ((mu_p - mu_q) / sig.reshape((-1,) + (1,) * (mu_p.ndim - 1))).reshape(R, -1)
    dd = np.sum(d * d, axis=1)
    dx = np.sum(d * xi.reshape(R, -1), axis=1)
    return -0.5 * dd - dx, dd, dx


def first_rejection(flags):
    """j* = smallest 1-based index with a rejected draft, len(flags)+1 if none (Section 3.1)."""
    for j, a in enumerate(flags, start=1):
        if not a:
            return j
    return len(flags) + 1


def reflect(mu_p, mu_q, sig, xi):
    """Reflection-maximal coupling of the rejected draft x~ = mu_p + sig xi (Section 3.1):
    x = mu_q + (I - 2 e e^T)(x~ - mu_p),  e = (mu_p - mu_q)/|mu_p - mu_q|."""
    delta = (mu_p - mu_q).ravel()
    nrm2 = float(delta @ delta)
    v = (sig * xi).ravel()
    if nrm2 == 0.0:                                  # identical means are never rejected; kept total
        return (mu_q.ravel() + v).reshape(mu_q.shape)
    e = delta / np.sqrt(nrm2)
    return (mu_q.ravel() + v - 2.0 * e * float(e @ v)).reshape(mu_q.shape)


def accept(sched, row_ptr, row_t, sigma_scale, env_id, seed, states, eps_p, eps_q, xi, y_last, clip=None, lam=None,
           bonus=False):
    """Acceptance test, first-rejection scan and commit / reflection for every environment.

    lam = None: the lossless stochastic test U <= min(1, alpha) (Section 3.1).  lam = per-environment
    thresholds in (0, 1]: the deterministic rule of Section 3.2, accept iff p = min(1, exp(log alpha)) >= lambda
    (not lossless; "log U" then reports log lambda).

    Returns x_out [B, ...], t_next [B], n_accept [B] (accepted drafts), n_adv [B] (denoising steps
    advanced), and per-row flags / log alpha / log U.
    """
    row_ptr = np.asarray(row_ptr, dtype=np.int64)
    row_t = np.asarray(row_t, dtype=np.int64)
    B = len(row_ptr) - 1
    R = int(row_ptr[-1])
    s = np.asarray(sigma_scale, dtype=np.float64)
    env_id = np.arange(B) if env_id is None else np.asarray(env_id, dtype=np.int64)
    states = np.asarray(states, dtype=np.float64)
    eps_p = np.asarray(eps_p, dtype=np.float64)
    eps_q = np.asarray(eps_q, dtype=np.float64)
    xi = np.asarray(xi, dtype=np.float64)
    y_last = np.asarray(y_last, dtype=np.float64)
    row_env = np.repeat(np.arange(B), np.diff(row_ptr))

    flags = np.zeros(R, dtype=np.uint8)
    logratio = np.zeros(R)
    logu = np.zeros(R)
    mu_q = sched.posterior_mean(states, eps_q, row_t, clip) if R else states
    mu_p = sched.posterior_mean(states, eps_p, row_t, clip) if R else states
    sig = s[row_env] * sched.sigma[row_t] if R else np.zeros(0)
    drafted = row_t > 0                              # t = 0 rows are base steps ...
    if bonus and R:
        drafted[row_ptr[1:][np.diff(row_ptr) > 0] - 1] = False      # ... and so is the last row of every environment
    dr = np.nonzero(drafted)[0]
    if len(dr):
        l, _, _ = log_ratio(mu_p[dr], mu_q[dr], sig[dr], xi[dr])
        logratio[dr] = l
        if lam is None:
            u = philox.uniform(seed, env_id[row_env[dr]], row_t[dr])
            logu[dr] = np.log(u)
            flags[dr] = (logu[dr] <= l).astype(np.uint8)
        else:
            lam_row = np.broadcast_to(np.asarray(lam, dtype=np.float64), (B,))[row_env[dr]]
            p = np.minimum(1.0, np.exp(l))
            logu[dr] = np.log(lam_row)
            flags[dr] = (p >= lam_row).astype(np.uint8)

    x_out = y_last.copy()
    t_next = np.full(B, -1, dtype=np.int64)
    n_accept = np.zeros(B, dtype=np.int64)
    n_adv = np.zeros(B, dtype=np.int64)
    for b in range(B):
        r0, r1 = int(row_ptr[b]), int(row_ptr[b + 1])
        if r1 == r0:                                 # finished environment: untouched
            continue
        t0 = int(row_t[r0])
        base_row = bonus or t0 == 0                  # the last row is a step of the base model itself
        K_eff = r1 - r0 - 1 if base_row else r1 - r0
        j = first_rejection(flags[r0:r0 + K_eff])
        n_accept[b] = j - 1
        if j <= K_eff:
            r = r0 + j - 1
            x_out[b] = reflect(mu_p[r], mu_q[r], sig[r], xi[r])
            n_adv[b] = j
        elif base_row:                               # exact base transition from y_{K_eff} (no noise at t = 0)
            r = r1 - 1
            x_out[b] = mu_q[r] + sig[r] * xi[r]
            n_adv[b] = K_eff + 1
        else:
            n_adv[b] = K_eff                         # x_out = y_{K_eff}
        t_next[b] = t0 - n_adv[b]
    return dict(x_out=x_out, t_next=t_next, n_accept=n_accept, n_adv=n_adv,
                flags=flags, logratio=logratio, logu=logu)


def spec_round(base, drafter, sched, x, t0, K, sigma_scale, env_id, seed, cond, clip=None, lam=None, bonus=False):
    """draft -> verify -> accept for a batch of environments; returns the accept dict plus the draft dict."""
    dr = draft(drafter, sched, x, t0, K, sigma_scale, env_id, seed, cond, clip, bonus)
    eps_q = verify(base, dr["row_env"], dr["row_t"], dr["states"], cond)
    ac = accept(sched, dr["row_ptr"], dr["row_t"], sigma_scale, env_id, seed,
                dr["states"], dr["eps_p"], eps_q, dr["xi"], dr["y_last"], clip, lam, bonus)
    ac["draft"] = dr
    ac["eps_q"] = eps_q
    return ac


def stage_select(t, t_hi, t_lo, table):
    """Per-environment entry of a [B, 3] stage table: column 0 while t >= t_hi, 1 while t_lo <= t < t_hi, else 2."""
    t = np.asarray(t, dtype=np.int64)
    table = np.asarray(table)
    stage = np.where(t >= t_hi, 0, np.where(t >= t_lo, 1, 2))
    return table[np.arange(len(t)), stage]


def chain(base, drafter, sched, x, t0, K, sigma_scale, env_id, seed, cond, clip=None, lam=None, bonus=False,
          stages=None, max_rounds=10 ** 6):
    """Rounds repeated until every environment has finished (the paper's inference loop).

    stages = (t_hi, t_lo) makes K, sigma_scale (and lam, if given) [B, 3] stage tables read at the
    start of every round.  Returns the final latents and timesteps, per-environment totals (accepted
    drafts, drafted transitions, rounds run), the number of rounds and every round's result.
    """
    x = np.asarray(x, dtype=np.float64).copy()
    t = np.asarray(t0, dtype=np.int64).copy()
    B = len(t)
    tot = {k: np.zeros(B, dtype=np.int64) for k in ("accept", "drafts", "rounds")}
    history = []
    while (t >= 0).any() and len(history) < max_rounds:
        if stages is None:
            K_r, s_r, lam_r = K, sigma_scale, lam
        else:
            K_r = stage_select(t, stages[0], stages[1], K)
            s_r = stage_select(t, stages[0], stages[1], sigma_scale)
            lam_r = None if lam is None else stage_select(t, stages[0], stages[1], lam)
        r = spec_round(base, drafter, sched, x, t, K_r, s_r, env_id, seed, cond, clip, lam_r, bonus)
        tot["accept"] += r["n_accept"]
        tot["drafts"] += r["draft"]["K_eff"]
        tot["rounds"] += t >= 0
        x, t = r["x_out"], r["t_next"]
        history.append(r)
    return dict(x=x, t=t, totals=tot, rounds=len(history), history=history)


def base_chain_step(base, sched, x, t, sigma_scale, env_id, seed, cond, clip=None):
    """One plain DDPM reverse step of the base model with the same noise stream
    (the process the round must reproduce in law; used by the invariants' tests)."""
    x = np.asarray(x, dtype=np.float64)
    t = np.asarray(t, dtype=np.int64)
    B = x.shape[0]
    env_id = np.arange(B) if env_id is None else np.asarray(env_id, dtype=np.int64)
    mu = sched.posterior_mean(x, base(x, t, cond), t, clip)
    z = philox.normal(seed, env_id, t, int(np.prod(x.shape[1:]))).reshape(x.shape)
    sig = (np.asarray(sigma_scale, dtype=np.float64) * sched.sigma[t]).reshape((-1,) + (1,) * (x.ndim - 1))
    return mu + sig * z


def distill_loss(sched, row_t, states, eps_p, eps_q, lam1, lam2, clip=None):
    """Forward value of the drafter's distillation objective (Section 3.2, Draft Model Training):
    L_pred = E ||m_hat - m||^2 on the network outputs, L_norm = E ||(mu_hat - mu)/sigma_t||^2 on the DDPM means,
    L = lam1 L_pred + lam2 L_norm, the expectations taken as means over the given rows.  Rows at t = 0 have
    sigma_0 = 0 and are left out of L_norm (reading: the normalised term is defined for noisy steps only)."""
    row_t = np.asarray(row_t, dtype=np.int64)
    eps_p = np.asarray(eps_p, dtype=np.float64); eps_q = np.asarray(eps_q, dtype=np.float64)
    R = len(row_t)
    if R == 0:
        return 0.0, 0.0, 0.0
    diff = (eps_p - eps_q).reshape(R, -1)
    l_pred = float(np.mean(np.sum(diff * diff, axis=1)))
    mu_p = sched.posterior_mean(states, eps_p, row_t, clip).reshape(R, -1)
    mu_q = sched.posterior_mean(states, eps_q, row_t, clip).reshape(R, -1)
    noisy = row_t > 0
    if noisy.any():
        d = (mu_p[noisy] - mu_q[noisy]) / sched.sigma[row_t[noisy]][:, None]
        l_norm = float(np.mean(np.sum(d * d, axis=1)))
    else:
        l_norm = 0.0
    return l_pred, l_norm, lam1 * l_pred + lam2 * l_norm
