"""DDPM schedule tables and the epsilon-prediction posterior (oracle, fp64).

The paper names only "the DDPM scheduler", its "data-aligned means" and its
"standard deviation sigma_t" (Section 3.2, Draft Generation / Verification);
the formulas are the textbook ones of the epsilon-prediction DDPM with the
fixed-small posterior variance, and the squared-cosine schedule of the
improved-DDPM paper.  Timesteps run t = T-1 .. 0; the step at t maps x_t to
x_{t-1}; no noise is added by the step at t = 0.
"""
import numpy as np


class Schedule:
    """beta, abar and the posterior coefficients, as fp64 arrays of length T.

    The tables are rounded to fp32 once (table storage format of the method's
    implementation) and then used in fp64 arithmetic.
    """

    def __init__(self, T, schedule, beta0=1e-4, beta1=0.02, round_fp32=True, sampler=0, eta=1.0):
        """sampler 0: DDPM posterior (above).  sampler 1: DDIM(eta), eta in (0, 1] (Section 3.2, Draft Model Training, names
        both schedulers without formulas; textbook DDIM): sigma_t = eta sqrt((1-abar_{t-1})/(1-abar_t)) sqrt(1-abar_t/abar_{t-1}),
        mean = sqrt(abar_{t-1}) x0_hat + sqrt(1-abar_{t-1}-sigma_t^2) eps.  Both are written as
        mu = c0 x0_hat + cx x + ce eps  (DDPM: ce = 0; DDIM: cx = 0)."""
        i = np.arange(T, dtype=np.float64)
        if schedule == 0:                       # linear
            beta = np.linspace(beta0, beta1, T, dtype=np.float64)
        elif schedule == 1:                     # squared cosine, offset 0.008, cap 0.999
            f = lambda j: np.cos(((j / T) + 0.008) / 1.008 * np.pi / 2.0) ** 2
            beta = np.minimum(1.0 - f(i + 1.0) / f(i), 0.999)
        else:
            raise ValueError("unknown schedule")
        alpha = 1.0 - beta
        abar = np.cumprod(alpha)
        abar_prev = np.concatenate([[1.0], abar[:-1]])
        self.T = T
        self.beta = beta
        self.abar = abar
        if sampler == 0:
            tables = dict(
                sqrt_abar=np.sqrt(abar),                                   # x_t = sqrt_abar x0 + sqrt_1m eps
                sqrt_1m=np.sqrt(1.0 - abar),
                c0=np.sqrt(abar_prev) * beta / (1.0 - abar),               # posterior mean coefficient of x0_hat
                cx=np.sqrt(alpha) * (1.0 - abar_prev) / (1.0 - abar),      # posterior mean coefficient of x_t
                ce=np.zeros(T),                                            # coefficient of the predicted noise
                sigma=np.sqrt(beta * (1.0 - abar_prev) / (1.0 - abar)),    # posterior std, 0 at t = 0
            )
        elif sampler == 1:
            if not (0.0 < eta <= 1.0):
                raise ValueError("DDIM eta must be in (0, 1]: eta = 0 has no Gaussian transition to test against")
            sig = eta * np.sqrt((1.0 - abar_prev) / (1.0 - abar)) * np.sqrt(1.0 - abar / abar_prev)
            tables = dict(
                sqrt_abar=np.sqrt(abar), sqrt_1m=np.sqrt(1.0 - abar),
                c0=np.sqrt(abar_prev), cx=np.zeros(T),
                ce=np.sqrt(np.maximum(1.0 - abar_prev - sig ** 2, 0.0)),
                sigma=sig,
            )
        else:
            raise ValueError("unknown sampler")
        for k, v in tables.items():
            if round_fp32:
                v = v.astype(np.float32).astype(np.float64)
            setattr(self, k, v)

    def posterior_mean(self, x, eps, t, clip=None):
        """mu_t(x, eps): x0_hat = (x - sqrt(1-abar) eps)/sqrt(abar) [clamped], mu = c0 x0_hat + cx x + ce eps.

        x, eps: [R, ...]; t: [R] int.  Returns fp64.
        """
        x = np.asarray(x, dtype=np.float64)
        eps = np.asarray(eps, dtype=np.float64)
        t = np.asarray(t)
        sh = (-1,) + (1,) * (x.ndim - 1)
        x0 = (x - self.sqrt_1m[t].reshape(sh) * eps) / self.sqrt_abar[t].reshape(sh)
        if clip is not None:
            x0 = np.clip(x0, -clip, clip)
        return self.c0[t].reshape(sh) * x0 + self.cx[t].reshape(sh) * x + self.ce[t].reshape(sh) * eps
