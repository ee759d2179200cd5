"""GPU parity over seeded random combinations of the configuration switches (sampler, bonus row, x0 clamp,
normalisation, accept rule, conditioning mode, precision, kernel path) on small networks (needs an MI355X)."""
import numpy as np
import pytest

import tsdp_inputs as ti
from oracle import spec_round as sr
from tests.helpers import assert_latents_close, drafted_rows, gpu_side, list_near_ties, oracle_side, scaled_err, to_dev

pytestmark = pytest.mark.gpu

# (dtype, cond_mode, base, drafter, H, A): fused bf16 / fp32 kernels and the general operator kernels
SHAPES = [
    ("bf16", 0, ti.NetShape(2, 256, 4), ti.NetShape(1, 128, 4), 16, 10),
    ("bf16", 0, ti.NetShape(1, 384, 6), ti.NetShape(1, 192, 6), 16, 7),
    ("bf16", 1, ti.NetShape(1, 512, 8), ti.NetShape(1, 256, 8), 32, 14),
    ("fp32", 0, ti.NetShape(2, 64, 2), ti.NetShape(1, 32, 2), 16, 2),
    ("fp32", 0, ti.NetShape(1, 256, 4), ti.NetShape(1, 128, 4), 16, 10),
    ("fp32", 0, ti.NetShape(1, 96, 3), ti.NetShape(1, 48, 3), 16, 4),       # no fused kernel: operator path
    ("fp32", 1, ti.NetShape(1, 96, 3), ti.NetShape(1, 48, 3), 8, 3),
]


@pytest.mark.parametrize("case", range(28))
def test_random_combination(case):
    import torch
    rng = np.random.default_rng(1000 + case)
    dtype, cm, base, draft, H, A = SHAPES[case % len(SHAPES)]
    B = int(rng.integers(2, 7))
    T = int(rng.choice([10, 50, 100]))
    K_max = int(rng.choice([4, 8, 16]))
    kw = dict(cond_dim=64 if cm == 0 else 768, cond_tokens=0 if cm == 0 else 64) if dtype == "bf16" else \
        dict(cond_dim=32 if cm == 0 else 24, cond_tokens=0 if cm == 0 else 5)
    wl = ti.small_variant(ti.C1, dtype=dtype, B=B, H=H, A=A, cond_mode=cm, base=base, draft=draft, T=T, K_max=K_max,
                          schedule=int(rng.integers(0, 2)), **kw)
    sampler = int(rng.integers(0, 2)); eta = float(rng.choice([0.5, 0.8, 1.0]))
    bonus = bool(rng.integers(0, 2)); norm = int(rng.integers(0, 2))
    clip = None if rng.integers(0, 2) else float(rng.choice([1.0, 3.0]))
    use_lambda = bool(rng.integers(0, 3) == 0)
    wb = ti.make_weights(wl, "base", b_std=0.02, head_scale=0.5)
    wd = ti.make_weights(wl, "draft", b_std=0.02, head_scale=0.5)
    cond = ti.make_cond(wl, B); x = ti.make_latents(wl, B)
    t0 = rng.integers(-1, T, B); t0[0] = T - 1
    K = rng.integers(0 if bonus else 1, K_max + 1, B); s = rng.uniform(1.0, 1.5, B).astype(np.float32)
    env = rng.integers(0, 10 ** 6, B)
    lam = rng.uniform(0.05, 1.0, B).astype(np.float32) if use_lambda else None
    base_o, draft_o, sched = oracle_side(wl, wb, wd, sampler=sampler, eta=eta, norm=norm)
    ctx = gpu_side(wl, wb, wd, cond, clip=clip, B_max=B, sampler=sampler, eta=eta, bonus_row=bonus, norm=norm)
    tol = 2e-2 if dtype == "bf16" else 1e-5
    rows = ctx.alloc_rows(B)
    sd, ed = to_dev(s), to_dev(env.astype(np.int32))
    ctx.tsdp_draft(to_dev(x), to_dev(t0.astype(np.int32)), to_dev(K.astype(np.int32)), sd, ed, rows)
    o = sr.draft(draft_o, sched, x, t0, K, s, env, wl.philox_seed, cond, clip, bonus)
    R = int(o["row_ptr"][-1])
    np.testing.assert_array_equal(rows["row_ptr"].cpu().numpy(), o["row_ptr"])
    np.testing.assert_array_equal(rows["row_t"].cpu().numpy()[:R], o["row_t"])
    assert scaled_err(rows["eps_p"].cpu().numpy()[:R], o["eps_p"]) < tol, (case, "eps_p")
    assert_latents_close(rows["states"].cpu().numpy()[:R], o["states"], dtype, f"case {case}: drafted states")
    ctx.tsdp_verify(B, rows)
    st = rows["states"].cpu().numpy()[:R]
    ref_q = sr.verify(base_o, o["row_env"], o["row_t"], st, cond)
    assert scaled_err(rows["eps_q"].cpu().numpy()[:R], ref_q) < tol, (case, "eps_q")
    if lam is None:
        out = ctx.tsdp_accept(B, sd, ed, rows)
    else:
        out = ctx.tsdp_accept_threshold(B, sd, to_dev(lam), rows)
    g = {k: v.cpu().numpy() for k, v in out.items()}
    ref = sr.accept(sched, o["row_ptr"], o["row_t"], s, env, wl.philox_seed, st, rows["eps_p"].cpu().numpy()[:R],
                    rows["eps_q"].cpu().numpy()[:R], rows["xi"].cpu().numpy()[:R], rows["y_last"].cpu().numpy(), clip,
                    lam=lam, bonus=bonus)
    near = list_near_ties(f"case {case}", ref["logu"], ref["logratio"], o["row_ptr"], 1e-5,
                          drafted_rows(o["row_ptr"], o["row_t"], bonus))
    diff = g["flags"][:R] != ref["flags"]
    assert not np.any(diff & ~near), case
    ok = np.array([not np.any(diff[o["row_ptr"][b]:o["row_ptr"][b + 1]]) for b in range(B)])
    for k in ("n_accept", "n_adv", "t_next"):
        np.testing.assert_array_equal(g[k][ok], ref[k][ok])
    assert ok.any() or B == 0
    assert_latents_close(g["x_out"][ok], ref["x_out"][ok], "fp32", f"case {case}: x_out on identical tensors")
    ctx.close()
