"""GPU parity at the full BASELINE sizes, in the launch configuration bench.py times: the whole batch runs
on the GPU, the CPU oracle recomputes a sample of environments / rows one by one (needs an MI355X)."""
import numpy as np
import pytest

import bench
import tsdp_inputs as ti
from oracle import spec_round as sr
from tests.helpers import assert_latents_close, drafted_rows, gpu_side, list_near_ties, oracle_side, scaled_err, to_dev

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-5, "bf16": 2e-2}            # noise predictions: error relative to the tensor scale; latents: elementwise
TIE = 1e-5                                     # accept decisions may differ only inside this near-tie window
SAMPLES = {"C2": [0], "C3": [0, 7, 31, 63], "C4": [0, 129, 255], "C5": [0, 3, 500, 777, 1023]}


def _full(name, point="calibrated"):
    wl = ti.WORKLOADS[name]
    wb, wd, cond, x, t0, K, s = bench.make_problem(wl, point)
    base, drafter, sched = oracle_side(wl, wb, wd)
    ctx = gpu_side(wl, wb, wd, cond)
    return wl, dict(cond=cond, x=x, t0=t0, K=K, s=s, base=base, drafter=drafter, sched=sched, ctx=ctx)


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5"])
def test_full_size_stages_on_sampled_environments(name):
    wl, S = _full(name)
    ctx, B = S["ctx"], wl.B
    if wl.dtype == "bf16":
        assert ctx.path_name(0) == "bf16-mfma-fused" and ctx.path_name(1) == "bf16-mfma-fused"
    rows = ctx.alloc_rows(B)
    sd = to_dev(S["s"])
    ctx.tsdp_draft(to_dev(S["x"]), to_dev(S["t0"]), to_dev(S["K"]), sd, None, rows)
    ctx.tsdp_verify(B, rows)
    out = ctx.tsdp_accept(B, sd, None, rows)
    g = {k: v.cpu().numpy() for k, v in {**rows, **out}.items()}
    K_eff, row_ptr, row_env, row_t = sr.plan_rows(S["t0"], S["K"])
    R = int(row_ptr[-1])
    np.testing.assert_array_equal(g["row_ptr"], row_ptr)               # the row table is exact at any size
    np.testing.assert_array_equal(g["row_t"][:R], row_t)
    np.testing.assert_array_equal(g["row_env"][:R], row_env)
    tol = TOL[wl.dtype]
    envs = np.array(SAMPLES[name])
    # drafter rollout of the sampled environments (environments are independent, noise is keyed by env id)
    o = sr.draft(S["drafter"], S["sched"], S["x"][envs], S["t0"][envs], S["K"][envs], S["s"][envs], envs,
                 wl.philox_seed, S["cond"][envs])
    for j, b in enumerate(envs):
        gs = slice(row_ptr[b], row_ptr[b + 1]); os_ = slice(o["row_ptr"][j], o["row_ptr"][j + 1])
        np.testing.assert_allclose(g["xi"][gs], o["xi"][os_], rtol=1e-5, atol=2e-6)
        e = scaled_err(g["eps_p"][gs], o["eps_p"][os_])
        assert e < tol, ("eps_p", int(b), e)
        assert_latents_close(g["states"][gs], o["states"][os_], wl.dtype, f"drafted states of env {int(b)}")
        assert_latents_close(g["y_last"][b], o["y_last"][j], wl.dtype, f"y_last of env {int(b)}")
        # verification of the GPU's own states of that environment
        ref = sr.verify(S["base"], np.full(gs.stop - gs.start, b), g["row_t"][gs], g["states"][gs], S["cond"])
        e = scaled_err(g["eps_q"][gs], ref)
        print(f"[{name}] env {int(b)}: verify scaled err {e:.3e}")
        assert e < tol, ("eps_q", int(b), e)
    # acceptance on the GPU's own tensors, every environment (the oracle's accept is cheap): indices bit-exact
    ref = sr.accept(S["sched"], row_ptr, row_t, S["s"], None, wl.philox_seed, g["states"][:R], g["eps_p"][:R],
                    g["eps_q"][:R], g["xi"][:R], g["y_last"])
    near = list_near_ties(name, ref["logu"], ref["logratio"], row_ptr, 1e-9, drafted_rows(row_ptr, row_t))
    assert not np.any((g["flags"][:R] != ref["flags"]) & ~near)
    ok = np.array([not np.any(near[row_ptr[b]:row_ptr[b + 1]]) for b in range(B)])
    assert ok.sum() >= B - 2
    for k in ("n_accept", "n_adv", "t_next"):
        np.testing.assert_array_equal(g[k][ok], ref[k][ok])
    assert_latents_close(g["x_out"][ok], ref["x_out"][ok], "fp32", "x_out of tsdp_accept on identical tensors")
    ctx.close()


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_full_size_bf16_round_against_oracle_round(name):
    """End-to-end bf16 round: accept decisions may differ from the fp64 oracle only on rows whose margin
    |log U - log alpha| is inside the error the bf16 networks put on log alpha; environments whose first
    rejection agrees end within the bf16 tolerance."""
    import torch
    wl, S = _full(name)
    ctx, B = S["ctx"], wl.B
    rows = ctx.alloc_rows(B)
    sd = to_dev(S["s"])
    ctx.tsdp_draft(to_dev(S["x"]), to_dev(S["t0"]), to_dev(S["K"]), sd, None, rows)
    ctx.tsdp_verify(B, rows)
    out = ctx.tsdp_accept(B, sd, None, rows)
    x = to_dev(S["x"]); t = to_dev(S["t0"])
    nacc = torch.zeros(B, dtype=torch.int32, device="cuda"); nadv = torch.zeros_like(nacc)
    ctx.tsdp_round(x, t, to_dev(S["K"]), sd, None, nacc, nadv)
    # the fused round is the three stages on context-owned buffers: identical results
    np.testing.assert_array_equal(nacc.cpu().numpy(), out["n_accept"].cpu().numpy())
    np.testing.assert_array_equal(t.cpu().numpy(), out["t_next"].cpu().numpy())
    np.testing.assert_array_equal(x.cpu().numpy(), out["x_out"].cpu().numpy())
    envs = np.array(SAMPLES[name])
    ref = sr.spec_round(S["base"], S["drafter"], S["sched"], S["x"][envs], S["t0"][envs], S["K"][envs], S["s"][envs],
                        envs, wl.philox_seed, S["cond"][envs])
    row_ptr = rows["row_ptr"].cpu().numpy()
    gl, gf = out["logratio"].cpu().numpy(), out["flags"].cpu().numpy()
    agree = 0
    for j, b in enumerate(envs):
        gs = slice(row_ptr[b], row_ptr[b + 1]); os_ = slice(ref["draft"]["row_ptr"][j], ref["draft"]["row_ptr"][j + 1])
        # rows up to the oracle's first rejection saw (nearly) the same states on both sides
        n = min(int(ref["n_accept"][j]) + 1, os_.stop - os_.start)
        dl = np.abs(gl[gs][:n] - ref["logratio"][os_][:n])
        margin = np.abs(ref["logu"][os_][:n] - ref["logratio"][os_][:n])
        mism = gf[gs][:n] != ref["flags"][os_][:n]
        for k in np.nonzero(mism)[0]:
            print(f"[{name}] env {int(b)} draft {int(k) + 1}: decision differs, margin {margin[k]:.3e}, "
                  f"bf16 error on log alpha {dl[k]:.3e}")
        assert np.all(margin[mism] <= dl[mism] + TIE), (int(b), margin[mism], dl[mism])
        assert dl.max() < 0.5, (int(b), dl.max())                     # bf16 error on log alpha stays a fraction of a nat
        if not mism.any():
            agree += 1
            assert int(nacc[b]) == ref["n_accept"][j] and int(t[b]) == ref["t_next"][j]
            w = assert_latents_close(x[b].cpu().numpy(), ref["x_out"][j], "bf16", f"final action of env {int(b)}")
            print(f"[{name}] env {int(b)}: final action at {w:.3f} of the elementwise bound, max log-alpha error {dl.max():.3e}")
    print(f"[{name}] sampled envs with identical accept decisions: {agree}/{len(envs)}")
    assert agree >= len(envs) - 2
    ctx.close()


def test_identity_drafter_accepts_every_draft_on_the_gpu():
    # drafter == base => mu_p == mu_q => all K_eff drafts pass and the round equals K_eff base DDPM steps
    import torch
    wl = ti.small_variant(ti.C3, B=8, draft=ti.C3.base)
    wb = ti.make_weights(wl, "base", b_std=0.02)
    cond, x = ti.make_cond(wl, 8), ti.make_latents(wl, 8)
    ctx = gpu_side(wl, wb, wb, cond)
    t0 = np.array([99, 50, 20, 16, 15, 3, 0, -1], np.int32); K = np.full(8, 16, np.int32); s = np.ones(8, np.float32)
    xd, td = to_dev(x), to_dev(t0)
    nacc = torch.zeros(8, dtype=torch.int32, device="cuda"); nadv = torch.zeros_like(nacc)
    ctx.tsdp_round(xd, td, to_dev(K), to_dev(s), None, nacc, nadv)
    keff = np.minimum(K, np.maximum(t0, 0))
    np.testing.assert_array_equal(nacc.cpu().numpy(), keff)
    np.testing.assert_array_equal(nadv.cpu().numpy(), [16, 16, 16, 16, 15, 3, 1, 0])
    np.testing.assert_array_equal(td.cpu().numpy(), [83, 34, 4, 0, 0, 0, -1, -1])
    ctx.close()


def test_round_is_deterministic_and_handles_empty_and_finished_batches():
    import torch
    wl = ti.small_variant(ti.C5, B=37)
    wb, wd = ti.make_weights(wl, "base"), ti.make_weights(wl, "draft")
    cond, x = ti.make_cond(wl, 37), ti.make_latents(wl, 37)
    t0, K, s = ti.make_schedule_inputs(wl, 37)
    ctx = gpu_side(wl, wb, wd, cond)
    res = []
    for _ in range(2):
        xd, td = to_dev(x), to_dev(t0)
        nacc = torch.zeros(37, dtype=torch.int32, device="cuda"); nadv = torch.zeros_like(nacc)
        ctx.tsdp_round(xd, td, to_dev(K), to_dev(s), None, nacc, nadv)
        res.append((xd.cpu().numpy().tobytes(), td.cpu().numpy().tobytes(), nacc.cpu().numpy().tobytes()))
    assert res[0] == res[1]
    # all environments finished: nothing runs, latents and counters pass through
    xd, td = to_dev(x), to_dev(np.full(37, -1, np.int32))
    nacc = torch.full((37,), 7, dtype=torch.int32, device="cuda"); nadv = torch.full((37,), 7, dtype=torch.int32, device="cuda")
    ctx.tsdp_round(xd, td, to_dev(K), to_dev(s), None, nacc, nadv)
    np.testing.assert_array_equal(xd.cpu().numpy(), x)
    assert int(nacc.sum()) == 0 and int(nadv.sum()) == 0 and (td.cpu().numpy() == -1).all()
    # B = 0 is accepted and does nothing
    e = torch.zeros(0, wl.H, wl.A, device="cuda"); ei = torch.zeros(0, dtype=torch.int32, device="cuda")
    ctx.tsdp_round(e, ei, ei, torch.zeros(0, device="cuda"), None, None, None)
    ctx.close()


def test_full_size_bonus_row_with_ddim_sampler():
    # the K+1 candidate set and the DDIM(eta) transition together, at the full C3 size (64 envs x (16 + 1) rows)
    wl = ti.WORKLOADS["C3"]
    wb, wd, cond, x, t0, K, s = bench.make_problem(wl, "calibrated")
    t0 = t0.copy(); t0[:4] = [0, 3, 16, 99]                            # base step only, t0 < K, t0 = K, chain start
    base, drafter, sched = oracle_side(wl, wb, wd, sampler=1, eta=0.8)
    ctx = gpu_side(wl, wb, wd, cond, sampler=1, eta=0.8, bonus_row=True)
    B = wl.B
    rows = ctx.alloc_rows(B)
    sd = to_dev(s)
    ctx.tsdp_draft(to_dev(x), to_dev(t0), to_dev(K), sd, None, rows)
    ctx.tsdp_verify(B, rows)
    out = ctx.tsdp_accept(B, sd, None, rows)
    g = {k: v.cpu().numpy() for k, v in {**rows, **out}.items()}
    K_eff, row_ptr, row_env, row_t = sr.plan_rows(t0, K, bonus=True)
    R = int(row_ptr[-1])
    assert R == int((K_eff + 1).sum())
    np.testing.assert_array_equal(g["row_ptr"], row_ptr)
    np.testing.assert_array_equal(g["row_t"][:R], row_t)
    np.testing.assert_array_equal(g["row_env"][:R], row_env)
    envs = np.array([0, 1, 2, 3, 40])
    o = sr.draft(drafter, sched, x[envs], t0[envs], K[envs], s[envs], envs, wl.philox_seed, cond[envs], bonus=True)
    for j, b in enumerate(envs):
        gs = slice(row_ptr[b], row_ptr[b + 1]); os_ = slice(o["row_ptr"][j], o["row_ptr"][j + 1])
        np.testing.assert_allclose(g["xi"][gs], o["xi"][os_], rtol=1e-5, atol=2e-6)
        assert scaled_err(g["eps_p"][gs], o["eps_p"][os_]) < TOL["bf16"], ("eps_p", int(b))
        assert_latents_close(g["states"][gs], o["states"][os_], "bf16", f"drafted states of env {int(b)}")
        ref = sr.verify(base, np.full(gs.stop - gs.start, b), g["row_t"][gs], g["states"][gs], cond)
        assert scaled_err(g["eps_q"][gs], ref) < TOL["bf16"], ("eps_q", int(b))
    ref = sr.accept(sched, row_ptr, row_t, s, None, wl.philox_seed, g["states"][:R], g["eps_p"][:R], g["eps_q"][:R],
                    g["xi"][:R], g["y_last"], bonus=True)
    near = list_near_ties("C3 bonus/DDIM", ref["logu"], ref["logratio"], row_ptr, TIE, drafted_rows(row_ptr, row_t, True))
    diff = g["flags"][:R] != ref["flags"]
    assert not np.any(diff & ~near)
    ok = np.array([not np.any(diff[row_ptr[b]:row_ptr[b + 1]]) for b in range(B)])
    assert ok.sum() >= B - 2
    for k in ("n_accept", "n_adv", "t_next"):
        np.testing.assert_array_equal(g[k][ok], ref[k][ok])
    assert_latents_close(g["x_out"][ok], ref["x_out"][ok], "fp32", "x_out of tsdp_accept on identical tensors")
    # every running environment ends its round with a corrected or an exact base step
    live = t0 >= 0
    assert (ref["n_adv"][live] == ref["n_accept"][live] + 1).all() and ref["n_adv"][0] == 1
    assert (ref["n_accept"] == K_eff).any()                            # some environment took its bonus step
    ctx.close()


@pytest.mark.parametrize("variant", ["plain", "bonus_row_ddim_enqueue"])
def test_speculative_chain_on_the_gpu_has_the_law_of_the_base_chain(variant):
    # Losslessness end to end on the device (second variant: the K+1 candidate set with the DDIM(0.7) transition, driven
    # by the enqueue-only chain): final actions of whole chains driven by an imperfect drafter against
    # final actions of the plain base chain (drafter = base, every draft accepted, which the identity test above
    # ties to plain DDPM steps).  Same conditioning for all environments, independent noise seeds and initial
    # latents for the two runs; per-dimension two-sample Kolmogorov-Smirnov tests with a Bonferroni bound.
    from scipy import stats
    n = 4096
    wl = ti.small_variant(ti.C1, B=n)
    wb = ti.make_weights(wl, "base", b_std=0.02, head_scale=1.5)
    wd = ti.make_weights(wl, "draft", b_std=0.02, head_scale=1.5)
    cond = np.repeat(ti.make_cond(wl, 1), n, axis=0)
    K = to_dev(np.full(n, 4, np.int32)); s = to_dev(np.ones(n, np.float32))
    finals = []
    rates = []
    import torch
    extra = dict(sampler=1, eta=0.7, bonus_row=True) if variant != "plain" else {}
    for run, (wl_run, w_draft, seed) in enumerate(((wl, wd, 11), (ti.small_variant(wl, draft=wl.base), wb, 12))):
        ctx = gpu_side(wl_run, wb, w_draft, cond, B_max=n, seed=seed, **extra)
        x = to_dev(np.random.default_rng(100 + run).standard_normal((n, wl.H, wl.A)).astype(np.float32))
        t = to_dev(np.full(n, wl.T - 1, np.int32))
        if variant == "plain":
            rounds, tot = ctx.tsdp_chain(x, t, K, s, None, check_every=2)
        else:
            tot = {k: torch.zeros(n, dtype=torch.int32, device="cuda") for k in ("accept", "drafts", "rounds")}
            ctx.tsdp_chain_enqueue(x, t, K, s, None, None, wl.T, totals=tot)
        assert (t.cpu().numpy() == -1).all()
        finals.append(x.cpu().numpy().reshape(n, -1))
        rates.append(tot["accept"].sum().item() / tot["drafts"].sum().item())
        ctx.close()
    assert 0.2 < rates[0] < 0.98 and rates[1] == 1.0                   # rejections happen in the speculative run
    # power of the detector: the drafter's own chain (threshold rule with a vanishing threshold accepts every
    # draft) has a visibly different law
    ctx = gpu_side(wl, wb, wd, cond, B_max=n, seed=13, **extra)
    x = to_dev(np.random.default_rng(102).standard_normal((n, wl.H, wl.A)).astype(np.float32))
    t = to_dev(np.full(n, wl.T - 1, np.int32))
    ctx.tsdp_chain(x, t, K, s, None, lam=to_dev(np.full(n, 1e-30, np.float32)), check_every=2)
    c = x.cpu().numpy().reshape(n, -1)
    ctx.close()
    assert min(stats.ks_2samp(c[:, j], finals[1][:, j]).pvalue for j in range(c.shape[1])) < 1e-6
    a, b = finals
    D = a.shape[1]
    pvals = np.array([stats.ks_2samp(a[:, j], b[:, j]).pvalue for j in range(D)])
    assert pvals.min() > 1e-3 / D, pvals.min()
    sd = np.sqrt((a.var(0) + b.var(0)) / n)
    assert (np.abs(a.mean(0) - b.mean(0)) < 5 * sd).all()
    assert (np.abs(a.var(0) / b.var(0) - 1) < 6 * np.sqrt(2 / n)).all()


def _sentinel_rows(ctx, B):
    """Caller buffers filled with a NaN bit pattern no kernel produces."""
    import torch
    rows = ctx.alloc_rows(B)
    for k in ("states", "eps_p", "eps_q", "xi"):
        rows[k].view(torch.int32).fill_(0x7FC0BEEF)
    for k in ("row_t", "row_env"):
        rows[k].fill_(-777)
    return rows


def _check_tail_untouched(rows, R):
    import torch
    for k in ("states", "eps_p", "eps_q", "xi"):
        bits = rows[k].view(torch.int32).reshape(rows[k].shape[0], -1)
        assert bool((bits[R:] == 0x7FC0BEEF).all()), f"{k}: a row at or beyond row_ptr[B] was written"
        assert bool(torch.isfinite(rows[k][:R]).all()), f"{k}: a live row was left unwritten"
    for k in ("row_t", "row_env"):
        assert bool((rows[k][R:] == -777).all()), f"{k}: an entry at or beyond row_ptr[B] was written"
        assert bool((rows[k][:R] >= 0).all())


def test_rows_beyond_the_live_count_are_never_written():
    # ragged batch at the full C5 size (fused bf16 kernels, K ~ U{2..16}: about 9200 live rows of 16384), then the
    # fused fp32 kernels and the general operator kernels on small batches: NaN sentinels behind row_ptr[B] survive
    # tsdp_draft and tsdp_verify, every live row is written
    wl, S = _full("C5")
    ctx, B = S["ctx"], wl.B
    rows = _sentinel_rows(ctx, B)
    ctx.tsdp_draft(to_dev(S["x"]), to_dev(S["t0"]), to_dev(S["K"]), to_dev(S["s"]), None, rows)
    ctx.tsdp_verify(B, rows)
    R = int(rows["row_ptr"][-1].item())
    assert 0 < R < rows["row_t"].shape[0] - 1000
    _check_tail_untouched(rows, R)
    ctx.close()
    for wl in (ti.small_variant(ti.C2, B=5, base=ti.NetShape(2, 256, 4)),
               ti.small_variant(ti.C1, B=5, base=ti.NetShape(2, 96, 3), draft=ti.NetShape(1, 48, 3)),
               ti.small_variant(ti.C4, B=5, base=ti.NetShape(1, 512, 8))):
        wb, wd = ti.make_weights(wl, "base", b_std=0.02), ti.make_weights(wl, "draft", b_std=0.02)
        for bonus in (False, True):
            ctx = gpu_side(wl, wb, wd, ti.make_cond(wl, 5), bonus_row=bonus)
            rows = _sentinel_rows(ctx, 5)
            t0 = np.array([wl.T - 1, 2, 0, -1, 1], np.int32); K = np.array([wl.K_max, wl.K_max, 3, 2, 1], np.int32)
            ctx.tsdp_draft(to_dev(ti.make_latents(wl, 5)), to_dev(t0), to_dev(K), to_dev(np.ones(5, np.float32)), None, rows)
            ctx.tsdp_verify(5, rows)
            R = int(rows["row_ptr"][-1].item())
            assert R == int(sr.plan_rows(t0, K, bonus)[1][-1]) and R < rows["row_t"].shape[0]
            _check_tail_untouched(rows, R)
            ctx.close()


def test_verify_range_checks_a_callers_row_table():
    # tsdp_verify indexes the timestep and conditioning tables with the caller's row table: entries out of range are
    # clamped (no read out of bounds) and reported in the status word
    import torch
    wl = ti.small_variant(ti.C3, B=4, base=ti.NetShape(1, 256, 4))
    wb, wd = ti.make_weights(wl, "base"), ti.make_weights(wl, "draft")
    ctx = gpu_side(wl, wb, wd, ti.make_cond(wl, 4))
    rows = ctx.alloc_rows(4)
    t0 = np.array([50, 40, 30, 20], np.int32); K = np.full(4, 2, np.int32)
    ctx.tsdp_draft(to_dev(ti.make_latents(wl, 4)), to_dev(t0), to_dev(K), to_dev(np.array([1.0, 0.0, 1.0, 1.0], np.float32)), None, rows)
    assert ctx.tsdp_status() == 4                                      # sigma_scale = 0 is reported
    ctx.tsdp_verify(4, rows)
    assert ctx.tsdp_status() == 0
    good = rows["eps_q"].clone()
    rows["row_env"][1] = 9; rows["row_t"][2] = 100; rows["row_env"][7] = -3
    ctx.tsdp_verify(4, rows)
    assert ctx.tsdp_status() == 2 + 8
    rows["row_env"][1] = 3; rows["row_t"][2] = 99; rows["row_env"][7] = 0   # what the clamp made of them
    want = rows["eps_q"].clone()
    ctx.tsdp_verify(4, rows)
    assert ctx.tsdp_status() == 0 and torch.equal(rows["eps_q"], want)
    assert torch.equal(want[[0, 3, 4, 5, 6]], good[[0, 3, 4, 5, 6]])
    ctx.close()
