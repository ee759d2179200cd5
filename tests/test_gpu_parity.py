"""GPU parity: every C entry point against the CPU oracle on the same seeded inputs (needs an MI355X)."""
import numpy as np
import pytest

import tsdp_inputs as ti
from oracle import philox, spec_round as sr
from tests.helpers import assert_latents_close, drafted_rows, gpu_side, list_near_ties, oracle_side, scaled_err, to_dev

pytestmark = pytest.mark.gpu

# Tolerances.  Latents (drafted states, final actions): elementwise, rtol 1e-5 for fp32 networks and 2e-2 for bf16
# networks (tests/helpers.py: assert_latents_close).  Intermediate noise predictions: max error relative to the
# tensor's scale below the same numbers (the GPU accumulates dot products of length <= 4d in fp32 through L residual
# layers, the oracle in fp64; bf16 matrix-multiply inputs carry 2^-9 relative rounding).
TOL = {"fp32": 1e-5, "bf16": 2e-2}
TIE = 1e-5          # accept decisions may differ only where |log U - log alpha| is below this


def _setup(wl, B, clip=None, K_max=None, b_std=0.02, head_scale=1.0, seed=None, sampler=0, eta=1.0, bonus=False, norm=0):
    wb = ti.make_weights(wl, "base", b_std=b_std, head_scale=head_scale)
    wd = ti.make_weights(wl, "draft", b_std=b_std, head_scale=head_scale)
    cond = ti.make_cond(wl, B)
    x = ti.make_latents(wl, B)
    base, drafter, sched = oracle_side(wl, wb, wd, sampler=sampler, eta=eta, norm=norm)
    ctx = gpu_side(wl, wb, wd, cond, clip=clip, B_max=B, K_max=K_max, seed=seed, sampler=sampler, eta=eta,
                   bonus_row=bonus, norm=norm)
    return dict(wl=wl, B=B, cond=cond, x=x, base=base, drafter=drafter, sched=sched, ctx=ctx, clip=clip, bonus=bonus,
                seed=wl.philox_seed if seed is None else seed)


def _gpu_draft(S, t0, K, s, env):
    ctx, B = S["ctx"], S["B"]
    rows = ctx.alloc_rows(B)
    ctx.tsdp_draft(to_dev(S["x"]), to_dev(t0.astype(np.int32)), to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32)),
                   None if env is None else to_dev(env.astype(np.int32)), rows)
    return rows


def _check_draft(S, rows, t0, K, s, env, tol):
    o = sr.draft(S["drafter"], S["sched"], S["x"], t0, K, s, env, S["seed"], S["cond"], S["clip"], S["bonus"])
    R = int(o["row_ptr"][-1])
    np.testing.assert_array_equal(rows["row_ptr"].cpu().numpy(), o["row_ptr"])
    np.testing.assert_array_equal(rows["row_t"].cpu().numpy()[:R], o["row_t"])
    np.testing.assert_array_equal(rows["row_env"].cpu().numpy()[:R], o["row_env"])
    xi = rows["xi"].cpu().numpy()[:R]
    np.testing.assert_allclose(xi, o["xi"], rtol=1e-5, atol=2e-6)      # fp32 Box-Muller vs fp64
    e = scaled_err(rows["eps_p"].cpu().numpy()[:R], o["eps_p"])
    print(f"[{S['wl'].name}] draft eps_p: scaled err {e:.3e}")
    assert e < tol, ("eps_p", e)
    w = assert_latents_close(rows["states"].cpu().numpy()[:R], o["states"], S["wl"].dtype, "drafted states")
    w2 = assert_latents_close(rows["y_last"].cpu().numpy(), o["y_last"], S["wl"].dtype, "y_last")
    print(f"[{S['wl'].name}] draft states / y_last: {w:.3f} / {w2:.3f} of the elementwise bound")
    return o


def _check_verify(S, rows, o, tol):
    ctx, B = S["ctx"], S["B"]
    ctx.tsdp_verify(B, rows)
    R = int(o["row_ptr"][-1])
    st = rows["states"].cpu().numpy()[:R]
    ref = sr.verify(S["base"], o["row_env"], o["row_t"], st, S["cond"])   # oracle on the GPU's own states
    got = rows["eps_q"].cpu().numpy()[:R]
    e = scaled_err(got, ref)
    print(f"[{S['wl'].name}] verify eps_q: scaled err {e:.3e}")
    assert e < tol, ("eps_q", e)
    return ref


def _check_accept(S, rows, o, s, env, window):
    """tsdp_accept against the oracle on the identical tensors: indices exact outside the near-tie
    window, latents to fp32 rounding."""
    ctx, B = S["ctx"], S["B"]
    out = ctx.tsdp_accept(B, to_dev(s.astype(np.float32)), None if env is None else to_dev(env.astype(np.int32)), rows)
    R = int(o["row_ptr"][-1])
    g = {k: v.cpu().numpy() for k, v in out.items()}
    ref = sr.accept(S["sched"], o["row_ptr"], o["row_t"], s.astype(np.float32), env, S["seed"],
                    rows["states"].cpu().numpy()[:R], rows["eps_p"].cpu().numpy()[:R], rows["eps_q"].cpu().numpy()[:R],
                    rows["xi"].cpu().numpy()[:R], rows["y_last"].cpu().numpy(), S["clip"], bonus=S["bonus"])
    np.testing.assert_allclose(g["logu"][:R], ref["logu"], rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(g["logratio"][:R], ref["logratio"], rtol=1e-6, atol=1e-6)
    near = list_near_ties(S["wl"].name, ref["logu"], ref["logratio"], o["row_ptr"], window,
                          drafted_rows(o["row_ptr"], o["row_t"], S["bonus"]))
    diff = g["flags"][:R] != ref["flags"]
    assert not np.any(diff & ~near), "accept flag differs outside the near-tie window"
    env_ok = np.array([not np.any(diff[o["row_ptr"][b]:o["row_ptr"][b + 1]]) for b in range(B)])
    for k in ("n_accept", "n_adv", "t_next"):
        np.testing.assert_array_equal(g[k][env_ok], ref[k][env_ok])
    np.testing.assert_allclose(g["x_out"][env_ok], ref["x_out"][env_ok], rtol=1e-5, atol=1e-6)
    return g, ref, env_ok


def _stage_parity(wl, B, t0, K, s, env=None, clip=None, b_std=0.02, paths=None, sampler=0, eta=1.0, bonus=False, norm=0):
    S = _setup(wl, B, clip=clip, b_std=b_std, sampler=sampler, eta=eta, bonus=bonus, norm=norm)
    if paths is not None:
        assert (S["ctx"].path_name(0), S["ctx"].path_name(1)) == paths
    tol = TOL[wl.dtype]
    rows = _gpu_draft(S, t0, K, s, env)
    o = _check_draft(S, rows, t0, K, s, env, tol)
    _check_verify(S, rows, o, tol)
    g, ref, _ = _check_accept(S, rows, o, s, env, 1e-9)
    S["ctx"].close()
    return g, ref


def test_c1_stages():
    wl = ti.C1
    g, ref = _stage_parity(wl, 1, np.array([9]), np.array([4]), np.array([1.0]), paths=("f32-mfma-fused", "f32-mfma-fused"))
    assert ref["n_adv"][0] >= 1


def test_c1_ragged_edges_with_clip():
    # K_eff = 0 (t0 = 0), finished env, t0 < K, K = 1, per-env sigma scale, env ids, clamped x0
    wl = ti.small_variant(ti.C1, B=8)
    t0 = np.array([9, 0, -1, 2, 5, 7, 1, 9]); K = np.array([4, 4, 4, 4, 1, 1, 3, 2])
    s = np.array([1.0, 1.0, 1.0, 1.3, 1.0, 1.5, 1.2, 1.1]); env = np.array([5, 900, 3, 77, 1, 0, 12345678, 42])
    for clip in (None, 1.0):
        g, ref = _stage_parity(wl, 8, t0, K, s, env, clip=clip)
        np.testing.assert_array_equal(ref["n_adv"][[1, 2, 4]], [1, 0, 1])


def test_c2_stages():
    wl = ti.C2
    _stage_parity(wl, 1, np.array([99]), np.array([8]), np.array([1.0]), paths=("f32-mfma-fused", "f32-mfma-fused"))
    _stage_parity(wl, 1, np.array([50]), np.array([8]), np.array([1.0]))


@pytest.mark.parametrize("name,B", [("C3", 3), ("C5", 6)])
def test_bf16_vector_cond_stages(name, B):
    wl = ti.small_variant(ti.WORKLOADS[name], B=B)
    t0, K, s = ti.make_schedule_inputs(wl, B, t0=None if wl.ragged else 60)
    _stage_parity(wl, B, t0, K, s, paths=("bf16-mfma-fused", "bf16-mfma-fused"))


def test_c4_cross_attention_stages():
    wl = ti.small_variant(ti.C4, B=2, base=ti.NetShape(3, 512, 8))
    t0, K, s = ti.make_schedule_inputs(wl, 2, t0=40)
    _stage_parity(wl, 2, t0, K, s, paths=("bf16-mfma-fused", "bf16-mfma-fused"))


def _round_parity(wl, B, t0, K, s, env, head_scale=1.0):
    """tsdp_round against the oracle's round.  The same inputs also go through the three stages with diagnostics,
    which gives the GPU's own log alpha of every row: the fused round must equal the stages bit for bit, accept
    decisions must equal the oracle's outside the near-tie window (near-tie rows are printed), and the final actions
    of every compared environment must agree elementwise.  At least one environment must be compared."""
    import torch
    S = _setup(wl, B, head_scale=head_scale)
    ctx = S["ctx"]
    sd = to_dev(s.astype(np.float32)); ed = None if env is None else to_dev(env.astype(np.int32))
    rows = _gpu_draft(S, t0, K, s, env)
    ctx.tsdp_verify(B, rows)
    st = {k: v.cpu().numpy() for k, v in ctx.tsdp_accept(B, sd, ed, rows).items()}
    x = to_dev(S["x"]); t = to_dev(t0.astype(np.int32))
    nacc = torch.zeros(B, dtype=torch.int32, device="cuda"); nadv = torch.zeros_like(nacc)
    ctx.tsdp_round(x, t, to_dev(K.astype(np.int32)), sd, ed, nacc, nadv)
    g = dict(x=x.cpu().numpy(), t=t.cpu().numpy(), nacc=nacc.cpu().numpy(), nadv=nadv.cpu().numpy())
    np.testing.assert_array_equal(g["nacc"], st["n_accept"])
    np.testing.assert_array_equal(g["nadv"], st["n_adv"])
    np.testing.assert_array_equal(g["t"], st["t_next"])
    np.testing.assert_array_equal(g["x"], st["x_out"])
    ref = sr.spec_round(S["base"], S["drafter"], S["sched"], S["x"], t0, K, s, env, S["seed"], S["cond"])
    d = ref["draft"]; rp = d["row_ptr"]; R = int(rp[-1])
    drafted = d["row_t"] > 0
    near = list_near_ties(wl.name, ref["logu"], ref["logratio"], rp, TIE, drafted)
    dl = np.abs(st["logratio"][:R] - ref["logratio"])
    # rows up to the oracle's first rejection see the same states on both sides: there the decisions are comparable
    seen = np.zeros(R, bool)
    for b in range(B):
        seen[rp[b]:rp[b] + min(int(ref["n_accept"][b]) + 1, rp[b + 1] - rp[b])] = True
    print(f"[{wl.name}] round: max |log alpha (GPU) - log alpha (oracle)| on compared rows = {dl[seen & drafted].max(initial=0.0):.3e}")
    mism = (st["flags"][:R] != ref["flags"]) & seen & drafted
    # a decision may differ inside the near-tie window, or where the network's own rounding error on log alpha (the
    # GPU's fp32 / bf16 forward against the oracle's fp64, shown here per row) reaches the margin of that row
    margin = np.abs(ref["logu"] - ref["logratio"])
    for r in np.nonzero(mism)[0]:
        print(f"[{wl.name}] row {int(r)}: decision differs, margin {margin[r]:.3e}, network error on log alpha {dl[r]:.3e}")
    bad = mism & ~near & (margin > dl + TIE)
    assert not np.any(bad), ("accept decision differs outside the near-tie window", np.nonzero(bad)[0], margin[bad], dl[bad])
    ok = np.array([not np.any((near | mism)[rp[b]:rp[b + 1]] & seen[rp[b]:rp[b + 1]]) for b in range(B)])
    assert ok.any(), "every environment has a near-tie row: nothing was compared"
    np.testing.assert_array_equal(g["nacc"][ok], ref["n_accept"][ok])
    np.testing.assert_array_equal(g["nadv"][ok], ref["n_adv"][ok])
    np.testing.assert_array_equal(g["t"][ok], ref["t_next"][ok])
    w = assert_latents_close(g["x"][ok], ref["x_out"][ok], wl.dtype, "final actions of tsdp_round")
    print(f"[{wl.name}] round: {int(ok.sum())}/{B} environments compared, final actions at {w:.3f} of the elementwise bound")
    assert ctx.tsdp_status() == 0
    ctx.close()
    return ref, ~ok


def test_c1_round():
    ref, near = _round_parity(ti.C1, 1, np.array([9]), np.array([4]), np.array([1.0]), None)
    assert not near.any()


def test_c2_round_and_chain():
    wl = ti.C2
    for t0 in (99, 50, 8, 3):
        ref, near = _round_parity(wl, 1, np.array([t0]), np.array([8]), np.array([1.0]), None)
        assert not near.any()


def test_round_ragged_batch_fp32():
    wl = ti.small_variant(ti.C2, B=12, base=ti.NetShape(3, 256, 4))
    rng = np.random.default_rng(3)
    t0 = rng.integers(-1, 100, 12); K = rng.integers(1, 9, 12); s = rng.uniform(1, 1.5, 12)
    t0[:3] = [0, -1, 2]
    ref, near = _round_parity(wl, 12, t0, K, s, np.arange(12) + 1000, head_scale=0.5)
    assert near.sum() <= 2
    assert (ref["n_accept"] > 0).any() and (ref["n_accept"] < ref["draft"]["K_eff"]).any()


def test_device_status_reports_clamped_inputs():
    wl = ti.C1
    S = _setup(wl, 1)
    rows = S["ctx"].alloc_rows(1)
    S["ctx"].tsdp_draft(to_dev(S["x"]), to_dev(np.array([50], np.int32)), to_dev(np.array([9], np.int32)),
                        to_dev(np.array([1.0], np.float32)), None, rows)
    assert S["ctx"].tsdp_status() == 3                                # K > K_max and t0 >= T, both clamped
    assert rows["row_ptr"].cpu().numpy().tolist() == [0, 4]
    assert rows["row_t"].cpu().numpy()[:4].tolist() == [9, 8, 7, 6]
    assert S["ctx"].tsdp_status() == 0
    # K = 0 has no meaning without the bonus row: reported and run as K = 1
    S["ctx"].tsdp_draft(to_dev(S["x"]), to_dev(np.array([5], np.int32)), to_dev(np.array([0], np.int32)),
                        to_dev(np.array([1.0], np.float32)), None, rows)
    assert S["ctx"].tsdp_status() == 1
    assert rows["row_ptr"].cpu().numpy().tolist() == [0, 1] and rows["row_t"].cpu().numpy()[0] == 5
    np.testing.assert_array_equal(rows["states"].cpu().numpy()[0], np.asarray(S["x"][0], np.float32))
    S["ctx"].close()


def test_error_paths_return_codes():
    import torch
    from paper_2512_15773_amd import Tsdp, TsdpError
    wl = ti.C1
    ctx = Tsdp.from_workload(wl)
    x = torch.zeros(1, wl.H, wl.A, device="cuda"); i = torch.zeros(1, dtype=torch.int32, device="cuda")
    f = torch.ones(1, device="cuda")
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_round(x, i, i, f, None)
    assert e.value.code == -5                                          # weights not loaded
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_load_weights(0, np.zeros(7, np.float32))
    assert e.value.code == -2
    ctx.tsdp_load_weights(0, ti.pack_blob(ti.make_weights(wl, "base")))
    ctx.tsdp_load_weights(1, ti.pack_blob(ti.make_weights(wl, "draft")))
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_round(x, i, i, f, None)
    assert e.value.code == -5                                          # conditioning not set
    ctx.tsdp_set_cond(torch.zeros(1, wl.cond_dim, device="cuda"))
    x2 = torch.zeros(2, wl.H, wl.A, device="cuda")
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_round(x2, torch.zeros(2, dtype=torch.int32, device="cuda"), torch.zeros(2, dtype=torch.int32, device="cuda"),
                       torch.ones(2, device="cuda"), None)
    assert e.value.code == -2                                          # B > B_max
    ctx.tsdp_round(x, i, i, f, None)
    # the enqueue-only chain: negative round count, bad stage bounds, null latents
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_chain_enqueue(x, i, i, f, None, None, -1)
    assert e.value.code == -1
    with pytest.raises(TsdpError) as e:
        ctx.tsdp_chain_enqueue(x, i, torch.zeros(1, 3, dtype=torch.int32, device="cuda"), torch.ones(1, 3, device="cuda"),
                               None, None, 2, stages=(2, 3))
    assert e.value.code == -1
    assert ctx.lib.tsdp_chain_enqueue(ctx.ctx, 1, None, None, None, None, None, 0, 0, 0, None, 1, None, None, None, None, None) == -1
    assert ctx.lib.tsdp_prepare(None) == -1
    ctx.close()


def test_threshold_rule_matches_oracle():
    # deterministic p >= lambda rule (Section 3.2) on identical tensors: flags exact outside the near-tie window
    wl = ti.small_variant(ti.C2, B=10, base=ti.NetShape(2, 256, 4))
    S = _setup(wl, 10, head_scale=0.5)
    rng = np.random.default_rng(4)
    t0 = rng.integers(0, 100, 10); K = rng.integers(1, 9, 10); s = rng.uniform(1, 1.5, 10); lam = rng.uniform(0.05, 1.0, 10)
    lam[0] = 1.0
    rows = _gpu_draft(S, t0, K, s, None)
    S["ctx"].tsdp_verify(10, rows)
    out = S["ctx"].tsdp_accept_threshold(10, to_dev(s.astype(np.float32)), to_dev(lam.astype(np.float32)), rows)
    g = {k: v.cpu().numpy() for k, v in out.items()}
    R = int(rows["row_ptr"].cpu().numpy()[-1])
    ref = sr.accept(S["sched"], rows["row_ptr"].cpu().numpy(), rows["row_t"].cpu().numpy()[:R], s.astype(np.float32), None,
                    S["seed"], rows["states"].cpu().numpy()[:R], rows["eps_p"].cpu().numpy()[:R],
                    rows["eps_q"].cpu().numpy()[:R], rows["xi"].cpu().numpy()[:R], rows["y_last"].cpu().numpy(),
                    lam=lam.astype(np.float32))
    near = np.abs(ref["logu"] - ref["logratio"]) < 1e-6
    assert not np.any((g["flags"][:R] != ref["flags"]) & ~near)
    assert not near.any()
    for k in ("n_accept", "n_adv", "t_next"):
        np.testing.assert_array_equal(g[k], ref[k])
    np.testing.assert_allclose(g["x_out"], ref["x_out"], rtol=1e-5, atol=1e-6)
    assert 0 < g["flags"][:R].sum() < R
    # the fused round with the same thresholds gives the same counters
    import torch
    x = to_dev(S["x"]); t = to_dev(t0.astype(np.int32)); na = torch.zeros(10, dtype=torch.int32, device="cuda"); nd = torch.zeros_like(na)
    S["ctx"].tsdp_round_threshold(x, t, to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32)), None,
                                  to_dev(lam.astype(np.float32)), na, nd)
    np.testing.assert_array_equal(na.cpu().numpy(), ref["n_accept"])
    np.testing.assert_array_equal(t.cpu().numpy(), ref["t_next"])
    S["ctx"].close()


def test_chain_runs_rounds_until_every_environment_finishes():
    # fp32: the chain driver must equal the oracle's round applied repeatedly (same noise stream, same decisions)
    wl = ti.small_variant(ti.C1, B=6)
    S = _setup(wl, 6, head_scale=0.6)
    t0 = np.array([9, 9, 6, 3, 0, -1]); K = np.array([4, 2, 4, 3, 4, 4]); s = np.array([1.0, 1.2, 1.0, 1.0, 1.0, 1.0])
    x = to_dev(S["x"]); t = to_dev(t0.astype(np.int32))
    rounds, tot = S["ctx"].tsdp_chain(x, t, to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32)), None, check_every=1)
    xr, tr = np.asarray(S["x"], float), t0.copy()
    acc = np.zeros(6, int); drafts = np.zeros(6, int); nr = np.zeros(6, int); n = 0
    while (tr >= 0).any():
        r = sr.spec_round(S["base"], S["drafter"], S["sched"], xr, tr, K, s, None, S["seed"], S["cond"])
        ran = tr >= 0
        acc += r["n_accept"]; drafts += r["draft"]["K_eff"]; nr += ran
        near = list_near_ties("C1 chain", r["logu"], r["logratio"], r["draft"]["row_ptr"], TIE, r["draft"]["row_t"] > 0)
        assert not near.any()                                             # no near-tie on this seed: decisions are comparable
        xr, tr = r["x_out"], r["t_next"]; n += 1
    assert rounds == n
    assert (t.cpu().numpy() == -1).all()
    np.testing.assert_array_equal(tot["accept"].cpu().numpy(), acc)
    np.testing.assert_array_equal(tot["drafts"].cpu().numpy(), drafts)
    np.testing.assert_array_equal(tot["rounds"].cpu().numpy(), nr)
    # up to four rounds compound their fp32 rounding in the final action: the per-round bound, once per round
    assert assert_latents_close(x.cpu().numpy(), xr, "fp32", "final actions of the chain") <= 1.0
    S["ctx"].close()


def test_chain_bf16_invariants():
    # every environment ends at t = -1 and the rounds it ran advance it by exactly t0 + 1 steps in total
    wl = ti.small_variant(ti.C3, B=12)
    S = _setup(wl, 12, head_scale=0.2, b_std=0.0)
    t0 = np.array([99, 99, 80, 64, 50, 33, 17, 16, 15, 1, 0, -1]); K = np.full(12, 16); s = np.ones(12)
    x = to_dev(S["x"]); t = to_dev(t0.astype(np.int32))
    rounds, tot = S["ctx"].tsdp_chain(x, t, to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32)), None, check_every=3)
    assert (t.cpu().numpy() == -1).all() and np.isfinite(x.cpu().numpy()).all()
    a, d, r = (tot[k].cpu().numpy() for k in ("accept", "drafts", "rounds"))
    assert r[-1] == 0 and r[-2] == 1 and (r[:-1] >= 1).all() and rounds >= r.max()
    assert (a <= d).all() and (a[:4] > 0).all()
    # steps advanced = accepted drafts + one corrected / base step per round that did not accept everything;
    # at least one step per round and never more than t0 + 1 in total
    assert ((a + r >= t0 + 1) | (t0 < 0)).all()
    S["ctx"].close()


def test_operator_kernel_path_for_shapes_without_a_fused_kernel():
    # a width with no compiled fused kernel (d = 96) runs the general fp32 operator kernels, both conditioning modes
    for cm, extra in ((0, {}), (1, dict(cond_dim=24, cond_tokens=5))):
        wl = ti.small_variant(ti.C1, B=3, cond_mode=cm, base=ti.NetShape(2, 96, 3), draft=ti.NetShape(1, 48, 3), **extra)
        t0 = np.array([9, 4, 0]); K = np.array([4, 3, 2]); s = np.array([1.0, 1.3, 1.0])
        _stage_parity(wl, 3, t0, K, s, paths=("f32-ops", "f32-ops"))


def test_distillation_loss_matches_oracle():
    wl = ti.small_variant(ti.C2, B=9, base=ti.NetShape(2, 256, 4))
    for clip in (None, 1.5):
        S = _setup(wl, 9, clip=clip)
        t0 = np.array([99, 70, 40, 20, 9, 3, 1, 0, -1]); K = np.full(9, 8); s = np.ones(9)
        rows = _gpu_draft(S, t0, K, s, None)
        S["ctx"].tsdp_verify(9, rows)
        R = int(rows["row_ptr"].cpu().numpy()[-1])
        got = S["ctx"].tsdp_distill_loss(R, rows, 0.7, 0.3).cpu().numpy()
        ref = sr.distill_loss(S["sched"], rows["row_t"].cpu().numpy()[:R], rows["states"].cpu().numpy()[:R],
                              rows["eps_p"].cpu().numpy()[:R], rows["eps_q"].cpu().numpy()[:R],
                              float(np.float32(0.7)), float(np.float32(0.3)), clip)   # the ABI takes the weights as fp32
        np.testing.assert_allclose(got, ref, rtol=1e-10)
        again = S["ctx"].tsdp_distill_loss(R, rows, 0.7, 0.3).cpu().numpy()
        assert got.tobytes() == again.tobytes()                            # fixed reduction order
        assert got[0] > 0 and got[1] > 0
        S["ctx"].close()


def test_ddim_sampler_stages_and_loss():
    # DDIM(eta) transitions in the draft step, the acceptance ratio, the reflection, the last step and the loss
    wl = ti.small_variant(ti.C1, B=7)
    t0 = np.array([9, 6, 3, 1, 0, -1, 9]); K = np.array([4, 4, 4, 2, 4, 4, 1]); s = np.array([1.0, 1.3, 1.0, 1.0, 1.0, 1.0, 1.1])
    for clip in (None, 1.0):
        _stage_parity(wl, 7, t0, K, s, clip=clip, sampler=1, eta=0.6)
    wl = ti.small_variant(ti.C3, B=4)
    t0, K, s = ti.make_schedule_inputs(wl, 4, t0=45)
    _stage_parity(wl, 4, t0, K, s, sampler=1, eta=1.0, paths=("bf16-mfma-fused", "bf16-mfma-fused"))
    S = _setup(ti.small_variant(ti.C2, B=3, base=ti.NetShape(2, 256, 4)), 3, clip=2.0, sampler=1, eta=0.5)
    rows = _gpu_draft(S, np.array([60, 9, 0]), np.full(3, 8), np.ones(3), None)
    S["ctx"].tsdp_verify(3, rows)
    R = int(rows["row_ptr"].cpu().numpy()[-1])
    got = S["ctx"].tsdp_distill_loss(R, rows, 1.0, 1.0).cpu().numpy()
    ref = sr.distill_loss(S["sched"], rows["row_t"].cpu().numpy()[:R], rows["states"].cpu().numpy()[:R],
                          rows["eps_p"].cpu().numpy()[:R], rows["eps_q"].cpu().numpy()[:R], 1.0, 1.0, 2.0)
    np.testing.assert_allclose(got, ref, rtol=1e-10)
    S["ctx"].close()


def test_bonus_row_stages_rounds_and_chain():
    # K+1 candidate set: the extra base row in the row table, in verification and in the commit; K = 0 = plain base step
    wl = ti.small_variant(ti.C1, B=8)
    t0 = np.array([9, 0, -1, 2, 5, 7, 1, 9]); K = np.array([4, 4, 4, 4, 0, 1, 3, 2])
    s = np.array([1.0, 1.0, 1.0, 1.3, 1.0, 1.5, 1.2, 1.1]); env = np.array([5, 900, 3, 77, 1, 0, 12345678, 42])
    for clip in (None, 1.0):
        g, ref = _stage_parity(wl, 8, t0, K, s, env, clip=clip, bonus=True)
        np.testing.assert_array_equal(ref["n_adv"][[1, 2, 4]], [1, 0, 1])
        assert (ref["n_adv"] == ref["n_accept"] + 1)[t0 >= 0].all()     # a corrected or a base step ends every round
    wl = ti.small_variant(ti.C3, B=5)
    t0, K, s = ti.make_schedule_inputs(wl, 5, t0=45)
    t0[3] = 2; t0[4] = 0
    _stage_parity(wl, 5, t0, K, s, bonus=True, paths=("bf16-mfma-fused", "bf16-mfma-fused"))
    # identical networks: every draft passes and each round advances K_eff + 1 exact base steps
    wl = ti.small_variant(ti.C1, B=4)
    wb = ti.make_weights(wl, "base", b_std=0.02)
    cond = ti.make_cond(wl, 4); x0 = ti.make_latents(wl, 4)
    wl_same = ti.small_variant(wl, draft=wl.base)
    base, _, sched = oracle_side(wl_same, wb, wb)
    ctx = gpu_side(wl_same, wb, wb, cond, B_max=4, bonus_row=True)
    t0 = np.array([9, 9, 4, 1]); K = np.array([3, 2, 4, 4]); s = np.ones(4)
    x = to_dev(x0); t = to_dev(t0.astype(np.int32))
    rounds, tot = ctx.tsdp_chain(x, t, to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32)), None, check_every=2)
    ref = sr.chain(base, base, sched, x0, t0, K, s, None, wl.philox_seed, cond, bonus=True)
    assert rounds >= ref["rounds"] and (t.cpu().numpy() == -1).all()
    np.testing.assert_array_equal(tot["rounds"].cpu().numpy(), ref["totals"]["rounds"])
    np.testing.assert_array_equal(tot["rounds"].cpu().numpy(), [3, 4, 1, 1])            # ceil((t0+1)/(K+1))
    np.testing.assert_array_equal(tot["accept"].cpu().numpy(), ref["totals"]["accept"])
    assert_latents_close(x.cpu().numpy(), ref["x"], "fp32", "final actions of the bonus-row chain")
    ctx.close()


@pytest.mark.parametrize("bonus", [False, True])
def test_row_table_of_a_batch_of_several_thousand_environments(bonus):
    # the plan kernel scans environments in chunks of 1024: a batch over several chunks with a ragged tail, finished
    # environments, t0 = 0 and (bonus row) K = 0 against the oracle's row table; the base rows' states are the inputs
    B = 2500
    wl = ti.small_variant(ti.C1, B=B)
    rng = np.random.default_rng(77)
    t0 = rng.integers(-1, wl.T, B); K = rng.integers(0 if bonus else 1, wl.K_max + 1, B)
    t0[1023:1026] = [0, -1, wl.T - 1]; K[1023:1026] = [wl.K_max, 1, 0 if bonus else 1]
    S = _setup(wl, B, bonus=bonus)
    rows = _gpu_draft(S, t0, K, np.ones(B), None)
    K_eff, row_ptr, row_env, row_t = sr.plan_rows(t0, K, bonus)
    R = int(row_ptr[-1])
    np.testing.assert_array_equal(rows["row_ptr"].cpu().numpy(), row_ptr)
    np.testing.assert_array_equal(rows["row_t"].cpu().numpy()[:R], row_t)
    np.testing.assert_array_equal(rows["row_env"].cpu().numpy()[:R], row_env)
    first = row_ptr[:-1][np.diff(row_ptr) > 0]                       # every running environment's first row holds x
    live = np.flatnonzero(np.diff(row_ptr) > 0)
    np.testing.assert_array_equal(rows["states"].cpu().numpy()[first], S["x"][live])
    assert S["ctx"].tsdp_status() == 0
    S["ctx"].close()


def test_two_contexts_on_two_streams_do_not_share_state():
    # two contexts (different shapes, both with a FiLM product on their own second stream) run whole rounds at the same
    # time on two streams; every result is bit-identical to the same rounds run one context after the other
    import torch
    specs = [(ti.small_variant(ti.C3, B=24), 24, 30), (ti.small_variant(ti.C5, B=40), 40, None)]
    S, inputs = [], []
    for wl, B, t_fix in specs:
        S.append(_setup(wl, B, head_scale=0.3))
        t0, K, s = ti.make_schedule_inputs(wl, B, t0=t_fix)
        inputs.append((t0.astype(np.int32), K.astype(np.int32), s.astype(np.float32)))

    def tensors(i):
        t0, K, s = inputs[i]
        return dict(x=to_dev(S[i]["x"]), t=to_dev(t0), K=to_dev(K), s=to_dev(s),
                    na=torch.zeros(len(t0), dtype=torch.int32, device="cuda"),
                    nd=torch.zeros(len(t0), dtype=torch.int32, device="cuda"))

    def rounds(i, T, stream, n=3):
        with torch.cuda.stream(stream):
            for _ in range(n):
                S[i]["ctx"].tsdp_round(T["x"], T["t"], T["K"], T["s"], None, T["na"], T["nd"])

    main = torch.cuda.current_stream()
    want = [tensors(0), tensors(1)]
    for i in range(2):
        rounds(i, want[i], main)
        torch.cuda.synchronize()
    # every input exists (and stays alive) before anything is enqueued on the side streams: a tensor freed while a
    # stream that the allocator does not know of still reads it would be handed out again
    got = [tensors(0), tensors(1)]
    torch.cuda.synchronize()
    st = [torch.cuda.Stream(), torch.cuda.Stream()]
    rounds(0, got[0], st[0]); rounds(1, got[1], st[1])         # enqueued back to back, nothing waits in between
    torch.cuda.synchronize()
    for i in range(2):
        for name in ("x", "t", "na", "nd"):
            assert torch.equal(got[i][name], want[i][name]), (i, name)
        assert S[i]["ctx"].tsdp_status() == 0
        S[i]["ctx"].close()


def test_kernel_timing_brackets_the_chosen_stages():
    # measurement aid: event pairs around the stage kernels; a stage without a timed launch is an error, not a number
    from paper_2512_15773_amd import TsdpError
    wl = ti.small_variant(ti.C3, B=6)
    S = _setup(wl, 6)
    ctx = S["ctx"]
    t0, K, s = ti.make_schedule_inputs(wl, 6, t0=40)
    rows = _gpu_draft(S, t0, K, s, None)
    ctx.tsdp_verify(6, rows)
    ctx.tsdp_accept(6, to_dev(s.astype(np.float32)), None, rows)
    before = {k: v.clone() for k, v in rows.items()}
    ctx.tsdp_kernel_timing(True)                               # all stages
    with pytest.raises(TsdpError):
        ctx.tsdp_kernel_ms(1)                                  # nothing launched since timing was switched on
    ctx.tsdp_draft(to_dev(S["x"]), to_dev(t0.astype(np.int32)), to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32)),
                   None, rows)
    ctx.tsdp_verify(6, rows)
    ctx.tsdp_accept(6, to_dev(s.astype(np.float32)), None, rows)
    ms = [ctx.tsdp_kernel_ms(st) for st in range(4)]           # rollout, verify forward, acceptance, FiLM product
    assert all(0.0 < m < 1000.0 for m in ms), ms
    for k in ("states", "eps_p", "eps_q", "xi", "row_t"):      # timing changes no result
        assert torch_equal(rows[k], before[k]), k
    ctx.tsdp_kernel_timing(2 * 0b0010)                         # the verify forward only
    ctx.tsdp_verify(6, rows)
    assert ctx.tsdp_kernel_ms(1) > 0.0
    for st in (0, 2, 3):
        with pytest.raises(TsdpError):
            ctx.tsdp_kernel_ms(st)
    ctx.tsdp_kernel_timing(False)
    ctx.close()


def torch_equal(a, b):
    import torch
    return bool(torch.equal(a, b))


def test_draft_count_zero_is_the_plain_base_chain():
    # bonus-row context, K = 0 everywhere: every round is one base evaluation and one sampler step per environment
    # (no drafter work at all), so the chain is the base model's own reverse process with the round's noise stream
    for wl, B, dtype, paths in ((ti.small_variant(ti.C1, B=3), 3, "fp32", None),
                                (ti.small_variant(ti.C3, B=5), 5, "bf16", ("bf16-mfma-fused", "bf16-mfma-fused"))):
        S = _setup(wl, B, bonus=True)
        if paths is not None:
            assert (S["ctx"].path_name(0), S["ctx"].path_name(1)) == paths
        t0 = np.full(B, min(wl.T - 1, 9)); t0[-1] = 3           # a short chain: bf16 rounding adds up over the steps
        s = np.linspace(1.0, 1.4, B)
        x = to_dev(S["x"]); t = to_dev(t0.astype(np.int32))
        K0 = to_dev(np.zeros(B, dtype=np.int32))
        rounds, tot = S["ctx"].tsdp_chain(x, t, K0, to_dev(s.astype(np.float32)), None, check_every=1)
        assert rounds == t0.max() + 1 and (t.cpu().numpy() == -1).all()
        np.testing.assert_array_equal(tot["rounds"].cpu().numpy(), t0 + 1)
        np.testing.assert_array_equal(tot["drafts"].cpu().numpy(), 0)
        ref = S["x"].astype(np.float64); tt = t0.copy()
        while (tt >= 0).any():
            live = tt >= 0
            step = sr.base_chain_step(S["base"], S["sched"], ref[live], tt[live], s[live], np.arange(B)[live], S["seed"],
                                      S["cond"][live])
            ref[live] = step
            tt[live] -= 1
        assert_latents_close(x.cpu().numpy(), ref, dtype, "final actions of the plain chain")
        S["ctx"].close()


def test_staged_chain_follows_the_stage_tables():
    wl = ti.small_variant(ti.C1, B=6)
    S = _setup(wl, 6, head_scale=0.6)
    t0 = np.array([9, 9, 6, 3, 0, -1])
    K3 = np.array([[1, 4, 2], [2, 3, 1], [4, 4, 4], [1, 1, 3], [2, 2, 2], [1, 1, 1]])
    s3 = np.array([[1.0, 1.2, 1.0]] * 6); l3 = np.array([[0.3, 0.5, 0.9]] * 6)
    for lam in (None, l3):
        x = to_dev(S["x"]); t = to_dev(t0.astype(np.int32))
        rounds, tot = S["ctx"].tsdp_chain_staged(x, t, to_dev(K3.astype(np.int32)), to_dev(s3.astype(np.float32)),
                                                 None if lam is None else to_dev(lam.astype(np.float32)), 7, 3, None,
                                                 check_every=1)
        ref = sr.chain(S["base"], S["drafter"], S["sched"], S["x"], t0, K3, s3.astype(np.float32),
                       None, S["seed"], S["cond"], lam=None if lam is None else lam.astype(np.float32), stages=(7, 3))
        for r in ref["history"]:
            near = list_near_ties("C1 staged chain", r["logu"], r["logratio"], r["draft"]["row_ptr"], TIE, r["draft"]["row_t"] > 0)
            assert not near.any()
        assert rounds == ref["rounds"] and (t.cpu().numpy() == -1).all()
        for k in ("accept", "drafts", "rounds"):
            np.testing.assert_array_equal(tot[k].cpu().numpy(), ref["totals"][k])
        assert_latents_close(x.cpu().numpy(), ref["x"], "fp32", "final actions of the staged chain")
    import pytest as _pt
    from paper_2512_15773_amd import TsdpError
    with _pt.raises(TsdpError):
        S["ctx"].tsdp_chain_staged(x, t, to_dev(K3.astype(np.int32)), to_dev(s3.astype(np.float32)), None, 2, 3, None)
    S["ctx"].close()


def test_maximum_sizes_on_the_general_path():
    # the limits of the configuration: H*A = 512 elements per latent, K_max = 64 drafts, T = 4096 timesteps
    wl = ti.small_variant(ti.C1, B=3, H=32, A=16, T=4096, K_max=64, base=ti.NetShape(1, 96, 3), draft=ti.NetShape(1, 48, 3))
    t0 = np.array([4095, 2000, 40]); K = np.array([64, 64, 64]); s = np.array([1.0, 1.2, 1.0])
    g, ref = _stage_parity(wl, 3, t0, K, s, paths=("f32-ops", "f32-ops"))
    assert (ref["n_adv"] >= 1).all() and (ref["n_adv"] <= [64, 64, 40]).all()
    # past the limits the context is refused
    from paper_2512_15773_amd import Tsdp, TsdpError
    for kw in (dict(K_max=65), dict(T=4097), dict(A=17)):
        bad = ti.small_variant(wl, **kw)
        with pytest.raises(TsdpError):
            Tsdp.from_workload(bad, B_max=1)


def test_round_replays_from_a_captured_hip_graph():
    # a round is a fixed sequence of kernel launches on the caller's stream (no allocation after the first call, no
    # host synchronisation, no memset node): captured once, every replay must equal the eager round it stands for
    import torch
    wl = ti.small_variant(ti.C1, B=5)
    S = _setup(wl, 5, head_scale=0.6)
    ctx = S["ctx"]
    t0 = np.array([9, 9, 7, 5, 9], np.int32); K = to_dev(np.array([4, 2, 3, 4, 1], np.int32))
    s = to_dev(np.array([1.0, 1.1, 1.0, 1.2, 1.0], np.float32))

    def fresh():
        return to_dev(S["x"]), to_dev(t0), torch.zeros(5, dtype=torch.int32, device="cuda"), torch.zeros(5, dtype=torch.int32, device="cuda")

    # eager reference: four rounds in a row, with the state after each
    x, t, na, nd = fresh()
    eager = []
    for _ in range(4):
        ctx.tsdp_round(x, t, K, s, None, na, nd)
        torch.cuda.synchronize()
        eager.append((x.clone(), t.clone(), na.clone(), nd.clone()))
    # captured: the same buffers are updated in place by every replay
    x, t, na, nd = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        xw, tw, naw, ndw = fresh()
        ctx.tsdp_round(xw, tw, K, s, None, naw, ndw)              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.tsdp_round(x, t, K, s, None, na, nd)
    x.copy_(to_dev(S["x"])); t.copy_(to_dev(t0))                   # capture does not execute: start from the inputs
    for i in range(4):
        graph.replay()
        torch.cuda.synchronize()
        _ = (x * 2).sum().item()                                   # eager work and a synchronisation between replays
        for got, want in zip((x, t, na, nd), eager[i]):
            assert torch.equal(got, want), f"replay {i} differs from the eager round"
    assert ctx.tsdp_status() == 0
    ctx.close()


def test_round_does_not_depend_on_batch_composition():
    # sharding invariance: with global environment ids as Philox counters, an environment's round is bit-identical
    # whatever batch (order, neighbours, size) it is computed in
    import torch
    wl = ti.small_variant(ti.C3, B=12)
    S = _setup(wl, 12, head_scale=0.3)
    ctx = S["ctx"]
    rng = np.random.default_rng(5)
    t0 = rng.integers(0, 100, 12).astype(np.int32); K = rng.integers(1, 17, 12).astype(np.int32)
    s = rng.uniform(1, 1.5, 12).astype(np.float32); env = (np.arange(12) + 500).astype(np.int32)

    def run(idx):
        ctx.tsdp_set_cond(to_dev(S["cond"][idx]))
        x = to_dev(np.asarray(S["x"])[idx]); t = to_dev(t0[idx])
        na = torch.zeros(len(idx), dtype=torch.int32, device="cuda"); nd = torch.zeros_like(na)
        ctx.tsdp_round(x, t, to_dev(K[idx]), to_dev(s[idx]), to_dev(env[idx]), na, nd)
        return x.cpu().numpy(), t.cpu().numpy(), na.cpu().numpy()

    full = run(np.arange(12))
    perm = rng.permutation(12)
    shuffled = run(perm)
    part = run(np.array([7, 2, 9]))
    for got, idx in ((shuffled, perm), (part, np.array([7, 2, 9]))):
        for a, b in zip(got, full):
            np.testing.assert_array_equal(a, b[idx])
    ctx.close()
    # also across the drafter's tile variants: 800 environments take the four-environment tile, 5 the single one
    wl = ti.small_variant(ti.C5, B=800, base=ti.NetShape(1, 384, 6))
    wb = ti.make_weights(wl, "base", head_scale=0.3); wd = ti.make_weights(wl, "draft", head_scale=0.3)
    cond = ti.make_cond(wl, 800); x0 = np.asarray(ti.make_latents(wl, 800))
    t0, K, s = ti.make_schedule_inputs(wl, 800)
    env = np.arange(800, dtype=np.int32)
    ctx = gpu_side(wl, wb, wd, cond, B_max=800)

    def run5(idx):
        ctx.tsdp_set_cond(to_dev(cond[idx]))
        x = to_dev(x0[idx]); t = to_dev(t0[idx].astype(np.int32))
        na = torch.zeros(len(idx), dtype=torch.int32, device="cuda")
        ctx.tsdp_round(x, t, to_dev(K[idx].astype(np.int32)), to_dev(s[idx].astype(np.float32)), to_dev(env[idx]), na, None)
        return x.cpu().numpy(), t.cpu().numpy(), na.cpu().numpy()

    full = run5(np.arange(800))
    idx = np.array([3, 250, 251, 600, 799])
    for a, b in zip(run5(idx), full):
        np.testing.assert_array_equal(a, b[idx])
    ctx.close()


def test_acceptance_with_regenerated_noise_matches_stored_noise():
    # d_xi = NULL in tsdp_draft / tsdp_accept: the kernel redraws the Philox blocks of every row
    wl = ti.small_variant(ti.C1, B=8)
    t0 = np.array([9, 0, -1, 2, 5, 7, 1, 9]); K = np.array([4, 4, 4, 4, 1, 1, 3, 2])
    s = np.array([1.0, 1.0, 1.0, 1.3, 1.0, 1.5, 1.2, 1.1]); env = np.array([5, 900, 3, 77, 1, 0, 12345678, 42])
    for clip, bonus in ((None, False), (1.0, False), (None, True)):
        S = _setup(wl, 8, clip=clip, bonus=bonus)
        ctx = S["ctx"]
        rows = _gpu_draft(S, t0, K, s, env)
        ctx.tsdp_verify(8, rows)
        sd, ed = to_dev(s.astype(np.float32)), to_dev(env.astype(np.int32))
        stored = {k: v.cpu().numpy() for k, v in ctx.tsdp_accept(8, sd, ed, rows).items()}
        rows_nx = dict(rows); rows_nx["xi"] = None
        redrawn = {k: v.cpu().numpy() for k, v in ctx.tsdp_accept(8, sd, ed, rows_nx).items()}
        for k in ("flags", "n_accept", "n_adv", "t_next", "logratio", "logu", "x_out"):
            np.testing.assert_array_equal(redrawn[k], stored[k])     # the same fp32 noise, bit for bit
        # and a rollout that never stored the noise leaves the other outputs unchanged
        rows2 = ctx.alloc_rows(8); rows2["xi"] = None
        ctx.tsdp_draft(to_dev(S["x"]), to_dev(t0.astype(np.int32)), to_dev(K.astype(np.int32)), sd, ed, rows2)
        for k in ("row_ptr", "states", "eps_p", "y_last"):
            np.testing.assert_array_equal(rows2[k].cpu().numpy(), rows[k].cpu().numpy())
        ctx.close()


def test_rmsnorm_networks_on_every_path():
    # norm = 1: RMSNorm in place of LayerNorm in both networks (fused fp32, fused bf16 with either conditioning,
    # general operator kernels)
    wl = ti.small_variant(ti.C1, B=3)
    _stage_parity(wl, 3, np.array([9, 5, 0]), np.array([4, 4, 4]), np.ones(3), norm=1, paths=("f32-mfma-fused", "f32-mfma-fused"))
    wl = ti.small_variant(ti.C3, B=3)
    t0, K, s = ti.make_schedule_inputs(wl, 3, t0=60)
    _stage_parity(wl, 3, t0, K, s, norm=1, paths=("bf16-mfma-fused", "bf16-mfma-fused"))
    wl = ti.small_variant(ti.C4, B=2, base=ti.NetShape(2, 512, 8))
    t0, K, s = ti.make_schedule_inputs(wl, 2, t0=40)
    _stage_parity(wl, 2, t0, K, s, norm=1, paths=("bf16-mfma-fused", "bf16-mfma-fused"))
    wl = ti.small_variant(ti.C1, B=2, base=ti.NetShape(2, 96, 3), draft=ti.NetShape(1, 48, 3))
    _stage_parity(wl, 2, np.array([9, 4]), np.array([4, 4]), np.ones(2), norm=1, paths=("f32-ops", "f32-ops"))


def test_action_dim_above_one_head_fragment():
    # A = 20, 33: the output head spans two / three 16-row MFMA fragments in the fused kernels (verify and drafter)
    wl = ti.small_variant(ti.C3, B=3, A=20, base=ti.NetShape(2, 256, 4))
    t0, K, s = ti.make_schedule_inputs(wl, 3, t0=60)
    _stage_parity(wl, 3, t0, K, s, paths=("bf16-mfma-fused", "bf16-mfma-fused"))
    wl = ti.small_variant(ti.C2, B=2, H=16, A=20, base=ti.NetShape(2, 256, 4))
    _stage_parity(wl, 2, np.array([70, 5]), np.array([8, 8]), np.array([1.0, 1.2]), paths=("f32-mfma-fused", "f32-mfma-fused"))
    wl = ti.small_variant(ti.C1, B=2, H=16, A=32)
    _stage_parity(wl, 2, np.array([9, 3]), np.array([4, 4]), np.ones(2), paths=("f32-mfma-fused", "f32-mfma-fused"))


def _chain_both_ways(ctx, x0, t0, K, s, lam, env, stages, n_rounds, T):
    """Host-checked chain and enqueue-only chain (eager, then captured in a HIP graph and replayed three times with
    eager work between the replays) on the same inputs."""
    import torch
    dev = "cuda"
    Kd, sd = to_dev(K.astype(np.int32)), to_dev(s.astype(np.float32))
    ld = None if lam is None else to_dev(lam.astype(np.float32))
    ed = None if env is None else to_dev(env.astype(np.int32))
    x, t = to_dev(x0), to_dev(t0.astype(np.int32))
    if stages is None:
        rounds, tot = ctx.tsdp_chain(x, t, Kd, sd, ed, lam=ld, check_every=1)
    else:
        rounds, tot = ctx.tsdp_chain_staged(x, t, Kd, sd, ld, stages[0], stages[1], ed, check_every=1)
    want = dict(x=x.clone(), t=t.clone(), **{k: v.clone() for k, v in tot.items()})
    B = x.shape[0]
    x2, t2 = to_dev(x0), to_dev(t0.astype(np.int32))
    tot2 = {k: torch.full((B,), -5, dtype=torch.int32, device=dev) for k in ("accept", "drafts", "rounds")}
    run = torch.full((1,), -5, dtype=torch.int32, device=dev)
    ctx.tsdp_chain_enqueue(x2, t2, Kd, sd, ld, ed, n_rounds, stages=stages, totals=tot2, rounds_run=run)
    torch.cuda.synchronize()

    def check(tag):
        assert int(run.item()) == rounds, (tag, int(run.item()), rounds)
        assert torch.equal(x2, want["x"]) and torch.equal(t2, want["t"]), tag
        for k in tot2:
            assert torch.equal(tot2[k], want[k]), (tag, k)

    check("eager")
    # captured: kernel launches only, so the whole chain is one graph
    ctx.tsdp_prepare()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        xw, tw = to_dev(x0), to_dev(t0.astype(np.int32))
        ctx.tsdp_chain_enqueue(xw, tw, Kd, sd, ld, ed, 2, stages=stages)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.tsdp_chain_enqueue(x2, t2, Kd, sd, ld, ed, n_rounds, stages=stages, totals=tot2, rounds_run=run)
    for i in range(3):
        x2.copy_(to_dev(x0)); t2.copy_(to_dev(t0.astype(np.int32)))
        graph.replay()
        torch.cuda.synchronize()
        _ = (x2 * 2).sum().item()                                  # eager work and a synchronisation between replays
        check(f"replay {i}")
    assert rounds < n_rounds                                       # rounds past the end ran as empty launches
    return rounds


def test_enqueue_only_chain_is_bit_identical_to_the_host_checked_chain():
    # C1 (fp32) and C3 (bf16) shapes; plain, bonus row, stage tables with and without the threshold rule
    for name, B, bonus in (("C1", 6, False), ("C1", 6, True), ("C3", 12, False), ("C3", 12, True)):
        wl = ti.small_variant(ti.WORKLOADS[name], B=B)
        S = _setup(wl, B, head_scale=0.6 if name == "C1" else 0.2, bonus=bonus)
        rng = np.random.default_rng(17)
        t0 = rng.integers(-1, wl.T, B); t0[0] = wl.T - 1; t0[1] = 0
        K = rng.integers(0 if bonus else 1, wl.K_max + 1, B); s = rng.uniform(1.0, 1.3, B)
        env = rng.integers(0, 10 ** 6, B)
        n = _chain_both_ways(S["ctx"], S["x"], t0, K, s, None, env, None, wl.T + 3, wl.T)
        assert n >= 1
        K3 = rng.integers(0 if bonus else 1, wl.K_max + 1, (B, 3)); s3 = rng.uniform(1.0, 1.3, (B, 3))
        l3 = rng.uniform(0.2, 0.9, (B, 3))
        stages = (7 * wl.T // 10, 3 * wl.T // 10)
        _chain_both_ways(S["ctx"], S["x"], t0, K3, s3, None, None, stages, wl.T + 3, wl.T)
        _chain_both_ways(S["ctx"], S["x"], t0, K3, s3, l3, env, stages, wl.T + 3, wl.T)
        assert S["ctx"].tsdp_status() == 0
        S["ctx"].close()


def test_layernorm_statistics_survive_a_large_mean_in_fp32():
    # a residual stream whose mean is 12x its spread (token-embedding bias 0.5 on features of spread 0.04): the
    # one-pass variance E[x^2] - mean^2 loses 2^-24 mean^2 / var = 1e-5 of the variance in fp32, at the fp32
    # tolerance; the fused fp32 kernels centre their statistics
    for wl in (ti.small_variant(ti.C1, B=3), ti.small_variant(ti.C2, B=2, base=ti.NetShape(2, 256, 4))):
        wb = ti.make_weights(wl, "base", b_std=0.02); wd = ti.make_weights(wl, "draft", b_std=0.02)
        for w in (wb, wd):
            w["tok_b"] = (w["tok_b"] + np.float32(0.5)).astype(np.float32)
        B = wl.B
        cond, x = ti.make_cond(wl, B), ti.make_latents(wl, B)
        base, drafter, sched = oracle_side(wl, wb, wd)
        ctx = gpu_side(wl, wb, wd, cond)
        assert ctx.path_name(0) == "f32-mfma-fused" and ctx.path_name(1) == "f32-mfma-fused"
        t0 = np.full(B, wl.T - 2); K = np.full(B, wl.K_max); s = np.ones(B)
        S = dict(wl=wl, B=B, cond=cond, x=x, base=base, drafter=drafter, sched=sched, ctx=ctx, clip=None, bonus=False,
                 seed=wl.philox_seed)
        rows = _gpu_draft(S, t0, K, s, None)
        o = _check_draft(S, rows, t0, K, s, None, TOL["fp32"])
        _check_verify(S, rows, o, TOL["fp32"])
        ctx.close()


def test_prepare_makes_a_fresh_context_capturable_and_short_chains_stop_where_asked():
    # tsdp_prepare on a context that has never run: the very first round is recorded into a HIP graph (an allocation
    # or a launch-attribute call during capture would fail it) and its replay equals the eager round of a second
    # context; an enqueue-only chain of 2 rounds equals the host-checked chain cut at max_rounds = 2
    import torch
    wl = ti.small_variant(ti.C3, B=9)
    wb = ti.make_weights(wl, "base", head_scale=0.2); wd = ti.make_weights(wl, "draft", head_scale=0.2)
    cond, x0 = ti.make_cond(wl, 9), ti.make_latents(wl, 9)
    t0 = np.array([99, 80, 60, 40, 20, 10, 3, 0, -1], np.int32); K = np.full(9, 16, np.int32); s = np.ones(9, np.float32)
    Kd, sd = to_dev(K), to_dev(s)
    ref_ctx = gpu_side(wl, wb, wd, cond)
    xr, tr = to_dev(x0), to_dev(t0)
    na_r = torch.zeros(9, dtype=torch.int32, device="cuda"); nd_r = torch.zeros_like(na_r)
    ref_ctx.tsdp_round(xr, tr, Kd, sd, None, na_r, nd_r)
    torch.cuda.synchronize()
    ctx = gpu_side(wl, wb, wd, cond)
    ctx.tsdp_prepare()
    x, t = to_dev(x0), to_dev(t0)
    na = torch.zeros(9, dtype=torch.int32, device="cuda"); nd = torch.zeros_like(na)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.tsdp_round(x, t, Kd, sd, None, na, nd)
    for i in range(2):
        x.copy_(to_dev(x0)); t.copy_(to_dev(t0))
        graph.replay()
        torch.cuda.synchronize()
        for got, want in ((x, xr), (t, tr), (na, na_r), (nd, nd_r)):
            assert torch.equal(got, want), f"replay {i}"
    # a chain cut short
    xa, ta = to_dev(x0), to_dev(t0)
    rounds, tot = ref_ctx.tsdp_chain(xa, ta, Kd, sd, None, max_rounds=2, check_every=1)
    assert rounds == 2 and (ta.cpu().numpy()[:5] >= 0).all()
    xb, tb = to_dev(x0), to_dev(t0)
    totb = {k: torch.zeros(9, dtype=torch.int32, device="cuda") for k in ("accept", "drafts", "rounds")}
    run = torch.zeros(1, dtype=torch.int32, device="cuda")
    ctx.tsdp_chain_enqueue(xb, tb, Kd, sd, None, None, 2, totals=totb, rounds_run=run)
    torch.cuda.synchronize()
    assert int(run.item()) == 2 and torch.equal(xa, xb) and torch.equal(ta, tb)
    for k in totb:
        assert torch.equal(totb[k], tot[k])
    ctx.tsdp_chain_enqueue(xb, tb, Kd, sd, None, None, 0, rounds_run=run)     # zero rounds: nothing but the counter
    torch.cuda.synchronize()
    assert int(run.item()) == 0 and torch.equal(xa, xb)
    ref_ctx.close(); ctx.close()
