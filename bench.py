#!/usr/bin/env python3
"""Benchmark of the speculative denoising round on one MI355X.

One step = one tsdp_round (drafter rollout -> ragged batched verification -> acceptance) over one
batch of synthetic environments already resident in HBM.  Prints ONE JSON line:
accepted denoising steps/s (sum of steps advanced / wall time), the roofline of the dominant kernel
(the fused verify forward, bf16 MFMA) measured live with HIP events on the launch stream, the HBM
roofline of the acceptance kernel on a scaled stress shape, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import tsdp_inputs as ti  # noqa: E402

# head_scale that brings the per-draft acceptance (accepted / tested drafts) of the random-init
# (base, drafter) pair to about 85 %, the rate the paper tabulates in its supplementary per-task tables;
# found with --calibrate on the synthetic inputs of make_problem().
CALIBRATED_HEAD_SCALE = {"C1": 0.7, "C2": 0.15, "C3": 0.21, "C4": 0.12, "C5": 0.29}
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
# HBM bytes per launch of the fused verify forward (FETCH_SIZE + WRITE_SIZE, scaled by a 1 GiB copy), from the
# rocprofv3 --pmc runs summarised in profiles/verify_forward_hbm_traffic_c4_c5.txt
MEASURED_TRAFFIC_BYTES = {"C4": int((4.261 + 0.003) * 2 ** 30), "C5": int((2.192 + 0.004) * 2 ** 30)}


def verify_flops(wl, R):
    """Algorithmic flops of the fused verify forward over R rows: per token and layer the q|k|v, output and
    MLP products (24 d^2 for a 4x MLP) plus attention 4 H d (plus cross-attention 4 d^2 + 4 S d), and the token
    embedding / output head 4 A d per token.  The FiLM projections (8 d^2 per row and layer) are not counted:
    they run in their own kernel, or come from a per-timestep table, and are under 1 % of the total."""
    d, L, H, A, m = wl.base.d, wl.base.layers, wl.H, wl.A, wl.base.mlp_ratio * wl.base.d
    per_tok_layer = 2 * d * 3 * d + 2 * d * d + 4 * d * m + 4 * H * d
    per_row_layer = 0
    if wl.cond_mode == 1:
        per_tok_layer += 4 * d * d + 4 * wl.cond_tokens * d
    per_tok = L * per_tok_layer + 4 * A * d
    return R * (H * per_tok + L * per_row_layer)


def make_problem(wl, point):
    hs = {"natural": 1.0, "calibrated": CALIBRATED_HEAD_SCALE[wl.name]}.get(point, 1.0)
    wb = ti.make_weights(wl, "base", head_scale=hs)
    wd = wb if point == "identical" else ti.make_weights(wl, "draft", head_scale=hs)
    cond, x = ti.make_cond(wl), ti.make_latents(wl)
    rng = np.random.default_rng(99)
    if wl.ragged:
        t0, K, s = ti.make_schedule_inputs(wl)
    else:                                            # environments spread over the denoising chain
        _, K, s = ti.make_schedule_inputs(wl)
        t0 = rng.integers(wl.K_max, wl.T, size=wl.B).astype(np.int32)
    return wb, wd, cond, x, t0, K, s


def time_events(fn, iters, torch):
    """Durations (mean, p50, p95 in ms) of fn() on torch's current stream (the stream the library launches on)."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in ev:
        a.record(); fn(); b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in ev)
    return float(np.mean(ts)), ts[len(ts) // 2], ts[min(len(ts) - 1, int(0.95 * len(ts)))]


def time_kernel(ctx, fn, stage, iters):
    """Mean duration (ms) of the dominant kernel of a stage, from the library's own HIP events."""
    ctx.tsdp_kernel_timing(True)
    ts = []
    for _ in range(iters):
        fn()
        ts.append(ctx.tsdp_kernel_ms(stage))
    ctx.tsdp_kernel_timing(False)
    return float(np.mean(ts)), float(np.median(ts))


def cpu_baseline(wl, wb, wd, cond, x, t0, K, s, n_env, budget_s=20.0):
    from oracle import spec_round as sr
    from oracle.ddpm import Schedule
    from oracle.denoiser import Denoiser
    bf16 = wl.dtype == "bf16"
    base = Denoiser(wb, wl.base.layers, wl.base.heads, wl.cond_mode, bf16)
    drafter = Denoiser(wd, wl.draft.layers, wl.draft.heads, wl.cond_mode, bf16)
    sched = Schedule(wl.T, wl.schedule, wl.beta0 or 1e-4, wl.beta1 or 0.02)
    n_env = min(n_env, wl.B)
    sl = slice(0, n_env)
    reps, adv, t_start = 0, 0, time.perf_counter()
    while True:
        r = sr.spec_round(base, drafter, sched, x[sl], t0[sl], K[sl], s[sl], None, wl.philox_seed, cond[sl])
        adv += int(r["n_adv"].sum()); reps += 1
        el = time.perf_counter() - t_start
        if el > budget_s or reps >= 50:
            break
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = 1
    return {"value": adv / el, "unit": "accepted denoising steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{reps} oracle round(s) over the first {n_env} of {wl.B} environments of {wl.name} "
                      f"({el:.1f} s of CPU time, numpy fp64 with its BLAS threads)"}


def accept_xl(torch, Tsdp, dev, iters=20):
    """HBM roofline of the acceptance kernel on the scaled stress shape: 65536 environments x K = 16 rows of
    160 elements (2^20 rows), fp32 inputs written by other kernels beforehand (cold in the caches)."""
    wl = ti.C3
    B, K, D = 65536, 16, wl.D
    ctx = Tsdp.from_workload(wl, B_max=B, K_max=K)
    g = torch.Generator(device=dev); g.manual_seed(1)
    R = B * K
    rows = dict(row_ptr=(torch.arange(B + 1, device=dev, dtype=torch.int32) * K),
                row_env=torch.arange(B, device=dev, dtype=torch.int32).repeat_interleave(K),
                states=torch.randn(R, wl.H, wl.A, device=dev, generator=g),
                eps_p=0.3 * torch.randn(R, wl.H, wl.A, device=dev, generator=g),
                xi=torch.randn(R, wl.H, wl.A, device=dev, generator=g),
                y_last=torch.randn(B, wl.H, wl.A, device=dev, generator=g))
    # every draft passes (noise predictions agree to 1e-4): all rows are needed, the kernel's largest traffic
    rows["eps_q"] = rows["eps_p"] + 1e-4 * torch.randn(R, wl.H, wl.A, device=dev, generator=g)
    t0 = torch.randint(K, wl.T, (B,), device=dev, generator=g, dtype=torch.int32)
    rows["row_t"] = (t0.repeat_interleave(K) - torch.arange(K, device=dev, dtype=torch.int32).repeat(B)).contiguous()
    s = torch.ones(B, device=dev)
    out = ctx.tsdp_accept(B, s, None, rows, diagnostics=False)
    flush = torch.empty(512 * 1024 * 1024 // 4, device=dev)          # 512 MiB > L2 + Infinity Cache
    ctx.tsdp_kernel_timing(True)
    ts = []
    for _ in range(iters):
        flush.add_(1.0)                                              # evicts the inputs
        ctx.tsdp_accept_into(B, s, None, rows, out)
        ts.append(ctx.tsdp_kernel_ms(2))
    ctx.tsdp_kernel_timing(False)
    ms = float(np.mean(ts))
    alg = 3 * R * D * 4 + B * (2 * D * 4 + 12)       # eps_p, eps_q, xi per row; y_last read and x written per env
    acc = float(out["n_accept"].float().mean().item())
    # the same launch with the noise regenerated from its Philox counters instead of read back (xi = NULL):
    # one third fewer bytes for about 40 integer operations and 3 transcendentals per pair of normals
    rows_nx = dict(rows); rows_nx["xi"] = None
    ctx.tsdp_kernel_timing(True)
    ts = []
    for _ in range(iters):
        flush.add_(1.0)
        ctx.tsdp_accept_into(B, s, None, rows_nx, out)
        ts.append(ctx.tsdp_kernel_ms(2))
    ctx.tsdp_kernel_timing(False)
    ms_nx = float(np.mean(ts))
    alg_nx = 2 * R * D * 4 + B * (2 * D * 4 + 12)
    ctx.close()
    del flush
    return {"kernel": "k_accept", "shape": f"B={B} K={K} D={D} fp32 ({R} rows), all drafts accepted", "bound": "hbm",
            "achieved": alg / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": alg / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None, "ms": ms,
            "algorithmic_bytes": alg, "mean_accepted_drafts": acc,
            "noise_regenerated": {"ms": ms_nx, "algorithmic_bytes": alg_nx, "achieved": alg_nx / (ms_nx * 1e-3) / 1e9,
                                  "frac": alg_nx / (ms_nx * 1e-3) / 1e9 / PEAK_HBM_GBS}}


def operating_points(ctx, wl, torch, dev, round_ms):
    """Acceptance-dependent part of the metric at the other operating points (kernel time does not depend on the
    data, so steps/s = steps advanced per round / the measured round latency): natural = independent random-init
    pair; the two bounds: every draft accepted (a drafter identical to the base: K_eff steps per environment and
    round) and every first draft rejected (one step per environment and round); then the calibrated pair with every environment at the same timestep."""
    out = {}
    na = torch.zeros(wl.B, dtype=torch.int32, device=dev); nd = torch.zeros_like(na)

    def one_round(x, t0, K, s):
        xd, td = torch.from_numpy(x).to(dev), torch.from_numpy(t0.astype(np.int32)).to(dev)
        ctx.tsdp_round(xd, td, torch.from_numpy(K).to(dev), torch.from_numpy(s).to(dev), None, na, nd)
        keff = np.minimum(K, np.maximum(t0, 0))
        a = na.cpu().numpy()
        tested = int(np.minimum(a + 1, keff).sum())
        adv = int(nd.sum().item())
        return {"steps_advanced_per_round": adv, "acceptance_of_tested_drafts": int(a.sum()) / max(tested, 1),
                "acceptance_of_all_drafts": int(a.sum()) / max(int(keff.sum()), 1),
                "accepted_steps_per_s": adv / (round_ms * 1e-3)}

    wb, wd, cond, x, t0, K, s = make_problem(wl, "natural")
    ctx.tsdp_load_weights(0, ti.pack_blob(wb)); ctx.tsdp_load_weights(1, ti.pack_blob(wd))
    ctx.tsdp_set_cond(torch.from_numpy(cond).to(dev))
    out["natural"] = one_round(x, t0, K, s)
    keff = np.minimum(K, np.maximum(t0, 0))
    all_acc = int(np.where(t0 >= 0, np.maximum(keff, 1), 0).sum())    # identical drafter: every draft passes
    out["all_accept_bound"] = {"steps_advanced_per_round": all_acc, "accepted_steps_per_s": all_acc / (round_ms * 1e-3)}
    live = int((make_problem(wl, "calibrated")[4] >= 0).sum())
    out["all_reject_bound"] = {"steps_advanced_per_round": live, "accepted_steps_per_s": live / (round_ms * 1e-3)}
    wb, wd, cond, x, t0, K, s = make_problem(wl, "calibrated")
    ctx.tsdp_load_weights(0, ti.pack_blob(wb)); ctx.tsdp_load_weights(1, ti.pack_blob(wd))
    ctx.tsdp_set_cond(torch.from_numpy(cond).to(dev))
    sweep = {}
    for tt in sorted({wl.T - 1, 3 * wl.T // 4, wl.T // 2, wl.T // 4, wl.K_max}, reverse=True):
        r = one_round(x, np.full(wl.B, tt, dtype=np.int32), K, s)
        sweep[str(tt)] = {k: r[k] for k in ("steps_advanced_per_round", "acceptance_of_tested_drafts")}
    out["calibrated_by_start_timestep"] = sweep
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4", choices=list(ti.WORKLOADS))
    ap.add_argument("--point", default="calibrated", choices=["natural", "calibrated", "identical"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-chain", action="store_true", help="skip the whole-chain (action prediction) measurement")
    ap.add_argument("--no-accept-xl", action="store_true", help="skip the acceptance-kernel HBM stress shape")
    ap.add_argument("--no-points", action="store_true", help="skip the other acceptance operating points")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="end with one 1 GiB device-to-device copy (known traffic that scales rocprofv3's byte counters)")
    ap.add_argument("--cpu-envs", type=int, default=0, help="environments of the oracle sample (0 = by workload)")
    ap.add_argument("--calibrate", action="store_true", help="print acceptance vs head_scale and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (environments are independent; more GPUs would each "
              "take a slice of the batch). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_15773_amd import Tsdp
    wl = ti.WORKLOADS[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.calibrate:
        for hs in (1.0, 0.5, 0.35, 0.25, 0.18, 0.12, 0.08):
            CALIBRATED_HEAD_SCALE[wl.name] = hs
            wb, wd, cond, x, t0, K, s = make_problem(wl, "calibrated")
            ctx = Tsdp.from_workload(wl)
            ctx.tsdp_load_weights(0, ti.pack_blob(wb)); ctx.tsdp_load_weights(1, ti.pack_blob(wd))
            ctx.tsdp_set_cond(torch.from_numpy(cond).to(dev))
            xd, td = torch.from_numpy(x).to(dev), torch.from_numpy(t0).to(dev)
            na = torch.zeros(wl.B, dtype=torch.int32, device=dev); nd = torch.zeros_like(na)
            ctx.tsdp_round(xd, td, torch.from_numpy(K).to(dev), torch.from_numpy(s).to(dev), None, na, nd)
            keff = np.minimum(K, np.maximum(t0, 0))
            tested = np.minimum(na.cpu().numpy() + 1, keff).sum()      # drafts examined up to the first rejection
            print(f"head_scale {hs}: accepted/tested = {na.sum().item() / tested:.3f}, "
                  f"accepted/drafted = {na.sum().item() / keff.sum():.3f}, steps/round/env = {nd.float().mean().item():.2f}")
            ctx.close()
        return

    wb, wd, cond, x, t0, K, s = make_problem(wl, args.point)
    ctx = Tsdp.from_workload(wl)
    ctx.tsdp_load_weights(0, ti.pack_blob(wb)); ctx.tsdp_load_weights(1, ti.pack_blob(wd))
    ctx.tsdp_set_cond(torch.from_numpy(cond).to(dev))
    x0d, t0d = torch.from_numpy(x).to(dev), torch.from_numpy(t0).to(dev)
    Kd, sd = torch.from_numpy(K).to(dev), torch.from_numpy(s).to(dev)
    xd, td = x0d.clone(), t0d.clone()
    nacc = torch.zeros(wl.B, dtype=torch.int32, device=dev); nadv = torch.zeros_like(nacc)

    def step():
        xd.copy_(x0d); td.copy_(t0d)                 # every step runs the same round (fixed work per step)
        ctx.tsdp_round(xd, td, Kd, sd, None, nacc, nadv)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    fused = "mfma-fused" in ctx.path_name(0)
    if fused:
        ctx.tsdp_kernel_timing(True)                 # one event pair per stage and step, on the launch stream
    tic = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - tic
    last_verify_kernel_ms = ctx.tsdp_kernel_ms(1) if fused else None
    ctx.tsdp_kernel_timing(False)
    adv = int(nadv.sum().item()); acc = int(nacc.sum().item())
    keff = np.minimum(K, np.maximum(t0, 0))
    tested = int(np.minimum(nacc.cpu().numpy() + 1, keff).sum())
    R = int(np.where(t0 >= 0, np.maximum(keff, 1), 0).sum())
    ms_step = 1e3 * wall / args.steps

    # stage timings with HIP events on the launch stream
    rows = ctx.alloc_rows(wl.B)
    ctx.tsdp_draft(x0d, t0d, Kd, sd, None, rows)
    ctx.tsdp_verify(wl.B, rows)
    out = ctx.tsdp_accept(wl.B, sd, None, rows, diagnostics=False)
    n_it = max(10, min(100, args.steps))
    t_draft = time_events(lambda: ctx.tsdp_draft(x0d, t0d, Kd, sd, None, rows), n_it, torch)
    t_verify = time_events(lambda: ctx.tsdp_verify(wl.B, rows), n_it, torch)
    t_accept = time_events(lambda: ctx.tsdp_accept_into(wl.B, sd, None, rows, out), n_it, torch)
    t_round = time_events(step, n_it, torch)

    # the same step replayed from a captured HIP graph (a round is a fixed launch sequence: no allocation, no host
    # synchronisation): what launch overhead costs at the small workloads
    ctx.tsdp_kernel_timing(False)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    graph.replay()
    t_graph = time_events(graph.replay, n_it, torch)

    flops = verify_flops(wl, R)
    bf16 = wl.dtype == "bf16"
    if fused:
        k_ms, k_med = time_kernel(ctx, lambda: ctx.tsdp_verify(wl.B, rows), 1, n_it)
        kd_ms, _ = time_kernel(ctx, lambda: ctx.tsdp_draft(x0d, t0d, Kd, sd, None, rows), 0, n_it)
        kname = "k_fused_forward (verify forward, all layers in one launch)"
    else:
        k_ms, k_med, kd_ms, kname = t_verify[0], t_verify[1], None, "tsdp_verify (sequence of fp32 operator kernels)"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS    # fp32 networks: fp32 MFMA / vector peak
    achieved = flops / (k_ms * 1e-3) / 1e12
    res = {
        "metric": "accepted denoising steps/s on 1 GPU", "value": adv * args.steps / wall,
        "unit": "accepted denoising steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "batch_envs": wl.B, "horizon": wl.H, "action_dim": wl.A,
                   "K_max": wl.K_max, "verify_rows": R, "operating_point": args.point,
                   "base": f"{wl.base.layers}L d{wl.base.d} h{wl.base.heads}",
                   "drafter": f"{wl.draft.layers}L d{wl.draft.d}", "T": wl.T,
                   "cond": "vector+FiLM" if wl.cond_mode == 0 else f"{wl.cond_tokens} tokens x {wl.cond_dim} cross-attention",
                   "paths": {"base": ctx.path_name(0), "drafter": ctx.path_name(1)}},
        "round": {"steps_advanced_per_round": adv, "accepted_drafts_per_round": acc, "drafts_per_round": int(keff.sum()),
                  "acceptance_of_tested_drafts": acc / max(tested, 1), "acceptance_of_all_drafts": acc / max(int(keff.sum()), 1),
                  "rounds_per_s": args.steps / wall, "accepted_drafts_per_s": acc * args.steps / wall},
        "latency_ms": {"round": {"mean": t_round[0], "p50": t_round[1], "p95": t_round[2]},
                       "draft": {"mean": t_draft[0], "p50": t_draft[1], "p95": t_draft[2]},
                       "verify": {"mean": t_verify[0], "p50": t_verify[1], "p95": t_verify[2]},
                       "accept": {"mean": t_accept[0], "p50": t_accept[1], "p95": t_accept[2]},
                       "round_from_hip_graph": {"mean": t_graph[0], "p50": t_graph[1], "p95": t_graph[2]},
                       "drafter_kernel": kd_ms},
        "roofline": {"kernel": kname, "bound": "mfma" if (bf16 or fused) else "alu", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name) if fused else None, "kernel_ms": k_ms,
                     "kernel_ms_median": k_med, "kernel_ms_last_timed_step": last_verify_kernel_ms,
                     "algorithmic_flops_per_launch": flops},
    }
    if not args.no_chain:
        # whole action prediction: every environment from t = T-1 down to the clean action (tsdp_chain)
        tT = torch.full((wl.B,), wl.T - 1, dtype=torch.int32, device=dev)
        xc, tc = x0d.clone(), tT.clone()
        ctx.tsdp_chain(xc, tc, Kd, sd, None, check_every=4, totals=False)          # warm-up
        xc, tc = x0d.clone(), tT.clone()
        torch.cuda.synchronize(); tic = time.perf_counter()
        n_rounds, tot = ctx.tsdp_chain(xc, tc, Kd, sd, None, check_every=4)
        torch.cuda.synchronize(); el = time.perf_counter() - tic
        a, d, r = (float(tot[k].float().mean().item()) for k in ("accept", "drafts", "rounds"))
        res["chain"] = {"denoising_steps": wl.T, "rounds_enqueued": n_rounds, "seconds": el,
                        "action_predictions_per_s": wl.B / el, "denoising_steps_per_s": wl.B * wl.T / el,
                        "latency_ms_per_action_prediction": 1e3 * el,
                        "mean_rounds_per_env": r, "mean_drafts_per_env": d, "mean_accepted_drafts_per_env": a,
                        "acceptance_of_all_drafts": a / max(d, 1e-9),
                        # paper's convention: a drafter call costs (drafter blocks / base blocks) of a base call
                        "nfe_fraction_of_plain_chain": (r + d * wl.draft.layers / wl.base.layers) / wl.T}
        # the same chain with a three-stage draft count (the scheduler's hook): one draft per round while the
        # noise is high and acceptance is nil, the full count in the middle, half of it for the last steps
        K3 = np.tile(np.array([1, wl.K_max, max(1, wl.K_max // 2)], dtype=np.int32), (wl.B, 1))
        s3 = np.repeat(s.astype(np.float32)[:, None], 3, axis=1)
        K3d, s3d = torch.from_numpy(K3).to(dev), torch.from_numpy(np.ascontiguousarray(s3)).to(dev)
        t_hi, t_lo = 9 * wl.T // 10, min(wl.K_max, wl.T // 4)
        xc, tc = x0d.clone(), tT.clone()
        ctx.tsdp_chain_staged(xc, tc, K3d, s3d, None, t_hi, t_lo, None, check_every=4, totals=False)
        xc, tc = x0d.clone(), tT.clone()
        torch.cuda.synchronize(); tic = time.perf_counter()
        n_rounds, tot = ctx.tsdp_chain_staged(xc, tc, K3d, s3d, None, t_hi, t_lo, None, check_every=4)
        torch.cuda.synchronize(); el = time.perf_counter() - tic
        a, d, r = (float(tot[k].float().mean().item()) for k in ("accept", "drafts", "rounds"))
        res["chain_staged"] = {"K_by_stage": [1, wl.K_max, max(1, wl.K_max // 2)], "stage_bounds": [t_hi, t_lo],
                               "rounds_enqueued": n_rounds, "seconds": el, "action_predictions_per_s": wl.B / el,
                               "denoising_steps_per_s": wl.B * wl.T / el, "mean_rounds_per_env": r,
                               "mean_drafts_per_env": d, "acceptance_of_all_drafts": a / max(d, 1e-9),
                               "nfe_fraction_of_plain_chain": (r + d * wl.draft.layers / wl.base.layers) / wl.T}
    if not args.no_accept_xl:
        res["accept_roofline"] = accept_xl(torch, Tsdp, dev)
    if not args.no_cpu:
        n_env = args.cpu_envs or {"C1": 1, "C2": 1, "C3": 4, "C4": 1, "C5": 4}[wl.name]
        res["cpu_baseline"] = cpu_baseline(wl, wb, wd, cond, x, t0, K, s, n_env)
    if not args.no_points and args.point == "calibrated":
        res["operating_points"] = operating_points(ctx, wl, torch, dev, t_round[0])
    print(json.dumps(res))
    ctx.close()
    if args.pmc_copy:
        a = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()


if __name__ == "__main__":
    main()
