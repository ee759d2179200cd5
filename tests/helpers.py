"""Shared plumbing of the GPU parity tests: builds the oracle objects and the library context for a
workload from the same seeded inputs."""
import numpy as np

import tsdp_inputs as ti
from oracle.ddpm import Schedule
from oracle.denoiser import Denoiser


def oracle_side(wl, wb, wd, clip=None, sampler=0, eta=1.0, norm=0):
    bf16 = wl.dtype == "bf16"
    base = Denoiser(wb, wl.base.layers, wl.base.heads, wl.cond_mode, bf16, norm)
    drafter = Denoiser(wd, wl.draft.layers, wl.draft.heads, wl.cond_mode, bf16, norm)
    sched = Schedule(wl.T, wl.schedule, wl.beta0 or 1e-4, wl.beta1 or 0.02, sampler=sampler, eta=eta)
    return base, drafter, sched


def gpu_side(wl, wb, wd, cond, clip=None, B_max=None, K_max=None, seed=None, sampler=0, eta=1.0, bonus_row=False, norm=0):
    import torch
    from paper_2512_15773_amd import Tsdp
    ctx = Tsdp.from_workload(wl, B_max=B_max, K_max=K_max, clip=clip, seed=seed, sampler=sampler, eta=eta, bonus_row=bonus_row,
                             norm=norm)
    ctx.tsdp_load_weights(0, ti.pack_blob(wb))
    ctx.tsdp_load_weights(1, ti.pack_blob(wd))
    ctx.tsdp_set_cond(torch.from_numpy(cond).cuda())
    return ctx


def to_dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def scaled_err(got, ref):
    """max |got - ref| / max |ref|: error relative to the tensor's scale."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))
