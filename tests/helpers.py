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


# Latents (states, final actions): elementwise |got - ref| <= atol + rtol |ref| with the stated rtol (1e-5 for fp32
# networks, 2e-2 for bf16 networks).  An element near zero is a sum of terms of the tensor's scale and carries their
# absolute rounding error, which no relative bound covers: atol = a few rounding units u of the network's
# matrix-multiply inputs at the tensor's scale max |ref| -- fp32: 16 u, u = 2^-24 (9.5e-7 of scale); bf16: 4 u,
# u = 2^-9 (7.8e-3 of scale; a posterior mean amplifies the noise prediction's error by up to c0 sqrt(1-abar)/sqrt(abar),
# about 30 at the first steps of the squared-cosine schedule).
RTOL = {"fp32": 1e-5, "bf16": 2e-2}
ATOL_OF_SCALE = {"fp32": 16 * 2.0 ** -24, "bf16": 4 * 2.0 ** -9}


def assert_latents_close(got, ref, dtype, what=""):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rtol = RTOL[dtype]
    atol = ATOL_OF_SCALE[dtype] * float(np.abs(ref).max())
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    worst = float((err / bound).max())
    assert worst <= 1.0, f"{what}: elementwise error {worst:.3f}x the bound (rtol {rtol}, atol {atol:.3e})"
    return worst


def drafted_rows(row_ptr, row_t, bonus=False):
    """Mask of the rows that hold a drafted transition (a row at timestep 0, and with the bonus row the last row of
    every environment, is a step of the base model itself: it is not tested and has no margin)."""
    row_ptr = np.asarray(row_ptr); row_t = np.asarray(row_t)
    m = row_t[:int(row_ptr[-1])] > 0
    if bonus:
        last = row_ptr[1:][np.diff(row_ptr) > 0] - 1
        m[last] = False
    return m


def list_near_ties(tag, logu, logratio, row_ptr, window, drafted=None):
    """Rows whose accept decision is within `window` of a tie: printed (never hidden), returned as a row mask."""
    margin = np.abs(np.asarray(logu) - np.asarray(logratio))
    near = margin < window
    if drafted is not None:
        near &= drafted
    for r in np.nonzero(near)[0]:
        b = int(np.searchsorted(row_ptr, r, side="right") - 1)
        print(f"[{tag}] near-tie row {int(r)} (env {b}, draft {int(r - row_ptr[b]) + 1}): |log U - log alpha| = {margin[r]:.3e}")
    return near
