"""Seeded synthetic inputs for the speculative denoising round (shared by the
CPU oracle's tests and by the HIP path's tests and benchmark).

This module holds shapes and random draws only: no DDPM formula, no network
forward, no acceptance arithmetic and no Philox stream of the method lives
here.  Everything is produced by numpy's PCG64 generator from explicit seeds,
so the oracle and the GPU library receive bit-identical fp32 arrays.

The five workloads stand in for the robot benchmarks of the paper's Section 4
(Robomimic, Push-T, Block-Push, Kitchen), whose data and trained checkpoints
are not available: the shapes follow Diffusion-Policy style action chunks
(horizon 16/32, action_dim 2..14, 100-step DDPM) and the weights are random
N(0, w_std) draws.
"""
from __future__ import annotations

from collections import OrderedDict
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class NetShape:
    layers: int
    d: int
    heads: int
    mlp_ratio: int = 4


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str              # "fp32" | "bf16" : precision of the network internals
    B: int                  # environments in one batch
    H: int                  # action horizon (tokens per latent)
    A: int                  # action dimension
    cond_mode: int          # 0 = conditioning vector (FiLM), 1 = observation tokens (cross-attn)
    cond_dim: int           # vector length (mode 0) or per-token feature size (mode 1)
    cond_tokens: int        # 0 (mode 0) or number of observation tokens (mode 1)
    base: NetShape
    draft: NetShape
    T: int                  # DDPM steps
    schedule: int           # 0 linear(beta0, beta1), 1 squared-cosine
    beta0: float
    beta1: float
    K_max: int              # largest draft count in the batch
    ragged: bool            # per-env K, sigma_scale and t0 drawn at random (adaptive-scheduler case)
    philox_seed: int
    weight_seed: int

    @property
    def D(self) -> int:
        return self.H * self.A


C1 = Workload("C1", "fp32", 1, 16, 2, 0, 64, 0, NetShape(2, 64, 2), NetShape(1, 32, 2),
              10, 0, 1e-4, 0.02, 4, False, 0, 101)
C2 = Workload("C2", "fp32", 1, 16, 10, 0, 1024, 0, NetShape(8, 256, 4), NetShape(2, 128, 4),
              100, 1, 0.0, 0.0, 8, False, 2, 202)
C3 = replace(C2, name="C3", dtype="bf16", B=64, K_max=16, philox_seed=3, weight_seed=303)
C4 = Workload("C4", "bf16", 256, 32, 14, 1, 768, 64, NetShape(12, 512, 8), NetShape(2, 256, 8),
              100, 1, 0.0, 0.0, 8, False, 4, 404)
C5 = Workload("C5", "bf16", 1024, 16, 7, 0, 1024, 0, NetShape(8, 384, 6), NetShape(2, 192, 6),
              100, 1, 0.0, 0.0, 16, True, 5, 505)

WORKLOADS = {w.name: w for w in (C1, C2, C3, C4, C5)}


def weight_spec(wl: Workload, which: str) -> "OrderedDict[str, tuple]":
    """Canonical tensor list (name -> shape) of one denoiser, in blob order.

    Linear weights are [out_features, in_features] row-major, as in the usual
    y = x W^T + b convention.  `which` is "base" or "draft".
    """
    net = wl.base if which == "base" else wl.draft
    d, m = net.d, net.mlp_ratio * net.d
    spec: "OrderedDict[str, tuple]" = OrderedDict()
    spec["tok_w"] = (d, wl.A); spec["tok_b"] = (d,); spec["pos"] = (wl.H, d)
    spec["t_w1"] = (d, d); spec["t_b1"] = (d,); spec["t_w2"] = (d, d); spec["t_b2"] = (d,)
    if wl.cond_mode == 0:
        spec["c_w"] = (d, wl.cond_dim); spec["c_b"] = (d,)
    for l in range(net.layers):
        p = f"l{l}."
        spec[p + "mod_w"] = (4 * d, d); spec[p + "mod_b"] = (4 * d,)
        spec[p + "qkv_w"] = (3 * d, d); spec[p + "qkv_b"] = (3 * d,)
        spec[p + "o_w"] = (d, d); spec[p + "o_b"] = (d,)
        if wl.cond_mode == 1:
            spec[p + "cq_w"] = (d, d); spec[p + "cq_b"] = (d,)
            spec[p + "ck_w"] = (d, wl.cond_dim); spec[p + "ck_b"] = (d,)
            spec[p + "cv_w"] = (d, wl.cond_dim); spec[p + "cv_b"] = (d,)
            spec[p + "co_w"] = (d, d); spec[p + "co_b"] = (d,)
        spec[p + "up_w"] = (m, d); spec[p + "up_b"] = (m,)
        spec[p + "dn_w"] = (d, m); spec[p + "dn_b"] = (d,)
    spec["head_w"] = (wl.A, d); spec["head_b"] = (wl.A,)
    return spec


def make_weights(wl: Workload, which: str, seed: int | None = None, w_std: float = 0.02,
                 b_std: float = 0.0, head_scale: float = 1.0) -> "OrderedDict[str, np.ndarray]":
    """Random-init weights ~N(0, w_std), biases ~N(0, b_std) (0 -> exactly zero), fp32.

    `head_scale` multiplies the output projection (weight and bias); it is the
    single calibration knob used to move the draft acceptance rate of the
    synthetic pair (base, drafter) towards the rate the paper tabulates.
    """
    if seed is None:
        seed = wl.weight_seed + (0 if which == "base" else 1)
    rng = np.random.default_rng(seed)
    out: "OrderedDict[str, np.ndarray]" = OrderedDict()
    for name, shape in weight_spec(wl, which).items():
        is_bias = name.endswith("_b")
        std = b_std if is_bias else w_std
        if std == 0.0:
            a = np.zeros(shape, dtype=np.float32)
        else:
            a = (rng.standard_normal(shape) * std).astype(np.float32)
        if name in ("head_w", "head_b"):
            a = (a * np.float32(head_scale)).astype(np.float32)
        out[name] = a
    return out


def pack_blob(weights: "OrderedDict[str, np.ndarray]") -> np.ndarray:
    """Flat fp32 blob: the tensors of `weight_spec` concatenated in order."""
    return np.concatenate([np.ascontiguousarray(a, dtype=np.float32).ravel() for a in weights.values()])


def make_cond(wl: Workload, B: int | None = None, seed: int = 7) -> np.ndarray:
    """Observation conditioning ~N(0,1): [B, cond_dim] or [B, cond_tokens, cond_dim], fp32."""
    B = wl.B if B is None else B
    rng = np.random.default_rng(seed + 1000 * wl.weight_seed)
    shape = (B, wl.cond_dim) if wl.cond_mode == 0 else (B, wl.cond_tokens, wl.cond_dim)
    return rng.standard_normal(shape).astype(np.float32)


def make_latents(wl: Workload, B: int | None = None, seed: int = 11) -> np.ndarray:
    """Initial action latents ~N(0, I): [B, H, A] fp32."""
    B = wl.B if B is None else B
    rng = np.random.default_rng(seed + 1000 * wl.weight_seed)
    return rng.standard_normal((B, wl.H, wl.A)).astype(np.float32)


def make_schedule_inputs(wl: Workload, B: int | None = None, seed: int = 13, t0: int | None = None):
    """Per-env scheduler outputs (t0, K, sigma_scale), which the round takes as inputs.

    Fixed workloads: K = K_max, sigma_scale = 1, t0 = the given value (default T-1).
    Ragged workload (adaptive-scheduler stress case): K ~ U{2..K_max},
    sigma_scale ~ U[1, 1.5], t0 ~ U{0..T-1}, each per environment.
    """
    B = wl.B if B is None else B
    rng = np.random.default_rng(seed + 1000 * wl.weight_seed)
    if wl.ragged and t0 is None:
        K = rng.integers(2, wl.K_max + 1, size=B).astype(np.int32)
        s = rng.uniform(1.0, 1.5, size=B).astype(np.float32)
        t = rng.integers(0, wl.T, size=B).astype(np.int32)
    else:
        K = np.full(B, wl.K_max, dtype=np.int32)
        s = np.ones(B, dtype=np.float32)
        t = np.full(B, wl.T - 1 if t0 is None else t0, dtype=np.int32)
    return t, K, s


def small_variant(wl: Workload, **kw) -> Workload:
    """A reduced copy of a workload (fewer envs / layers) for tests the CPU oracle finishes quickly."""
    return replace(wl, **kw)
