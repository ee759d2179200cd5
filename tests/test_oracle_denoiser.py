"""Pins of the oracle's Transformer against torch CPU library routines in fp64 (no GPU)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import tsdp_inputs as ti
from oracle import denoiser as dn


def _t(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def test_blocks_against_torch():
    rng = np.random.default_rng(0)
    h = rng.standard_normal((3, 16, 64))
    np.testing.assert_allclose(dn.layer_norm(h), F.layer_norm(_t(h), (64,), eps=1e-5).numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dn.rms_norm(h), F.rms_norm(_t(h), (64,), eps=1e-5).numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dn.gelu_tanh(h), F.gelu(_t(h), approximate="tanh").numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dn.silu(h), F.silu(_t(h)).numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dn.softmax(h), F.softmax(_t(h), dim=-1).numpy(), rtol=1e-12)
    q, k, v = rng.standard_normal((3, 2, 16, 64)), rng.standard_normal((3, 2, 9, 64)), rng.standard_normal((3, 2, 9, 64))
    for heads in (1, 2, 4):
        def split(a):
            return _t(a).reshape(2, a.shape[1], heads, 64 // heads).transpose(1, 2)
        ref = F.scaled_dot_product_attention(split(q[0]), split(k[0]), split(v[0]))
        ref = ref.transpose(1, 2).reshape(2, 16, 64).numpy()
        np.testing.assert_allclose(dn.attention(q[0], k[0], v[0], heads), ref, rtol=1e-10, atol=1e-12)


def test_sinusoid_layout():
    e = dn.sinusoid(np.array([0, 1, 37]), 8)
    f = 10000.0 ** (-np.arange(4) / 4)
    np.testing.assert_allclose(e[0], [0, 0, 0, 0, 1, 1, 1, 1], atol=1e-15)
    np.testing.assert_allclose(e[2], np.concatenate([np.sin(37 * f), np.cos(37 * f)]), rtol=1e-12)


def _torch_forward(w, net, cond_mode, x, t, cond, norm=0):
    """The same network composed only of torch.nn.functional calls (independent composition)."""
    w = {k: _t(v) for k, v in w.items()}
    d, nh = net.d, net.heads
    x, cond = _t(x), _t(cond)
    R, H, _ = x.shape
    LN = (lambda a: F.rms_norm(a, (d,), eps=1e-5)) if norm == 1 else (lambda a: F.layer_norm(a, (d,), eps=1e-5))

    def mha(q, k, v):
        sp = lambda a: a.reshape(R, a.shape[1], nh, d // nh).transpose(1, 2)
        return F.scaled_dot_product_attention(sp(q), sp(k), sp(v)).transpose(1, 2).reshape(R, q.shape[1], d)

    half = d // 2
    fr = torch.exp(-np.log(10000.0) * torch.arange(half, dtype=torch.float64) / half)
    ang = _t(t)[:, None] * fr[None]
    temb = F.linear(F.silu(F.linear(torch.cat([ang.sin(), ang.cos()], 1), w["t_w1"], w["t_b1"])), w["t_w2"], w["t_b2"])
    g = temb + F.linear(cond, w["c_w"], w["c_b"]) if cond_mode == 0 else temb
    h = F.linear(x, w["tok_w"], w["tok_b"]) + w["pos"]
    for l in range(net.layers):
        p = f"l{l}."
        g1, b1, g2, b2 = F.linear(F.silu(g), w[p + "mod_w"], w[p + "mod_b"]).chunk(4, dim=-1)
        a = LN(h) * (1 + g1[:, None]) + b1[:, None]
        q, k, v = F.linear(a, w[p + "qkv_w"], w[p + "qkv_b"]).chunk(3, dim=-1)
        h = h + F.linear(mha(q, k, v), w[p + "o_w"], w[p + "o_b"])
        if cond_mode == 1:
            h = h + F.linear(mha(F.linear(LN(h), w[p + "cq_w"], w[p + "cq_b"]),
                                 F.linear(cond, w[p + "ck_w"], w[p + "ck_b"]),
                                 F.linear(cond, w[p + "cv_w"], w[p + "cv_b"])), w[p + "co_w"], w[p + "co_b"])
        a = LN(h) * (1 + g2[:, None]) + b2[:, None]
        h = h + F.linear(F.gelu(F.linear(a, w[p + "up_w"], w[p + "up_b"]), approximate="tanh"), w[p + "dn_w"], w[p + "dn_b"])
    return F.linear(LN(h), w["head_w"], w["head_b"]).numpy()


@pytest.mark.parametrize("wl", [ti.C1, ti.small_variant(ti.C4, base=ti.NetShape(2, 64, 4), cond_dim=24, cond_tokens=5, H=8, A=3)])
def test_forward_against_torch_composition(wl):
    w = ti.make_weights(wl, "base", w_std=0.2, b_std=0.1)             # large weights: every path matters
    net = dn.Denoiser(w, wl.base.layers, wl.base.heads, wl.cond_mode)
    R = 5
    x = ti.make_latents(wl, R); cond = ti.make_cond(wl, R); t = np.array([0, 1, 5, 9, 3]) % wl.T
    out = net(x, t, cond)
    ref = _torch_forward(w, wl.base, wl.cond_mode, x, t, cond)
    assert out.shape == (R, wl.H, wl.A)
    np.testing.assert_allclose(out, ref, rtol=1e-9, atol=1e-11)
    # rows are independent: row-by-row evaluation and a permutation of rows give the same rows
    perm = np.array([3, 0, 4, 1, 2])
    np.testing.assert_allclose(net(x[perm], t[perm], cond[perm]), out[perm], rtol=1e-10, atol=1e-12)
    for r in range(R):
        np.testing.assert_allclose(net(x[r:r + 1], t[r:r + 1], cond[r:r + 1])[0], out[r], rtol=1e-10, atol=1e-12)
    # every input matters: timestep, conditioning, latent
    assert np.abs(net(x, (t + 1) % wl.T, cond) - out).max() > 1e-3
    assert np.abs(net(x, t, cond[::-1]) - out).max() > 1e-3
    # the RMSNorm alternative: same composition with torch's rms_norm, and a different function
    rms = dn.Denoiser(w, wl.base.layers, wl.base.heads, wl.cond_mode, norm=1)
    np.testing.assert_allclose(rms(x, t, cond), _torch_forward(w, wl.base, wl.cond_mode, x, t, cond, norm=1), rtol=1e-9, atol=1e-11)
    assert np.abs(rms(x, t, cond) - out).max() > 1e-3


def test_bf16_rounding_is_round_to_nearest_even():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.1415927, 1e-30], dtype=np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(dn.round_bf16(a), ref)
    assert dn.round_bf16(a)[1] == 1.0 and dn.round_bf16(a)[3] == np.float32(1.0 + 2 ** -6)   # ties to even
    rnd = np.random.default_rng(1).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(dn.round_bf16(rnd), torch.from_numpy(rnd).to(torch.bfloat16).float().numpy())
