"""Noise-prediction Transformer of the Diffusion Policy and of its drafter (oracle, fp64).

The paper states only that the base policy has 8 Transformer blocks, that the
drafter is a single Transformer block with the same input/output interface,
and that both share the observation encoder and the DDPM scheduler (Section
3.2, Draft Model Training; Section 4, Experiment Settings).  The architecture
below is this implementation's definition, built from standard parts:

  tokens    h = x W_tok^T + b_tok + pos                      x: [R, H, A]
  time      temb = W_t2 SiLU(W_t1 sinus(t) + b_t1) + b_t2   sinus = [sin(t f_i), cos(t f_i)],
                                                             f_i = 10000^(-i/(d/2)), i < d/2
  cond      mode 0 (vector): g = temb + W_c c + b_c ; mode 1 (tokens): g = temb
  per layer (g1, b1, g2, b2) = split4(W_mod SiLU(g) + b_mod)             (FiLM / adaLN)
            h += W_o  SelfAttn(W_qkv (LN(h) (1 + g1) + b1))              (non-causal, scale 1/sqrt(d_head))
            mode 1: h += W_co CrossAttn(W_cq LN(h); W_ck obs, W_cv obs)
            h += W_dn GELU_tanh(W_up (LN(h) (1 + g2) + b2))
  head      eps = W_head LN(h) + b_head
  LN = LayerNorm over d without affine parameters, eps = 1e-5.

In bf16 mode the weights are rounded to bfloat16 (round to nearest even)
before use; the arithmetic stays fp64 (the GPU rounds activations to bf16 at
matrix-multiply inputs as well, which the bf16 tolerance covers).
"""
import numpy as np


def round_bf16(a):
    """fp32 -> bfloat16 (round to nearest even) -> fp32, on the bit pattern."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = a.view(np.uint32).astype(np.uint64)
    b = (b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return b.astype(np.uint32).view(np.float32).reshape(a.shape)


def layer_norm(h, eps=1e-5):
    mu = h.mean(axis=-1, keepdims=True)
    var = ((h - mu) ** 2).mean(axis=-1, keepdims=True)
    return (h - mu) / np.sqrt(var + eps)


def rms_norm(h, eps=1e-5):
    """x / sqrt(mean(x^2) + eps), no affine parameters (the configurable alternative to layer_norm)."""
    return h / np.sqrt((h ** 2).mean(axis=-1, keepdims=True) + eps)


def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def softmax(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, heads):
    """q: [R, Hq, d], k, v: [R, Hk, d] -> [R, Hq, d]; softmax(q k^T / sqrt(d_head)) v per head."""
    R, Hq, d = q.shape
    Hk = k.shape[1]
    dh = d // heads
    qh = q.reshape(R, Hq, heads, dh).transpose(0, 2, 1, 3)
    kh = k.reshape(R, Hk, heads, dh).transpose(0, 2, 1, 3)
    vh = v.reshape(R, Hk, heads, dh).transpose(0, 2, 1, 3)
    p = softmax(np.matmul(qh, kh.transpose(0, 1, 3, 2)) / np.sqrt(dh))
    return np.matmul(p, vh).transpose(0, 2, 1, 3).reshape(R, Hq, d)


def sinusoid(t, d):
    half = d // 2
    f = np.exp(-np.log(10000.0) * np.arange(half, dtype=np.float64) / half)
    a = np.asarray(t, dtype=np.float64)[:, None] * f[None, :]
    return np.concatenate([np.sin(a), np.cos(a)], axis=1)


class Denoiser:
    """eps = M(x; t, cond) for a batch of independent rows."""

    def __init__(self, weights, layers, heads, cond_mode, bf16=False, norm=0):
        cvt = (lambda a: round_bf16(a).astype(np.float64)) if bf16 else (lambda a: np.asarray(a, np.float64))
        self.w = {k: cvt(v) for k, v in weights.items()}
        self.layers, self.heads, self.cond_mode = layers, heads, cond_mode
        self.norm = rms_norm if norm == 1 else layer_norm        # 0 = LayerNorm, 1 = RMSNorm
        self.d = self.w["tok_w"].shape[0]

    def __call__(self, x, t, cond):
        """x: [R, H, A]; t: [R] int; cond: [R, C] (mode 0) or [R, S, Cdim] (mode 1) -> eps [R, H, A]."""
        w = self.w
        x = np.asarray(x, dtype=np.float64)
        cond = np.asarray(cond, dtype=np.float64)
        lin = lambda a, name: a @ w[name + "_w"].T + w[name + "_b"]
        h = lin(x, "tok") + w["pos"][None]
        temb = silu(sinusoid(t, self.d) @ w["t_w1"].T + w["t_b1"]) @ w["t_w2"].T + w["t_b2"]
        g = temb + (cond @ w["c_w"].T + w["c_b"]) if self.cond_mode == 0 else temb
        sg = silu(g)
        for l in range(self.layers):
            p = f"l{l}."
            g1, b1, g2, b2 = np.split(lin(sg, p + "mod"), 4, axis=-1)
            a = self.norm(h) * (1.0 + g1[:, None, :]) + b1[:, None, :]
            q, k, v = np.split(lin(a, p + "qkv"), 3, axis=-1)
            h = h + lin(attention(q, k, v, self.heads), p + "o")
            if self.cond_mode == 1:
                qc = lin(self.norm(h), p + "cq")
                h = h + lin(attention(qc, lin(cond, p + "ck"), lin(cond, p + "cv"), self.heads), p + "co")
            a = self.norm(h) * (1.0 + g2[:, None, :]) + b2[:, None, :]
            h = h + lin(gelu_tanh(lin(a, p + "up")), p + "dn")
        return lin(self.norm(h), "head")
