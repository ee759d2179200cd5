"""Philox4x32-10 counter-based generator and the method's noise streams (oracle).

Philox4x32-10 is the public algorithm of Salmon et al., "Parallel random
numbers: as easy as 1, 2, 3" (SC'11): ten rounds of two 32x32->64 multiplies
with a Weyl key schedule.  The paper only requires independent U_j ~ Unif(0,1)
(Section 3.1, first-rejection index) and xi_i ~ N(0, I) (Section 3.2, log
acceptance ratio) and says the noise realisations of the rollout are retained;
the stream layout below is this implementation's reading:

  key     = (seed low 32 bits, seed high 32 bits)
  counter = (block index i, timestep t, global environment id, stream id)
  stream 0: Gaussian noise xi_{env,t}; block i yields elements 4i .. 4i+3
  stream 1: the acceptance uniform U_{env,t} (block 0, word 0)

  uniform: u = ((w >> 9) + 0.5) * 2^-23  in (0, 1); 24 significant bits, exact in fp32
  normals: Box-Muller on word pairs (w0,w1) and (w2,w3):
           r = sqrt(-2 ln u_a), (r cos 2 pi u_b, r sin 2 pi u_b)
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: [..., 4] uint32, key: [..., 2] uint32 (broadcastable) -> [..., 4] uint32."""
    c = np.asarray(counter, dtype=np.uint64)
    k = np.asarray(key, dtype=np.uint64)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = k[..., 0], k[..., 1]
    for rnd in range(10):
        p0 = _M0 * c0                      # 64-bit products of 32-bit values
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK, lo1, (hi0 ^ c3 ^ k1) & _MASK, lo0
        k0 = (k0 + np.uint64(_W0)) & _MASK
        k1 = (k1 + np.uint64(_W1)) & _MASK
    return np.stack(np.broadcast_arrays(c0, c1, c2, c3), axis=-1).astype(np.uint32)


def _key(seed):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint32)


def u01(w):
    """Uniform strictly inside (0,1) from the top 23 bits; exactly representable in fp32."""
    return ((np.asarray(w, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def normal(seed, env, t, D):
    """xi_{env,t}: [n, D] fp64 standard normals for n (env, t) pairs (stream 0)."""
    env = np.atleast_1d(np.asarray(env, dtype=np.int64))
    t = np.atleast_1d(np.asarray(t, dtype=np.int64))
    n = env.shape[0]
    nb = (D + 3) // 4
    ctr = np.zeros((n, nb, 4), dtype=np.uint32)
    ctr[..., 0] = np.arange(nb, dtype=np.uint32)[None, :]
    ctr[..., 1] = t.astype(np.uint32)[:, None]
    ctr[..., 2] = env.astype(np.uint32)[:, None]
    ctr[..., 3] = 0
    w = philox4x32_10(ctr, _key(seed))
    u = u01(w)
    out = np.empty((n, nb, 4), dtype=np.float64)
    for a in (0, 2):
        r = np.sqrt(-2.0 * np.log(u[..., a]))
        th = 2.0 * np.pi * u[..., a + 1]
        out[..., a] = r * np.cos(th)
        out[..., a + 1] = r * np.sin(th)
    return out.reshape(n, nb * 4)[:, :D]


def uniform(seed, env, t):
    """U_{env,t}: [n] fp64 uniforms in (0,1) (stream 1)."""
    env = np.atleast_1d(np.asarray(env, dtype=np.int64))
    t = np.atleast_1d(np.asarray(t, dtype=np.int64))
    ctr = np.zeros((env.shape[0], 4), dtype=np.uint32)
    ctr[:, 1] = t.astype(np.uint32)
    ctr[:, 2] = env.astype(np.uint32)
    ctr[:, 3] = 1
    return u01(philox4x32_10(ctr, _key(seed))[:, 0])
