"""ctypes binding of libtsdp.so: argument marshalling only, every step runs in the HIP kernels.

torch is used for device memory and streams.  The library must have been built in-tree
(`python -m paper_2512_15773_amd.build` or `__graft_entry__.build()`); there is no fallback.

Calls only enqueue work on the given (default: torch's current) stream.  The binding passes raw pointers: a tensor
handed to a call must stay alive until that stream has run the call -- torch's caching allocator does not know of the
use and would hand a freed tensor's memory out again (keep a reference, or call Tensor.record_stream yourself).
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtsdp.so")

EXPORTS = ["tsdp_create", "tsdp_destroy", "tsdp_load_weights", "tsdp_set_cond", "tsdp_draft", "tsdp_verify",
           "tsdp_accept", "tsdp_round", "tsdp_accept_threshold", "tsdp_round_threshold", "tsdp_chain", "tsdp_chain_staged",
           "tsdp_chain_enqueue", "tsdp_prepare",
           "tsdp_distill_loss", "tsdp_distill_loss_noalloc", "tsdp_status", "tsdp_kernel_timing", "tsdp_kernel_ms", "tsdp_path_name",
           "tsdp_last_error"]


class TsdpConfig(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("H", C.c_int32), ("A", C.c_int32), ("cond_mode", C.c_int32),
                ("cond_dim", C.c_int32), ("cond_tokens", C.c_int32),
                ("base_layers", C.c_int32), ("base_d", C.c_int32), ("base_heads", C.c_int32), ("base_mlp_ratio", C.c_int32),
                ("draft_layers", C.c_int32), ("draft_d", C.c_int32), ("draft_heads", C.c_int32), ("draft_mlp_ratio", C.c_int32),
                ("T", C.c_int32), ("schedule", C.c_int32), ("beta0", C.c_float), ("beta1", C.c_float),
                ("clip_x0", C.c_int32), ("clip_val", C.c_float), ("B_max", C.c_int32), ("K_max", C.c_int32),
                ("seed", C.c_uint64), ("sampler", C.c_int32), ("eta", C.c_float),
                ("bonus_row", C.c_int32), ("norm", C.c_int32)]


_lib = None


def load_library():
    """Loads libtsdp.so and declares the prototypes; raises if the library has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_15773_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int
    lib.tsdp_create.argtypes = [C.POINTER(TsdpConfig), C.POINTER(vp)]
    lib.tsdp_destroy.argtypes = [vp]; lib.tsdp_destroy.restype = None
    lib.tsdp_load_weights.argtypes = [vp, i32, vp, C.c_size_t]
    lib.tsdp_set_cond.argtypes = [vp, vp, i32, vp]
    lib.tsdp_draft.argtypes = [vp, i32] + [vp] * 12 + [vp]
    lib.tsdp_verify.argtypes = [vp, i32, i32] + [vp] * 5 + [vp]
    lib.tsdp_accept.argtypes = [vp, i32] + [vp] * 16 + [vp]
    lib.tsdp_round.argtypes = [vp, i32] + [vp] * 7 + [vp]
    lib.tsdp_accept_threshold.argtypes = [vp, i32] + [vp] * 15 + [vp]
    lib.tsdp_round_threshold.argtypes = [vp, i32] + [vp] * 8 + [vp]
    lib.tsdp_chain.argtypes = [vp, i32] + [vp] * 6 + [i32, i32] + [vp] * 3 + [C.POINTER(C.c_int32), vp]
    lib.tsdp_chain_staged.argtypes = [vp, i32] + [vp] * 5 + [i32, i32, vp, i32, i32] + [vp] * 3 + [C.POINTER(C.c_int32), vp]
    lib.tsdp_chain_enqueue.argtypes = [vp, i32] + [vp] * 5 + [i32, i32, i32, vp, i32] + [vp] * 4 + [vp]
    lib.tsdp_prepare.argtypes = [vp]
    lib.tsdp_distill_loss.argtypes = [vp, i32, vp, vp, vp, vp, C.c_float, C.c_float, vp, vp]
    lib.tsdp_distill_loss_noalloc.argtypes = lib.tsdp_distill_loss.argtypes
    lib.tsdp_status.argtypes = [vp, vp, C.POINTER(C.c_int32)]
    lib.tsdp_kernel_timing.argtypes = [vp, i32]
    lib.tsdp_kernel_ms.argtypes = [vp, i32, C.POINTER(C.c_float)]
    lib.tsdp_path_name.argtypes = [vp, i32]; lib.tsdp_path_name.restype = C.c_char_p
    lib.tsdp_last_error.argtypes = [vp]; lib.tsdp_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if getattr(lib, name).restype is C.c_int:
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


class TsdpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"tsdp error {code}: {msg}")
        self.code = code


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return t.data_ptr()


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


class Tsdp:
    """One library context.  Methods carry the names of the C entry points."""

    def __init__(self, *, dtype, H, A, cond_mode, cond_dim, cond_tokens, base, draft, T, schedule,
                 beta0=1e-4, beta1=0.02, clip=None, B_max, K_max, seed, sampler=0, eta=1.0, bonus_row=False, norm=0):
        """base / draft: (layers, d, heads, mlp_ratio)."""
        self.lib = load_library()
        self.cfg = TsdpConfig(dtype=dtype, H=H, A=A, cond_mode=cond_mode, cond_dim=cond_dim, cond_tokens=cond_tokens,
                              base_layers=base[0], base_d=base[1], base_heads=base[2], base_mlp_ratio=base[3],
                              draft_layers=draft[0], draft_d=draft[1], draft_heads=draft[2], draft_mlp_ratio=draft[3],
                              T=T, schedule=schedule, beta0=beta0, beta1=beta1, clip_x0=0 if clip is None else 1,
                              clip_val=0.0 if clip is None else float(clip), B_max=B_max, K_max=K_max, seed=seed,
                              sampler=sampler, eta=eta, bonus_row=1 if bonus_row else 0, norm=norm)
        self.ctx = C.c_void_p()
        rc = self.lib.tsdp_create(C.byref(self.cfg), C.byref(self.ctx))
        if rc != 0:
            self.ctx = C.c_void_p()
            raise TsdpError(rc, "tsdp_create rejected the configuration")
        self.H, self.A, self.D, self.K_max, self.B_max = H, A, H * A, K_max, B_max
        self.rows_per_env = K_max + (1 if bonus_row else 0)

    @classmethod
    def from_workload(cls, wl, *, B_max=None, K_max=None, clip=None, seed=None, sampler=0, eta=1.0, bonus_row=False, norm=0):
        return cls(dtype=0 if wl.dtype == "fp32" else 1, H=wl.H, A=wl.A, cond_mode=wl.cond_mode, cond_dim=wl.cond_dim,
                   cond_tokens=wl.cond_tokens, base=(wl.base.layers, wl.base.d, wl.base.heads, wl.base.mlp_ratio),
                   draft=(wl.draft.layers, wl.draft.d, wl.draft.heads, wl.draft.mlp_ratio), T=wl.T,
                   schedule=wl.schedule, beta0=wl.beta0 or 1e-4, beta1=wl.beta1 or 0.02, clip=clip,
                   B_max=wl.B if B_max is None else B_max, K_max=wl.K_max if K_max is None else K_max,
                   seed=wl.philox_seed if seed is None else seed, sampler=sampler, eta=eta,
                   bonus_row=bonus_row, norm=norm)

    def close(self):
        if self.ctx:
            self.lib.tsdp_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc):
        if rc != 0:
            raise TsdpError(rc, self.lib.tsdp_last_error(self.ctx).decode())

    def path_name(self, which):
        return self.lib.tsdp_path_name(self.ctx, which).decode()

    def tsdp_load_weights(self, which, blob):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        self._chk(self.lib.tsdp_load_weights(self.ctx, which, blob.ctypes.data, blob.nbytes))

    def tsdp_set_cond(self, cond, stream=None):
        self._chk(self.lib.tsdp_set_cond(self.ctx, _ptr(cond, torch.float32), cond.shape[0], _stream(stream)))

    def alloc_rows(self, B, device="cuda"):
        """Caller-side ragged buffers for tsdp_draft / tsdp_verify / tsdp_accept (R_cap = B*(K_max + bonus_row) rows)."""
        R, D = B * self.rows_per_env, self.D
        f = lambda *s: torch.zeros(*s, dtype=torch.float32, device=device)
        i = lambda *s: torch.zeros(*s, dtype=torch.int32, device=device)
        return dict(row_ptr=i(B + 1), row_t=i(R), row_env=i(R), states=f(R, self.H, self.A), eps_p=f(R, self.H, self.A),
                    eps_q=f(R, self.H, self.A), xi=f(R, self.H, self.A), y_last=f(B, self.H, self.A))

    def tsdp_draft(self, x, t0, K, sigma_scale, env_id, rows, stream=None):
        B = x.shape[0]
        self._chk(self.lib.tsdp_draft(self.ctx, B, _ptr(x, torch.float32), _ptr(t0, torch.int32), _ptr(K, torch.int32),
                                      _ptr(sigma_scale, torch.float32), _ptr(env_id, torch.int32),
                                      _ptr(rows["row_ptr"]), _ptr(rows["row_t"]), _ptr(rows["row_env"]),
                                      _ptr(rows["states"]), _ptr(rows["eps_p"]), _ptr(rows["xi"]), _ptr(rows["y_last"]),
                                      _stream(stream)))

    def tsdp_verify(self, B, rows, R_cap=None, stream=None):
        R_cap = rows["row_t"].shape[0] if R_cap is None else R_cap
        self._chk(self.lib.tsdp_verify(self.ctx, B, R_cap, _ptr(rows["row_ptr"], torch.int32), _ptr(rows["row_t"], torch.int32),
                                       _ptr(rows["row_env"], torch.int32), _ptr(rows["states"], torch.float32),
                                       _ptr(rows["eps_q"], torch.float32), _stream(stream)))

    def tsdp_accept(self, B, sigma_scale, env_id, rows, diagnostics=True, stream=None):
        dev = rows["states"].device
        R = rows["row_t"].shape[0]
        out = dict(x_out=torch.empty(B, self.H, self.A, dtype=torch.float32, device=dev),
                   t_next=torch.empty(B, dtype=torch.int32, device=dev),
                   n_accept=torch.empty(B, dtype=torch.int32, device=dev),
                   n_adv=torch.empty(B, dtype=torch.int32, device=dev))
        if diagnostics:
            out.update(flags=torch.zeros(R, dtype=torch.uint8, device=dev),
                       logratio=torch.zeros(R, dtype=torch.float32, device=dev),
                       logu=torch.zeros(R, dtype=torch.float32, device=dev))
        self.tsdp_accept_into(B, sigma_scale, env_id, rows, out, stream)
        return out

    def tsdp_accept_into(self, B, sigma_scale, env_id, rows, out, stream=None):
        self._chk(self.lib.tsdp_accept(self.ctx, B, _ptr(rows["row_ptr"], torch.int32), _ptr(rows["row_t"], torch.int32),
                                       _ptr(env_id, torch.int32), _ptr(sigma_scale, torch.float32),
                                       _ptr(rows["states"], torch.float32), _ptr(rows["eps_p"], torch.float32),
                                       _ptr(rows["eps_q"], torch.float32), _ptr(rows["xi"], torch.float32),
                                       _ptr(rows["y_last"], torch.float32), _ptr(out["x_out"]), _ptr(out["t_next"]),
                                       _ptr(out["n_accept"]), _ptr(out.get("n_adv")), _ptr(out.get("flags")),
                                       _ptr(out.get("logratio")), _ptr(out.get("logu")), _stream(stream)))

    def tsdp_accept_threshold(self, B, sigma_scale, lam, rows, stream=None):
        dev = rows["states"].device
        R = rows["row_t"].shape[0]
        out = dict(x_out=torch.empty(B, self.H, self.A, dtype=torch.float32, device=dev),
                   t_next=torch.empty(B, dtype=torch.int32, device=dev), n_accept=torch.empty(B, dtype=torch.int32, device=dev),
                   n_adv=torch.empty(B, dtype=torch.int32, device=dev), flags=torch.zeros(R, dtype=torch.uint8, device=dev),
                   logratio=torch.zeros(R, dtype=torch.float32, device=dev))
        self._chk(self.lib.tsdp_accept_threshold(self.ctx, B, _ptr(rows["row_ptr"], torch.int32), _ptr(rows["row_t"], torch.int32),
                                                 _ptr(sigma_scale, torch.float32), _ptr(lam, torch.float32),
                                                 _ptr(rows["states"], torch.float32), _ptr(rows["eps_p"], torch.float32),
                                                 _ptr(rows["eps_q"], torch.float32), _ptr(rows["xi"], torch.float32),
                                                 _ptr(rows["y_last"], torch.float32), _ptr(out["x_out"]), _ptr(out["t_next"]),
                                                 _ptr(out["n_accept"]), _ptr(out["n_adv"]), _ptr(out["flags"]),
                                                 _ptr(out["logratio"]), _stream(stream)))
        return out

    def tsdp_round_threshold(self, x, t, K, sigma_scale, env_id, lam, n_accept=None, n_advanced=None, stream=None):
        self._chk(self.lib.tsdp_round_threshold(self.ctx, x.shape[0], _ptr(x, torch.float32), _ptr(t, torch.int32),
                                                _ptr(K, torch.int32), _ptr(sigma_scale, torch.float32),
                                                _ptr(env_id, torch.int32), _ptr(lam, torch.float32),
                                                _ptr(n_accept, torch.int32), _ptr(n_advanced, torch.int32), _stream(stream)))

    def tsdp_chain(self, x, t, K, sigma_scale, env_id, lam=None, max_rounds=1000, check_every=4, totals=True, stream=None):
        """Runs rounds until every environment finishes; returns (rounds, totals dict or None)."""
        B = x.shape[0]
        tot = None
        if totals:
            tot = {k: torch.zeros(B, dtype=torch.int32, device=x.device) for k in ("accept", "drafts", "rounds")}
        n = C.c_int32(0)
        self._chk(self.lib.tsdp_chain(self.ctx, B, _ptr(x, torch.float32), _ptr(t, torch.int32), _ptr(K, torch.int32),
                                      _ptr(sigma_scale, torch.float32), _ptr(env_id, torch.int32), _ptr(lam, torch.float32),
                                      max_rounds, check_every, _ptr(tot["accept"]) if tot else None,
                                      _ptr(tot["drafts"]) if tot else None, _ptr(tot["rounds"]) if tot else None,
                                      C.byref(n), _stream(stream)))
        return n.value, tot

    def tsdp_chain_staged(self, x, t, K3, sigma_scale3, lam3, t_hi, t_lo, env_id, max_rounds=1000, check_every=4,
                          totals=True, stream=None):
        """tsdp_chain with [B,3] stage tables; returns (rounds, totals dict or None)."""
        B = x.shape[0]
        tot = None
        if totals:
            tot = {k: torch.zeros(B, dtype=torch.int32, device=x.device) for k in ("accept", "drafts", "rounds")}
        n = C.c_int32(0)
        self._chk(self.lib.tsdp_chain_staged(self.ctx, B, _ptr(x, torch.float32), _ptr(t, torch.int32),
                                             _ptr(K3, torch.int32), _ptr(sigma_scale3, torch.float32),
                                             _ptr(lam3, torch.float32), t_hi, t_lo, _ptr(env_id, torch.int32),
                                             max_rounds, check_every, _ptr(tot["accept"]) if tot else None,
                                             _ptr(tot["drafts"]) if tot else None, _ptr(tot["rounds"]) if tot else None,
                                             C.byref(n), _stream(stream)))
        return n.value, tot

    def tsdp_chain_enqueue(self, x, t, K, sigma_scale, lam, env_id, n_rounds, *, stages=None, totals=None,
                           rounds_run=None, stream=None):
        """Enqueues exactly n_rounds rounds with no host round trip.  stages = (t_hi, t_lo) makes K, sigma_scale and
        lam [B,3] stage tables.  totals: dict of caller-allocated int32[B] device tensors (accept, drafts, rounds) or
        None; rounds_run: caller-allocated int32[1] device tensor or None."""
        tot = totals or {}
        self._chk(self.lib.tsdp_chain_enqueue(self.ctx, x.shape[0], _ptr(x, torch.float32), _ptr(t, torch.int32),
                                              _ptr(K, torch.int32), _ptr(sigma_scale, torch.float32),
                                              _ptr(lam, torch.float32), 0 if stages is None else 1,
                                              0 if stages is None else stages[0], 0 if stages is None else stages[1],
                                              _ptr(env_id, torch.int32), n_rounds, _ptr(tot.get("accept")),
                                              _ptr(tot.get("drafts")), _ptr(tot.get("rounds")),
                                              _ptr(rounds_run, torch.int32), _stream(stream)))

    def tsdp_prepare(self):
        self._chk(self.lib.tsdp_prepare(self.ctx))

    def tsdp_distill_loss(self, R, rows, lambda1, lambda2, stream=None):
        loss = torch.zeros(3, dtype=torch.float64, device=rows["states"].device)
        self._chk(self.lib.tsdp_distill_loss(self.ctx, R, _ptr(rows["row_t"], torch.int32), _ptr(rows["states"], torch.float32),
                                             _ptr(rows["eps_p"], torch.float32), _ptr(rows["eps_q"], torch.float32),
                                             lambda1, lambda2, _ptr(loss), _stream(stream)))
        return loss

    def tsdp_distill_loss_noalloc(self, R, rows, lambda1, lambda2, loss, stream=None):
        """`loss`: caller-allocated float64[3] device tensor (this entry point allocates nothing)."""
        self._chk(self.lib.tsdp_distill_loss_noalloc(self.ctx, R, _ptr(rows["row_t"], torch.int32),
                                                     _ptr(rows["states"], torch.float32), _ptr(rows["eps_p"], torch.float32),
                                                     _ptr(rows["eps_q"], torch.float32), lambda1, lambda2,
                                                     _ptr(loss, torch.float64), _stream(stream)))

    def tsdp_round(self, x, t, K, sigma_scale, env_id, n_accept=None, n_advanced=None, stream=None):
        self._chk(self.lib.tsdp_round(self.ctx, x.shape[0], _ptr(x, torch.float32), _ptr(t, torch.int32),
                                      _ptr(K, torch.int32), _ptr(sigma_scale, torch.float32), _ptr(env_id, torch.int32),
                                      _ptr(n_accept, torch.int32), _ptr(n_advanced, torch.int32), _stream(stream)))

    def tsdp_kernel_timing(self, enable):
        """False / 0 = off, True / 1 = all stages, 2 * mask = chosen stages (mask bit 0 drafter, 1 verify, 2 accept)."""
        self._chk(self.lib.tsdp_kernel_timing(self.ctx, int(enable)))

    def tsdp_kernel_ms(self, stage):
        ms = C.c_float(0)
        self._chk(self.lib.tsdp_kernel_ms(self.ctx, stage, C.byref(ms)))
        return ms.value

    def tsdp_status(self, stream=None):
        st = C.c_int32(0)
        self._chk(self.lib.tsdp_status(self.ctx, _stream(stream), C.byref(st)))
        return st.value
