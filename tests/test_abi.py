"""Host-side checks of the C ABI: the library loads, exports every declared symbol and rejects bad
configurations without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    from paper_2512_15773_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2512_15773_amd.build import build_library
        build_library(verbose=False)
    return binding, binding.load_library()


def test_exports_match_header():
    binding, lib = _lib()
    header = open(os.path.join(ROOT, "include", "tsdp.h")).read()
    declared = set(re.findall(r"\b(tsdp_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_config_struct_matches_header_field_order():
    binding, _ = _lib()
    header = open(os.path.join(ROOT, "include", "tsdp.h")).read()
    body = header[header.index("typedef struct {"):header.index("} tsdp_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.replace("typedef struct {", "").strip()
        if not decl:
            continue
        names = decl.split(None, 1)[1]
        fields += [n.strip() for n in names.split(",")]
    assert fields == [f[0] for f in binding.TsdpConfig._fields_]


def test_create_rejects_bad_configs_on_the_host():
    binding, lib = _lib()
    good = dict(dtype=0, H=16, A=2, cond_mode=0, cond_dim=64, cond_tokens=0, base_layers=2, base_d=64, base_heads=2,
                base_mlp_ratio=4, draft_layers=1, draft_d=32, draft_heads=2, draft_mlp_ratio=4, T=10, schedule=0,
                beta0=1e-4, beta1=0.02, clip_x0=0, clip_val=0.0, B_max=1, K_max=4, seed=0, sampler=0, eta=1.0, bonus_row=0, norm=0)
    for bad in (dict(dtype=7), dict(H=0), dict(A=3, H=3), dict(base_heads=3), dict(T=0), dict(schedule=5),
                dict(K_max=0), dict(cond_mode=1, cond_tokens=0), dict(clip_x0=1, clip_val=0.0), dict(beta0=-1.0),
                dict(sampler=2), dict(bonus_row=2), dict(norm=2), dict(sampler=1, eta=0.0), dict(sampler=1, eta=1.5)):
        cfg = binding.TsdpConfig(**{**good, **bad})
        ctx = C.c_void_p()
        assert lib.tsdp_create(C.byref(cfg), C.byref(ctx)) == -1, bad
        assert not ctx.value
    assert lib.tsdp_create(None, None) == -1
    lib.tsdp_destroy(None)                                             # allowed
    assert lib.tsdp_last_error(None) == b"null context"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
    assert not any(line.startswith("{") for line in r.stdout.splitlines())      # no result line
