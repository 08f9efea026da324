"""Host-only checks of the C ABI (no GPU, no kernel launches): the library
loads, exports every symbol the headers declare, and validates arguments."""
import ctypes
import os
import re

import pytest

from paper_2510_24211_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for hdr in ("scd.h", "scd_workload.h"):
        src = open(os.path.join(ROOT, "include", hdr)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(scdw?_[a-z_]+)\s*\(", src))
    return names


def test_library_exports_every_declared_symbol():
    lib = B.load()
    decl = _declared_symbols()
    assert {"scd_step", "scd_verify", "scd_couple_draft", "scd_lm_head"} <= decl
    for name in decl:
        assert hasattr(lib, name), name


def test_config_struct_matches_header_layout(tmp_path):
    """sizeof / offsetof as the C compiler sees the header against the ctypes mirror."""
    import os
    import subprocess
    fields = [name for name, _ in B.ScdConfig._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "scd.h"\nint main(void) {\n'
                   '  printf("%zu", sizeof(scd_config));\n' +
                   "".join(f'  printf(" %zu", offsetof(scd_config, {f}));\n' for f in fields) +
                   "  return 0;\n}\n")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", inc, str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert got[0] == ctypes.sizeof(B.ScdConfig) == 64
    assert got[1:] == [getattr(B.ScdConfig, f).offset for f in fields]


def test_size_queries_validate_config():
    ok = B.make_config(B=2, L=32, N=100, V=1000, d=64, top_k=10)
    assert B.workspace_bytes(ok) > 0
    # state holds two copies of the [B, L, n] fp32 logits plus small arrays
    assert B.state_bytes(ok) >= 2 * 2 * 32 * 1000 * 4
    bad = [dict(B=0), dict(L=0), dict(L=257), dict(N=0), dict(V=0), dict(d=12), dict(d=-8),
           dict(v_lo=-1), dict(v_lo=10, v_hi=10), dict(v_hi=1001), dict(top_k=-1),
           dict(temperature=0.0), dict(temperature=float("nan")), dict(cfg_lambda=float("inf"))]
    for kw in bad:
        args = dict(B=2, L=32, N=100, V=1000, d=64, top_k=10)
        args.update(kw)
        cfg = B.make_config(**args)
        assert B.workspace_bytes(cfg) == 0, kw
        assert B.state_bytes(cfg) == 0, kw


def test_create_rejects_bad_arguments_without_touching_the_device():
    lib = B.load()
    cfg = B.make_config(B=1, L=8, N=64, V=1024)
    need = B.workspace_bytes(cfg)
    ctx = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x10000)          # never dereferenced by scd_create
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(cfg), None, need, None) == B.SCD_EWORKSPACE
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(cfg), ctypes.c_void_p(0x10010), need, None) \
        == B.SCD_EWORKSPACE                                   # misaligned
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(cfg), fake, need - 1, None) == B.SCD_EWORKSPACE
    assert lib.scd_create(None, ctypes.byref(cfg), fake, need, None) == B.SCD_EINVAL
    bad = B.make_config(B=1, L=8, N=64, V=1024, coupling=2)           # no such coupling
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(bad), fake, need, None) == B.SCD_EUNSUPPORTED
    neg = B.make_config(B=1, L=8, N=64, V=1024, sjd_mix=1.5)           # probability outside [0, 1]
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(neg), fake, need, None) == B.SCD_EINVAL
    big = B.make_config(B=1, L=8, N=64, V=70000, coupling=B.COUPLING_GS)   # GS: rows <= 65536 ids
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(big), fake, 1 << 40, None) == B.SCD_EUNSUPPORTED
    wide = B.make_config(B=1, L=8, N=64, V=70000, top_p=0.8)          # nucleus: rows <= 65536 ids
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(wide), fake, 1 << 40, None) == B.SCD_EUNSUPPORTED
    dg = B.make_config(B=1, L=8, N=64, V=70000, diagnostics=1)        # statistics: rows <= 65536 ids
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(dg), fake, 1 << 40, None) == B.SCD_EUNSUPPORTED
    off = B.make_config(B=1, L=8, N=64, V=1024, top_p=1.25)            # mass outside [0, 1]
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(off), fake, need, None) == B.SCD_EINVAL
    assert lib.scd_create(ctypes.byref(ctx), ctypes.byref(cfg), fake, need, None) == B.SCD_OK
    # null pointers are refused before any launch
    assert lib.scd_lm_head(ctx, None, None, None) == B.SCD_EINVAL
    assert lib.scd_step(ctx, None, None, None) == B.SCD_EINVAL
    assert lib.scd_step_logits(ctx, None, None) == B.SCD_EINVAL
    assert lib.scd_couple_draft(ctx, None, None, None, None, None, 0, None, None) == B.SCD_EINVAL
    assert lib.scd_verify(ctx, None, None, None, None, None) == B.SCD_EINVAL
    assert lib.scd_reset(ctx, None) == B.SCD_EINVAL
    # d == 0: the LM-head entry points are refused
    assert lib.scd_lm_head(ctx, fake, fake, fake) == B.SCD_EINVAL
    # state layout is host arithmetic: fields are disjoint, aligned, inside the buffer
    total = B.state_bytes(cfg)
    base = 0x100000
    spans = []
    for f in range(B.F_COUNT):
        p, nb = ctypes.c_void_p(), ctypes.c_size_t()
        assert lib.scd_state_field(ctx, ctypes.c_void_p(base), f, ctypes.byref(p), ctypes.byref(nb)) == 0
        assert p.value % 256 == 0 and nb.value > 0
        spans.append((p.value - base, p.value - base + nb.value))
    spans.sort()
    assert spans[-1][1] <= total
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    assert lib.scd_state_field(ctx, ctypes.c_void_p(base), B.F_COUNT, ctypes.byref(p), ctypes.byref(nb)) == B.SCD_EINVAL
    assert lib.scd_destroy(ctx) == B.SCD_OK
    assert lib.scd_destroy(None) == B.SCD_EINVAL
    assert B.strerror(B.SCD_EWORKSPACE).startswith("workspace")


def test_gather_rejects_bad_arguments():
    lib = B.load()
    fake = ctypes.c_void_p(0x10000)
    assert lib.scdw_gather_hidden(None, None, 1, 1, 8, 64, 64, 4, fake, fake, fake) == -1
    assert lib.scdw_gather_hidden(None, fake, 1, 1, 8, 64, 60, 4, fake, fake, fake) == -1
