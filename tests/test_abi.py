"""The C-ABI library: it loads, exports every symbol the header declares, and its host-side
argument checks work.  No kernel is launched here (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def zb():
    from paper_2503_10714_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding


def header_symbols():
    text = open(os.path.join(ROOT, "include", "zsm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zsm_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(zb):
    names = header_symbols()
    assert len(names) >= 13
    lib = zb.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/zsm.h but not exported"
    assert sorted(zb.EXPORTS) == names


def test_binding_has_the_same_names(zb):
    for n in header_symbols():
        assert callable(getattr(zb, n)), n


def test_cache_bytes_and_config_checks(zb):
    cfg = zb.make_config(2, 3, 4, 1, 128, 205, 1, "f16")
    n = zb.zsm_cache_bytes(cfg)
    units = 2 * 3 * 4
    kv = 2 * units * 204 * 128 * 2
    # scratch of the split decode step: per workgroup a denominator and an output share, per unit the
    # per-slot exponentials (fp64)
    wgs = min(units * 64, 8192)
    scratch = wgs * 8 + wgs * 128 * 4 + units * 206 * 8
    assert kv + scratch <= n <= kv + scratch + units * 205 * 12 + 2 * units * 128 * 4 + units * 16 + 22 * 256
    assert zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 129, 128, 205, 1, "f16")) == 0    # G = 129
    # more than eight query heads run as shares of eight or four: the scratch of eight, with one array of per-slot
    # sums per share (here 18 shares of four for 71 heads: more waves stay resident than with nine of eight) instead
    # of one per head (eight)
    n71, n8 = (zb.zsm_cache_bytes(zb.make_config(2, 3, 4, g, 128, 205, 1, "f16")) for g in (71, 8))
    assert 0 <= n71 - n8 - (18 - 8) * units * 206 * 8 < 256
    assert zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 0, 128, 205, 1, "f16")) == 0      # G = 0
    # three query heads run the kernels of four: the same scratch, hence the same cache size
    assert zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 3, 128, 205, 1, "f16")) == zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 4, 128, 205, 1, "f16"))
    assert zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 1, 96, 205, 1, "f16")) == 0       # d = 96
    assert zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 1, 128, 1, 1, "f16")) == 0        # no token slot
    assert zb.zsm_cache_bytes(zb.make_config(2, 3, 4, 1, 128, 205, 1, "f16", lam=1.5)) == 0


def test_alloc_rejects_bad_arguments_before_touching_the_device(zb):
    lib = zb.lib()
    cfg = zb.make_config(1, 2, 1, 1, 64, 16, 1, "f32")
    bp = (C.c_int32 * 2)(4, 4)
    bc = (C.c_int32 * 2)(4, 4)
    out = C.c_void_p()
    fake = C.c_void_p(1 << 20)     # never dereferenced: every call below fails validation first
    assert lib.zsm_cache_alloc(None, bp, bc, fake, 1 << 30, None, C.byref(out)) == -1
    assert lib.zsm_cache_alloc(C.byref(cfg), bp, bc, None, 1 << 30, None, C.byref(out)) == -1
    bad = (C.c_int32 * 2)(0, 4)
    assert lib.zsm_cache_alloc(C.byref(cfg), bad, bc, fake, 1 << 30, None, C.byref(out)) == -2     # B_p = 0
    big = (C.c_int32 * 2)(4, 12)
    assert lib.zsm_cache_alloc(C.byref(cfg), bp, big, fake, 1 << 30, None, C.byref(out)) == -2     # over capacity
    assert lib.zsm_cache_alloc(C.byref(cfg), bp, bc, C.c_void_p((1 << 20) + 16), 1 << 30, None, C.byref(out)) == -4
    assert lib.zsm_cache_alloc(C.byref(cfg), bp, bc, fake, 128, None, C.byref(out)) == -5
    cfg.kv_dtype = 7
    assert lib.zsm_cache_alloc(C.byref(cfg), bp, bc, fake, 1 << 30, None, C.byref(out)) == -3
    assert out.value is None


def test_null_handles_and_strerror(zb):
    lib = zb.lib()
    assert lib.zsm_cache_free(None) == -1
    assert lib.zsm_decode_step(None, 0, 1, None, None, None, None, None, None, None, None) == -1
    assert lib.zsm_prefill_workspace_bytes(None, 1, 10, 10) == 0
    assert lib.zsm_stream_copy(None, None, 16, None) == -1
    for code in range(-7, 1):
        assert zb.zsm_strerror(code)
    assert "unknown" in zb.zsm_strerror(-99)


def test_product_path_has_no_oracle_or_cpu_fallback():
    """Nothing under the package may import the oracle."""
    pkg = os.path.join(ROOT, "paper_2503_10714_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.replace("the oracle", "").replace("CPU oracle", "") or f == "synth.py", f
