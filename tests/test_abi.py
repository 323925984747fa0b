"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and
rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2603_11504_amd import longflow as lf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "longflow.h")).read()
    declared = set(re.findall(r"LF_API[^;(]*?\b(longflow_\w+)\s*\(", header))
    assert declared == set(lf.EXPORTS)
    L = lf.lib()
    for name in declared:
        assert hasattr(L, name), name


def _cfg(**kw):
    base = dict(batch=2, q_heads=8, kv_heads=2, head_dim=128, budget=512, dtype="bf16", flags=0)
    base.update(kw)
    return lf.make_config(**base)


def test_workspace_bytes_and_geometry_validation():
    L = lf.lib()
    assert lf.longflow_workspace_bytes(_cfg()) > 0
    assert lf.longflow_workspace_bytes(_cfg()) % 256 == 0
    for bad in (dict(q_heads=7), dict(head_dim=96), dict(batch=0), dict(budget=0),
                dict(q_heads=2 * 17), dict(dtype="f32", q_heads=2 * 9), dict(flags=64)):
        assert lf.longflow_workspace_bytes(_cfg(**bad)) == 0
        assert L.longflow_last_error() != b""
    assert L.longflow_workspace_bytes(None) == 0
    # group 16 is served by the matrix-core kernel only
    assert lf.longflow_workspace_bytes(_cfg(q_heads=32)) > 0
    assert lf.longflow_workspace_bytes(_cfg(q_heads=32, flags=lf.LF_FLAG_FORCE_VALU)) == 0
    # bigger budget needs a bigger workspace
    assert lf.longflow_workspace_bytes(_cfg(budget=4096)) > lf.longflow_workspace_bytes(_cfg(budget=512))


def test_argument_errors_are_reported_before_any_launch():
    L = lf.lib()
    h = ctypes.c_void_p()
    cfg = _cfg()
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails on the host
    vp = ctypes.c_void_p
    rc = L.longflow_init_cache(ctypes.byref(h), ctypes.byref(cfg), None, fake, None, None, 0, fake, 1 << 30, None)
    assert rc == lf.LF_ERR_INVALID_ARG and not h.value
    rc = L.longflow_init_cache(ctypes.byref(h), ctypes.byref(cfg), fake, fake, None, None, 513, fake, 1 << 30, None)
    assert rc == lf.LF_ERR_INVALID_ARG and b"n_init" in L.longflow_last_error()
    rc = L.longflow_init_cache(ctypes.byref(h), ctypes.byref(cfg), fake, fake, None, None, 4, fake, 1 << 30, None)
    assert rc == lf.LF_ERR_INVALID_ARG
    rc = L.longflow_init_cache(ctypes.byref(h), ctypes.byref(cfg), fake, fake, None, None, 0, fake, 16, None)
    assert rc == lf.LF_ERR_WORKSPACE
    rc = L.longflow_init_cache(ctypes.byref(h), ctypes.byref(cfg), fake, fake, None, None, 0, vp(0x1001), 1 << 30, None)
    assert rc == lf.LF_ERR_INVALID_ARG
    bad = _cfg(head_dim=80)
    rc = L.longflow_init_cache(ctypes.byref(h), ctypes.byref(bad), fake, fake, None, None, 0, fake, 1 << 30, None)
    assert rc == lf.LF_ERR_UNSUPPORTED
    assert L.longflow_init_cache(None, ctypes.byref(cfg), fake, fake, None, None, 0, fake, 1 << 30, None) == lf.LF_ERR_INVALID_ARG
    # calls on a NULL handle
    assert L.longflow_decode_step(None, fake, fake, fake, fake, None, None) == lf.LF_ERR_STATE
    assert L.longflow_scores(None, fake, None) == lf.LF_ERR_STATE
    assert L.longflow_set_pending(None, fake, None) == lf.LF_ERR_STATE
    assert L.longflow_destroy_cache(None) == lf.LF_ERR_STATE
    assert L.longflow_valid_count(None) < 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(lf, "_lib", None)
    monkeypatch.setattr(lf, "LIB_PATH", "/nonexistent/liblongflow.so")
    with pytest.raises(ImportError):
        lf.lib()
