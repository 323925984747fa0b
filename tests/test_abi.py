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
                dict(q_heads=2 * 17), dict(dtype="f32", q_heads=2 * 9, flags=lf.LF_FLAG_FORCE_VALU), dict(flags=64)):
        assert lf.longflow_workspace_bytes(_cfg(**bad)) == 0
        assert L.longflow_last_error() != b""
    assert L.longflow_workspace_bytes(None) == 0
    # group 16 is served by the matrix-core kernels only
    assert lf.longflow_workspace_bytes(_cfg(q_heads=32)) > 0
    assert lf.longflow_workspace_bytes(_cfg(q_heads=32, dtype="f32")) > 0
    assert lf.longflow_workspace_bytes(_cfg(q_heads=32, head_dim=64)) > 0
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


# ------------------------------------------------------------------ execution plan (host logic)

LDS_PER_CU = 160 * 1024


def _plans():
    import itertools
    for dtype, D, G, Hkv, B, N, flags in itertools.product(
            ("bf16", "f32"), (64, 128), (1, 4, 7, 8, 16), (1, 8), (1, 3, 32, 64, 300),
            (1, 16, 17, 255, 2048, 8192, 16384, 81920, 500000),
            (0, lf.LF_FLAG_ATTENTION_ONLY, lf.LF_FLAG_FORCE_SPLIT, lf.LF_FLAG_FORCE_VALU)):
        cfg = lf.make_config(B, G * Hkv, Hkv, D, N, dtype, flags)
        if lf.longflow_workspace_bytes(cfg) == 0:
            continue
        yield (dtype, D, G, Hkv, B, N, flags), cfg, lf.longflow_plan_info(cfg)


def test_every_accepted_configuration_has_a_consistent_plan():
    seen = set()
    count = 0
    for key, cfg, info in _plans():
        dtype, D, G, Hkv, B, N, flags = key
        count += 1
        seen.add(info.path)
        # the workgroups of a unit cover its slots, none of them idle at a full cache
        assert info.workgroups_per_unit >= 1
        assert info.workgroups_per_unit * info.slots_per_workgroup >= N, key
        assert (info.workgroups_per_unit - 1) * info.slots_per_workgroup < N, key
        assert info.launches_per_step in (1, 2)
        mfma_ok = dtype == "bf16" and D == 128 and not flags & lf.LF_FLAG_FORCE_VALU
        if info.path == lf.LF_PATH_UNIT_MFMA:
            assert mfma_ok and not flags & lf.LF_FLAG_FORCE_SPLIT
            assert info.workgroups_per_unit <= 8 and info.launches_per_step == 1
            assert info.threads_per_workgroup == 512
            # dynamic LDS plus the kernel's static arrays must fit one compute unit
            assert 0 < info.lds_bytes <= LDS_PER_CU - 12 * 1024, key
            if not flags & lf.LF_FLAG_ATTENTION_ONLY:
                # one byte per (head, slot) of the workgroup's share, plus per-tile references
                assert info.lds_bytes >= G * min(info.slots_per_workgroup, N), key
            if B * Hkv >= 192 and info.workgroups_per_unit > 1:
                # plenty of units: more than one workgroup only when the codes demand it
                one = G * N + (N // 16 + 1) * G * 4
                assert flags & lf.LF_FLAG_ATTENTION_ONLY == 0 and one > LDS_PER_CU - 12 * 1024, key
        else:
            valu = bool(flags & lf.LF_FLAG_FORCE_VALU)
            assert info.path == (lf.LF_PATH_SPLIT_MFMA if mfma_ok else lf.LF_PATH_SPLIT_VALU if valu else lf.LF_PATH_SPLIT_MFMA_F32), key
            assert not (valu and G > 8), key
            assert info.workgroups_per_unit <= 64 and info.slots_per_workgroup % 256 == 0
            big = info.workgroups_per_unit > 1 and B * Hkv * info.workgroups_per_unit > 256
            assert info.launches_per_step == (2 if big else 1), key
    assert count > 1000 and seen == {0, 1, 2, 3}


def test_plan_of_the_baseline_workloads():
    from paper_2603_11504_amd import workloads as W
    got = []
    for wl in W.CONFIGS:
        i = lf.longflow_plan_info(lf.make_config(wl.batch, wl.q_heads, wl.kv_heads, wl.head_dim, wl.budget, wl.dtype, 0))
        got.append((lf.PATH_KERNELS[i.path], i.workgroups_per_unit, i.slots_per_workgroup))
    assert got == [("split_mfma32_kernel", 1, 256), ("unit_mfma_kernel", 8, 256), ("unit_mfma_kernel", 2, 2048),
                   ("unit_mfma_kernel", 1, 8192), ("unit_mfma_kernel", 1, 16384)]


def test_plan_info_rejects_what_init_rejects():
    L = lf.lib()
    info = lf.lf_plan_info()
    bad = lf.make_config(2, 7, 2, 128, 512, "bf16", 0)
    assert L.longflow_plan_info(ctypes.byref(bad), ctypes.byref(info)) == lf.LF_ERR_UNSUPPORTED
    assert L.longflow_plan_info(ctypes.byref(bad), None) == lf.LF_ERR_INVALID_ARG
    assert L.longflow_plan_info(None, ctypes.byref(info)) == lf.LF_ERR_INVALID_ARG


def test_group_calls_reject_bad_arguments_on_the_host():
    L = lf.lib()
    assert L.longflow_group_workspace_bytes(0) == 0
    assert L.longflow_group_workspace_bytes(3) % 256 == 0 and L.longflow_group_workspace_bytes(3) > 0
    g = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x1000)
    assert L.longflow_group_create(ctypes.byref(g), None, 2, fake, 1 << 20, None) == lf.LF_ERR_INVALID_ARG
    none = (ctypes.c_void_p * 2)(None, None)
    assert L.longflow_group_create(ctypes.byref(g), none, 2, None, 1 << 20, None) == lf.LF_ERR_INVALID_ARG
    assert L.longflow_group_create(ctypes.byref(g), none, 2, fake, 16, None) == lf.LF_ERR_WORKSPACE
    assert L.longflow_group_create(ctypes.byref(g), none, 2, fake, 1 << 20, None) == lf.LF_ERR_STATE  # NULL members
    assert not g.value
    assert L.longflow_group_decode_step(None, fake, fake, fake, fake, None, None) == lf.LF_ERR_STATE
    assert L.longflow_group_destroy(None) == lf.LF_ERR_STATE


def test_unfused_comparison_path_is_validated_on_the_host():
    L = lf.lib()
    UNF = lf.LF_FLAG_UNFUSED_ACCUM
    fused = L.longflow_workspace_bytes(ctypes.byref(_cfg()))
    unf = L.longflow_workspace_bytes(ctypes.byref(_cfg(flags=UNF)))
    assert unf > 0 and fused > 0
    # the per-slot fp32 books are part of its workspace
    plain = L.longflow_workspace_bytes(ctypes.byref(_cfg(flags=lf.LF_FLAG_ATTENTION_ONLY)))
    assert unf >= plain + 4 * 2 * 2 * 512
    for bad in (_cfg(flags=UNF, head_dim=64), _cfg(flags=UNF, dtype="f32"),
                _cfg(flags=UNF | lf.LF_FLAG_ATTENTION_ONLY), _cfg(flags=UNF | lf.LF_FLAG_FORCE_VALU)):
        assert L.longflow_workspace_bytes(ctypes.byref(bad)) == 0
    a = lf.longflow_plan_info(_cfg(flags=lf.LF_FLAG_ATTENTION_ONLY))
    u = lf.longflow_plan_info(_cfg(flags=UNF))
    assert u.launches_per_step == a.launches_per_step + 3
    assert (u.path, u.workgroups_per_unit, u.slots_per_workgroup) == (a.path, a.workgroups_per_unit, a.slots_per_workgroup)


def test_binding_checks_what_the_c_side_cannot_see():
    import torch
    bf = torch.bfloat16
    ok = torch.zeros(2, 8, 128, dtype=bf)
    # not on a device, wrong element count, wrong element type, not contiguous
    for bad, n, dt in ((ok, 2048, bf), (ok, 1024, bf), (ok.float(), 2048, torch.float32), (ok.transpose(0, 1), 2048, bf)):
        with pytest.raises(ValueError):
            lf._arg(bad, n, dt, "q")
    assert lf._arg(None, 5, bf, "k_new") is None


# ------------------------------------------------------------------ workspace carving (host logic)

def test_workspace_regions_never_overlap_and_hold_every_index_the_kernels_form():
    # Bounds checks on the host: for every accepted configuration the regions of the workspace are
    # disjoint, aligned and inside longflow_workspace_bytes, and each is at least as large as the
    # highest index its kernels form.  The index bounds below are written out from the kernels'
    # addressing, independently of the library's own size computation:
    #   counters, pending      one int32 per (batch, KV head) unit
    #   q_last                 the step's query, [B][Hq][D] elements
    #   part_m / part_l        fused kernel: [unit][workgroup of the unit][16] floats;
    #                          split-K: [unit][split][G] floats
    #   part_o                 [unit][workgroup or split][G][D] floats
    #   stash_w                fused kernel, several workgroups per unit: 1-byte codes [unit][G][tiles*16];
    #                          split-K: bf16 [unit][tile][G][16]
    #   stash_m                [unit][tile][G] floats
    #   lu                     [unit][tiles*16] floats
    #   fin_m / fin_l          [unit][G] floats
    checked = 0
    for key, cfg, info in _plans():
        dtype, D, G, Hkv, B, N, flags = key
        units, esz, tiles = B * Hkv, (4 if dtype == "f32" else 2), (N + 15) // 16
        regs = lf.longflow_workspace_regions(cfg)
        total = lf.longflow_workspace_bytes(cfg)
        names = [r[0] for r in regs]
        assert len(set(names)) == len(names)
        end = 0
        for name, off, size in regs:
            assert off % 256 == 0 and off >= end, (key, name)      # aligned, in order, no overlap
            end = off + size
        assert end <= total
        have = {name: size for name, _, size in regs}
        wgs = info.workgroups_per_unit
        scoring = not flags & lf.LF_FLAG_ATTENTION_ONLY
        need = {"pending": 4 * units, "arrive": 4 * units, "first_hole": 4 * units,
                "q_last": esz * B * G * Hkv * D, "fin_m": 4 * units * G, "fin_l": 4 * units * G,
                "part_o": 4 * units * wgs * G * D}
        if info.path == lf.LF_PATH_UNIT_MFMA:
            need["part_m"] = need["part_l"] = 4 * units * wgs * 16
            if scoring and wgs > 1:
                need["stash_w"] = units * G * tiles * 16
                need["stash_m"] = 4 * units * tiles * G
        else:
            need["part_m"] = need["part_l"] = 4 * units * wgs * G
            if scoring:
                need["stash_w"] = 2 * units * tiles * G * 16
                need["stash_m"] = 4 * units * tiles * G
        if scoring:
            need["lu"] = 4 * units * tiles * 16
        for name, size in need.items():
            assert have[name] >= size, (key, name, have[name], size)
        checked += 1
    assert checked > 1000
    # the comparison path's books
    cfg = lf.make_config(4, 8, 2, 128, 1000, "bf16", lf.LF_FLAG_UNFUSED_ACCUM)
    have = {name: size for name, _, size in lf.longflow_workspace_regions(cfg)}
    assert have["acc"] >= 4 * 8 * 63 * 16 and have["acc_part_v"] > 0 and have["acc_part_i"] == have["acc_part_v"]


def test_compress_scratch_bytes_host_query():
    import ctypes
    L = lf.lib()
    cfg = _cfg(batch=4, q_heads=28, kv_heads=4, budget=1024)
    f = lambda T, W, c=cfg: int(L.longflow_compress_scratch_bytes(ctypes.byref(c), T, W))
    base = f(5000, 32)
    assert base > 0 and base % 256 == 0
    # votes and pooled votes (4 bytes per prefix row and unit each) and the kept rows must fit
    units = 16
    assert base >= 2 * 4 * units * (5000 - 32) + 4 * units * 1024
    assert f(10000, 32) > base and f(5000, 64) > base          # more rows, more query columns
    for T, W in ((0, 1), (10, 0), (10, 11), ((1 << 24) + 1, 32), (5000, 4096)):   # 4096 x 7 columns: too many
        assert f(T, W) == 0
    assert f(5000, 32, _cfg(head_dim=96)) == 0                  # invalid geometry
