"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2005_04347_amd as amd
    if not os.path.exists(amd.binding.LIB_PATH):
        from paper_2005_04347_amd.build import build
        build(verbose=False)
    return amd.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "asnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(asnn_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"asnn_build_levels", "asnn_pack_csr", "asnn_activate"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    import paper_2005_04347_amd.binding as b
    assert sorted(b.EXPORTS) == names


def test_error_strings(lib):
    assert lib.asnn_strerror(0) == b"ok"
    seen = set()
    for code in range(-12, 0):
        s = lib.asnn_strerror(code)
        assert s and s != b"unknown error" and s not in seen
        seen.add(s)
    assert lib.asnn_strerror(-99) == b"unknown error"
    assert lib.asnn_version() >= 1


def test_header_constants_match_binding():
    import paper_2005_04347_amd.binding as b
    text = open(os.path.join(ROOT, "include", "asnn.h")).read()
    for name, code in re.findall(r"#define (ASNN_ERR_[A-Z_]+) \((-\d+)\)", text):
        assert b.ERR_NAMES[int(code)] == name
    assert int(re.search(r"#define ASNN_HEAVY_INDEGREE (\d+)", text).group(1)) == b.HEAVY_INDEGREE
    assert int(re.search(r"#define ASNN_MEDIUM_INDEGREE (\d+)", text).group(1)) == b.MEDIUM_INDEGREE
    assert int(re.search(r"#define ASNN_CLASSES (\d+)", text).group(1)) == b.CLASSES
    assert int(re.search(r"#define ASNN_FLAG_RAW_INPUTS (\d+)u", text).group(1)) == b.FLAG_RAW_INPUTS
    assert int(re.search(r"#define ASNN_FLAG_ACC_F32 (\d+)u", text).group(1)) == b.FLAG_ACC_F32
    assert int(re.search(r"#define ASNN_FLAG_LEVEL_LAUNCHES (\d+)u", text).group(1)) == b.FLAG_LEVEL_LAUNCHES
    assert int(re.search(r"#define ASNN_FLAG_DATAFLOW (\d+)u", text).group(1)) == b.FLAG_DATAFLOW
    assert int(re.search(r"#define ASNN_FLAG_WORKGROUP (\d+)u", text).group(1)) == b.FLAG_WORKGROUP


def test_workspace_sizes_grow_and_align(lib):
    a = lib.asnn_levels_workspace_bytes(1000, 10000)
    b = lib.asnn_levels_workspace_bytes(100000, 1090000)
    assert 0 < a < b and a % 256 == 0 and b % 256 == 0
    # out-adjacency + two frontiers + a few node arrays: linear in N and E
    assert b < 16 * (100000 * 8 + 1090000)
    p = lib.asnn_pack_workspace_bytes(100000, 1090000)
    assert p % 256 == 0 and p > 4 * 4 * 1090000
    assert lib.asnn_levels_workspace_bytes(-1, 5) == 0


def test_argument_checks_need_no_device(lib):
    nl = ctypes.c_int32(-7)
    fake = ctypes.c_void_p(256)          # never dereferenced: every call below fails a host-side check first
    i32 = ctypes.c_int32
    assert lib.asnn_build_levels(-1, 0, None, None, None, 0, fake, ctypes.byref(nl), fake, 1 << 20, None) == -2
    assert lib.asnn_build_levels(4, -1, None, None, None, 0, fake, ctypes.byref(nl), fake, 1 << 20, None) == -2
    assert lib.asnn_build_levels(4, 2**31, fake, fake, None, 0, fake, ctypes.byref(nl), fake, 1 << 20, None) == -2
    assert lib.asnn_build_levels(4, 2**31 - 65535, fake, fake, None, 0, fake, ctypes.byref(nl), fake, 1 << 20, None) == -2
    # the largest count that is taken fails on the workspace, not on the size
    assert lib.asnn_build_levels(4, 2**31 - 65536, fake, fake, None, 0, fake, ctypes.byref(nl), ctypes.c_void_p(256), 1 << 20, None) == -7
    assert lib.asnn_build_levels(4, 2, None, fake, None, 0, fake, ctypes.byref(nl), fake, 1 << 20, None) == -1
    assert lib.asnn_build_levels(4, 2, fake, fake, None, 1, fake, ctypes.byref(nl), fake, 1 << 20, None) == -1
    assert lib.asnn_build_levels(4, 2, fake, fake, None, 0, fake, ctypes.byref(nl), None, 1 << 20, None) == -1
    assert lib.asnn_build_levels(4, 2, fake, fake, None, 0, fake, ctypes.byref(nl), fake, 16, None) == -7
    assert lib.asnn_build_levels(4, 2, fake, fake, None, 0, fake, ctypes.byref(nl), ctypes.c_void_p(264), 1 << 20, None) == -7
    assert lib.asnn_build_levels(0, 0, None, None, None, 0, None, ctypes.byref(nl), None, 0, None) == 0 and nl.value == 0
    import paper_2005_04347_amd.binding as b
    lph = (i32 * 4)(0, 0, 0, 4)
    F = 256

    def rec(**k):
        r = b.AsnnPacked(n_nodes=k.get("n", 4), n_levels=k.get("L", 1), n_edges=k.get("e", 0), n_units=1, first_unit=1,
                         level_ptr_host=ctypes.addressof(k.get("lph", lph)) if k.get("lph", lph) is not None else None,
                         level_ptr=F, perm=F, inv_perm=F, row_ptr=F, col=None, w=None, unit_ptr=F)
        for name in k.get("null", ()):
            setattr(r, name, None)
        return r

    pack = lambda r, ws=fake, nbytes=1 << 20: lib.asnn_pack_csr(None, None, None, fake, ctypes.byref(r), ws, nbytes, None)
    assert lib.asnn_pack_csr(None, None, None, fake, None, fake, 1 << 20, None) == -1
    assert pack(rec(n=0)) == -2
    assert pack(rec(L=9)) == -2
    assert pack(rec(null=("perm",))) == -1
    assert pack(rec(null=("unit_ptr",))) == -1
    assert pack(rec(), nbytes=8) == -7
    assert lib.asnn_pack_csr(None, None, None, None, ctypes.byref(rec()), fake, 1 << 20, None) == -1
    # activate: sizes, NULLs, alignment of V, and a level table that does not cover the rows
    act = lambda r, B=2, V=fake, flags=0, ws=None: lib.asnn_activate(ctypes.byref(r), fake, 1, None, 0, fake, B, V, None,
                                                                     ws, 0, flags, None)
    assert lib.asnn_activate(None, fake, 1, None, 0, fake, 2, fake, None, None, 0, 0, None) == -1
    assert act(rec(), B=0) == -2
    assert act(rec(n=0)) == -2
    assert act(rec(), V=None) == -1
    assert act(rec(), V=ctypes.c_void_p(260)) == -2
    assert act(rec(lph=(i32 * 4)(0, 0, 0, 3))) == -2
    assert act(rec(lph=(i32 * 4)(0, 5, 4, 4))) == -2
    assert act(rec(lph=None)) == -1
    assert act(rec(), flags=4 | 8) == -2                      # both schedules forced
    assert act(rec(), flags=8) == -1                          # dataflow forced without a workspace
    assert act(rec(), flags=4 | 16) == -2 and act(rec(), flags=8 | 16) == -2
    assert act(rec(null=("level_ptr",)), flags=16) == -1      # the workgroup schedule reads the device level table
    assert lib.asnn_activate_workspace_bytes(None, 4) == 0
    assert lib.asnn_activate_workspace_bytes(ctypes.byref(rec(n=0)), 4) == 0
    nbytes = lib.asnn_activate_workspace_bytes(ctypes.byref(rec(n=1000, e=16000)), 64)
    assert 0 < nbytes <= 4096 and nbytes % 256 == 0
    # a node with more than 512 connections is gathered in chunks whose partial sums pass through the workspace
    r = rec(n=1000, e=16000)
    r.max_heavy_indegree = 4096
    assert lib.asnn_activate_workspace_bytes(ctypes.byref(r), 64) >= 16000 * 64 // 32


def test_schedule_choice_follows_the_cost_estimate(lib):
    """asnn_activate_schedule is host arithmetic on the record: level launches (0) against the
    dataflow launch (1) by the per-level estimate, one workgroup per tile (2) for tiny jobs."""
    import paper_2005_04347_amd.binding as b
    F = 256

    def rec(n, L, e, heavy, units=None):            # light rows go 16 to a work unit
        return b.AsnnPacked(n_nodes=n, n_levels=L, n_edges=e, n_units=(n // 16 if units is None else units) + 10,
                            first_unit=10, max_heavy_indegree=heavy,
                            level_ptr_host=None, level_ptr=F, perm=F, inv_perm=F, row_ptr=F, col=F, w=F, unit_ptr=F)

    sched = lambda r, B, ws=1, flags=0: lib.asnn_activate_schedule(ctypes.byref(r), B, ws, flags)
    wide = rec(100000, 50, 1090000, 0)              # the 100k-node workload: no heavy rows
    assert [sched(wide, B) for B in (64, 256, 768, 1024)] == [1, 1, 1, 0]
    assert sched(wide, 256, ws=0) == 0              # no workspace, no dataflow
    deep = rec(1000000, 1000, 16000000, 4096)       # 1000 levels with rows of 4096 connections
    assert [sched(deep, B) for B in (8, 64, 512, 1024)] == [1, 1, 1, 1]
    assert sched(deep, 2048) == 1                   # also when the value matrix passes 4 GiB
    flat = rec(1000000, 1000, 16000000, 0)          # the same without heavy rows: the estimates meet near 20 M per level
    assert [sched(flat, B) for B in (64, 1024, 1536)] == [1, 1, 0]
    mlp = rec(2694, 4, 165680, 0, units=1910)       # few levels, a value matrix that fits the L2 caches, and
    assert [sched(mlp, B) for B in (16, 64, 256)] == [0, 0, 0]      # a work item per medium row with little in it
    assert sched(rec(400, 10, 17600, 0, units=380), 16) == 1        # the same rows, 40 to a level: dataflow
    tiny = rec(76, 20, 512, 0)
    assert sched(tiny, 1) == 2 and sched(tiny, 4096) == 2 and sched(tiny, 4096, ws=0) == 2
    assert sched(tiny, 1 << 20) == 0 and sched(tiny, 1 << 20, ws=0) == 0      # more tiles than the chip holds workgroups
    # the break-even of one workgroup per tile shrinks as the tile widens (fewer rows in flight)
    small = lambda e, L: rec(e // 10, L, e, 0)
    assert [sched(small(16000, 5), B) for B in (1, 4, 16)] == [2, 1, 1]
    assert [sched(small(4000, 20), B) for B in (1, 16, 64)] == [2, 2, 1]
    assert [sched(small(8000, 40), B) for B in (16, 64, 256)] == [2, 1, 2]
    assert [sched(small(70000, 80), B) for B in (1, 4)] == [2, 1]
    assert sched(wide, 256, flags=4) == 0 and sched(wide, 1024, flags=8) == 1 and sched(wide, 1024, flags=16) == 2


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    import paper_2005_04347_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(ImportError):
        b.load()


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2005_04347_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2005_04347_amd" not in text and "libasnn.so" not in text, f


def test_static_entry_point_refuses_on_the_host(lib):
    """asnn_activate_static checks its arguments, and whether the network and batch fit the library's
    scratch, before it touches a device."""
    import paper_2005_04347_amd.binding as b
    fake = ctypes.c_void_p(256)
    assert lib.asnn_activate_static(None, fake, 1, fake, 1, fake, 4, fake, fake, 0, None) == -1
    rec = b.AsnnPacked(n_nodes=1000, n_levels=3, n_edges=40_000_000, n_units=10, first_unit=1, max_heavy_indegree=4096)
    assert lib.asnn_activate_workspace_bytes(ctypes.byref(rec), 64) > b.STATIC_SCRATCH_BYTES
    assert lib.asnn_activate_static(ctypes.byref(rec), fake, 1, fake, 1, fake, 64, fake, fake, 0, None) == -12
    rec.n_nodes = 0
    assert lib.asnn_activate_static(ctypes.byref(rec), fake, 1, fake, 1, fake, 64, fake, fake, 0, None) == -2
    text = open(os.path.join(ROOT, "include", "asnn.h")).read()
    assert int(re.search(r"#define ASNN_STATIC_SCRATCH_BYTES \((\d+)u << 20\)", text).group(1)) << 20 == b.STATIC_SCRATCH_BYTES


def test_compaction_and_yardstick_argument_checks_need_no_device(lib):
    fake = ctypes.c_void_p(256)
    n = ctypes.c_int32(-1)
    assert lib.asnn_compact_workspace_bytes(-1) == 0
    big = lib.asnn_compact_workspace_bytes(1000)
    assert big > 4 * 1000 and big % 256 == 0
    assert lib.asnn_compact_required(0, fake, fake, ctypes.byref(n), fake, 1 << 20, None) == -2
    assert lib.asnn_compact_required(10, None, fake, ctypes.byref(n), fake, 1 << 20, None) == -1
    assert lib.asnn_compact_required(10, fake, fake, ctypes.byref(n), fake, 16, None) == -7
    assert lib.asnn_compact_required(10, fake, fake, ctypes.byref(n), ctypes.c_void_p(8), 1 << 20, None) == -7
    assert lib.asnn_relabel_ids(fake, -1, fake, 10, fake, None) == -2
    assert lib.asnn_relabel_ids(None, 5, fake, 10, fake, None) == -1
    assert lib.asnn_relabel_ids(None, 0, None, 10, None, None) == 0
    assert lib.asnn_device_read(None, 64, fake, None) == -1
    assert lib.asnn_device_read(fake, 63, fake, None) == -2
    assert lib.asnn_device_read(fake, 0, fake, None) == 0
    assert lib.asnn_device_gather(None, 10, 64, 4, 3, 0, fake, None) == -1
    assert lib.asnn_device_gather(fake, 10, 65, 4, 3, 0, fake, None) == -2          # rows of whole tiles only
    assert lib.asnn_device_gather(fake, 10, 64, 0, 3, 0, fake, None) == -2
    assert lib.asnn_device_gather_store(fake, 10, 64, 4, 3, 0, None, None) == -1
    assert lib.asnn_device_gather_store(fake, 10, 64, 4, 0, 0, fake, None) == -2
    assert lib.asnn_device_gather_store(fake, 10, 128, 4, 3, 0, ctypes.c_void_p(4100), None) == -2     # out is stored 8 bytes at a time
