"""CPU-side checks of the C ABI: the library loads, exports every symbol include/ea.h
declares, and rejects bad arguments on the host before any launch (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2510_00636_amd as ea
from oracle import ea_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ea.lib_path()):
        import __graft_entry__
        __graft_entry__.build()
    return ea.load_library()


def test_exports_every_declared_symbol(lib):
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read()
                  for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    names = set(re.findall(r"\b(ea_[a-z_0-9]+)\s*\(", hdr))
    assert {"ea_workspace_bytes", "ea_query_stats", "ea_score", "ea_select", "ea_select_static",
            "ea_compact", "ea_compress_layer", "ea_n_keep", "ea_status_string",
            "ea_compress_layer_timed", "ea_debug_status"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layout_matches_header():
    assert ctypes.sizeof(ea.EaParams) == 40
    hdr = open(os.path.join(ROOT, "include", "ea.h")).read()
    body = hdr[hdr.index("typedef struct {"):hdr.index("} ea_params;")]
    fields = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert fields == [f for f, _ in ea.EaParams._fields_]


def test_n_keep_matches_listing_truncation(lib):
    for n, r in [(1024, 0.5), (131072, 0.25), (131072, 0.75), (1000, 0.9), (7, 0.5), (10, 0.0),
                 (10, 1.0), (4608, 1 - 4096 / 4608)]:
        assert ea.n_keep(n, r) == O.n_keep(n, r)
    assert ea.n_keep(10, 1.5) == -1 and ea.n_keep(-1, 0.5) == -1


def test_status_strings(lib):
    assert ea.status_string(0) == "ok"
    assert len({ea.status_string(i) for i in range(5)}) == 5


def test_workspace_bytes_and_param_validation(lib):
    p = ea.make_params(1, 32, 8, 128, ea.EA_BF16)
    small, big = ea.workspace_bytes(p, 1024, 128), ea.workspace_bytes(p, 131072, 128)
    assert 0 < small < big < 2 ** 31
    assert ea.workspace_bytes(ea.make_params(1, 32, 8, 96, ea.EA_BF16), 1024, 128) == 0   # head_dim
    assert ea.workspace_bytes(ea.make_params(1, 30, 8, 128, ea.EA_BF16), 1024, 128) == 0  # Hq % Hkv
    assert ea.workspace_bytes(p, 0, 128) == 0 and ea.workspace_bytes(p, 1024, 0) == 0
    assert ea.workspace_bytes(p, 1024, 5000) == 0


def test_bad_arguments_are_rejected_before_any_launch(lib):
    p = ea.make_params(1, 4, 2, 64, ea.EA_F32)
    ok = 1 << 20            # fake, aligned, never dereferenced: validation fails first
    byref = ctypes.byref
    VP = ctypes.c_void_p
    # null / misaligned pointers
    assert lib.ea_score(byref(p), None, VP(ok), 8, 8, VP(ok), VP(ok), VP(ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_score(byref(p), VP(ok + 4), VP(ok), 8, 8, VP(ok), VP(ok), VP(ok), VP(ok), 1 << 30, None) == 1
    # n > n_cap, n_keep > n
    assert lib.ea_score(byref(p), VP(ok), VP(ok), 9, 8, VP(ok), VP(ok), VP(ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_select(byref(p), VP(ok), 8, 9, VP(ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_select(byref(p), VP(ok), 8, -1, VP(ok), VP(ok), 1 << 30, None) == 1
    # workspace too small / misaligned
    assert lib.ea_select(byref(p), VP(ok), 8, 4, VP(ok), VP(ok), 16, None) == 3
    assert lib.ea_select(byref(p), VP(ok), 8, 4, VP(ok), VP(ok + 16), 1 << 30, None) == 1
    # window too short for ddof, too long
    p1 = ea.make_params(1, 4, 2, 64, ea.EA_F32, cov_ddof=1)
    assert lib.ea_query_stats(byref(p1), VP(ok), 1, 0, VP(ok), 1, VP(ok), VP(ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_query_stats(byref(p), VP(ok), 5000, 0, VP(ok), 1, VP(ok), VP(ok), VP(ok), 1 << 30, None) == 2
    # unsupported head_dim / dtype; invalid epsilon
    assert lib.ea_select(byref(ea.make_params(1, 4, 2, 80, ea.EA_F32)), VP(ok), 8, 4, VP(ok), VP(ok), 1 << 30, None) == 2
    assert lib.ea_select(byref(ea.make_params(1, 4, 2, 64, 7)), VP(ok), 8, 4, VP(ok), VP(ok), 1 << 30, None) == 2
    assert lib.ea_select(byref(ea.make_params(1, 4, 2, 64, 0, epsilon=-1.0)), VP(ok), 8, 4, VP(ok), VP(ok), 1 << 30, None) == 1
    # compaction: one tensor in place and the other not; aliasing outputs
    assert lib.ea_compact(byref(p), VP(ok), VP(2 * ok), 8, 8, VP(ok), 4, VP(ok), VP(3 * ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_compact(byref(p), VP(ok), VP(2 * ok), 8, 8, VP(ok), 4, VP(3 * ok), VP(3 * ok), VP(ok), 1 << 30, None) == 1
    # compaction: outputs that overlap the inputs without being the same range
    assert lib.ea_compact(byref(p), VP(ok), VP(2 * ok), 8, 8, VP(ok), 4, VP(ok + 256), VP(3 * ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_compact(byref(p), VP(ok), VP(2 * ok), 8, 8, VP(ok), 4, VP(4 * ok), VP(2 * ok + 512), VP(ok), 1 << 30, None) == 1
    # more rows per head than the launch grids cover
    assert lib.ea_select(byref(p), VP(ok), (1 << 26) + 1, 4, VP(ok), VP(ok), 1 << 40, None) == 1
    assert ea.workspace_bytes(p, (1 << 26) + 1, 64) == 0
    # the allocation-free selection: limits of its static array, then the usual argument checks
    assert lib.ea_select_static(byref(ea.make_params(65, 1, 1, 64, ea.EA_F32)), VP(ok), 8, 4, VP(ok), None) == 2
    assert lib.ea_select_static(byref(p), VP(ok), (1 << 20) + 1, 4, VP(ok), None) == 2
    assert lib.ea_select_static(byref(p), VP(ok), 8, 9, VP(ok), None) == 1
    assert lib.ea_select_static(byref(p), VP(ok), 8, 0, None, None) == 0
    # scores with the output projection: d_model range, null norms, n > n_cap, workspace
    assert lib.ea_wo_gram(byref(p), VP(ok), 0, VP(ok), None) == 1
    assert lib.ea_wo_gram(byref(p), VP(ok), (1 << 20) + 1, VP(ok), None) == 1
    assert lib.ea_wo_gram(byref(p), None, 64, VP(ok), None) == 1
    assert lib.ea_value_norms_wo(byref(p), VP(ok), 9, 8, VP(ok), VP(ok), VP(ok), 1 << 30, None) == 1
    assert lib.ea_value_norms_wo(byref(p), VP(ok), 8, 8, VP(ok), VP(ok), VP(ok), 16, None) == 3
    assert lib.ea_score_wo(byref(p), VP(ok), VP(ok), 8, 8, VP(ok), VP(ok), None, VP(ok), VP(ok), 1 << 30, None) == 1
    # n_keep == 0 is a valid no-op (returns before any launch)
    assert lib.ea_select(byref(p), VP(ok), 8, 0, None, VP(ok), 1 << 30, None) == 0
    assert lib.ea_compact(byref(p), VP(ok), VP(2 * ok), 8, 8, None, 0, VP(ok), VP(2 * ok), VP(ok), 1 << 30, None) == 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more exits with a message instead of pretending."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_paged_arguments_are_checked_on_the_host(lib):
    """Block sizes that are not a power of two in [16, 65536], tables too short for n, null tables
    and fp32 caches are turned away before any launch (no GPU needed: the checks come first)."""
    import ctypes
    from paper_2510_00636_amd.binding import EaPaged, make_params, EA_BF16, EA_F32
    p = make_params(1, 4, 2, 128, EA_BF16)
    ws_bytes = lib.ea_workspace_bytes(ctypes.byref(p), 4096, 1)
    fake = ctypes.c_void_p(0x10000)          # never dereferenced: every call below fails its checks first

    def call(pg, n=4096, params=p):
        return lib.ea_score_paged(ctypes.byref(params), fake, fake, ctypes.byref(pg), n, fake, fake, fake, fake,
                                  ws_bytes, None)
    assert call(EaPaged(0x20000, 48, 100, 100)) == 2          # not a power of two
    assert call(EaPaged(0x20000, 8, 1000, 1000)) == 2         # below half a tile of 32 keys
    assert call(EaPaged(0x20000, 64, 10, 100)) == 1           # 10 blocks of 64 rows cannot hold 4096
    assert call(EaPaged(0, 64, 100, 100)) == 1                # no table
    assert call(EaPaged(0x20000, 64, 100, 0)) == 1            # empty pool
    assert call(EaPaged(0x20000, 64, 100, 100), params=make_params(1, 4, 2, 128, EA_F32)) == 2
