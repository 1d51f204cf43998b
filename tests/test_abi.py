"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/coop.h declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import paper_2310_12403_amd as P
from paper_2310_12403_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "coop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(coop_[a-z0-9_]+)\s*\(", text)
    return sorted(set(n for n in names if n != "coop_alloc_fn"))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"coop_graph_load", "coop_sample", "coop_gather", "coop_strerror"} <= set(names)
    L = P.lib()
    for n in names:
        assert hasattr(L, n), n


def test_error_names():
    assert P.coop_version() >= 1
    for code in range(0, -9, -1):
        assert P.coop_strerror(code) != "unknown error"
    assert P.coop_strerror(-99) == "unknown error"


def test_host_checked_arguments():
    L = P.lib()
    h = C.c_void_p()
    assert L.coop_graph_load(None, None, 10, 0, 0, None, C.byref(h)) == -1          # NULL indptr
    assert L.coop_graph_load(None, None, 10, 0, 0, None, None) == -1                # NULL out
    assert L.coop_graph_load_with(None, None, 10, 0, 0, None, None, None, C.byref(h)) == -1   # NULL indptr, whoever allocates
    assert L.coop_graph_load_with(None, None, -1, 0, 0, None, None, None, None) == -1         # NULL out comes first
    fan = (C.c_int32 * 2)(3, 3)
    blocks = (binding._CBlock * 2)()
    assert L.coop_sample(None, None, 0, fan, 2, 0, 0, 1, 0, None, None, None, blocks) == -1   # NULL graph
    assert L.coop_gather(None, 10, 4, 7, None, 5, None, None) == -4                 # unknown dtype
    assert L.coop_gather(None, 10, 0, 0, None, 5, None, None) == -4                 # dim < 1
    assert L.coop_gather(None, 10, 4, 0, None, 0, None, None) == 0                  # nothing to do
    assert L.coop_gather(None, 10, 4, 0, None, 5, None, None) == -1                 # NULL tables


def test_bucket_by_owner_host_checks():
    L = P.lib()
    L.coop_bucket_workspace_bytes.argtypes = [C.c_int64, C.c_int]
    L.coop_bucket_workspace_bytes.restype = C.c_size_t
    L.coop_bucket_by_owner.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    need = L.coop_bucket_workspace_bytes(1000, 8)
    assert 0 < need < (1 << 22) and L.coop_bucket_workspace_bytes(1 << 30, 64) < (1 << 23)   # a few MB whatever n
    assert L.coop_bucket_workspace_bytes(1000, 0) == 0 and L.coop_bucket_workspace_bytes(1000, 65) == 0
    assert L.coop_bucket_workspace_bytes(-1, 8) == 0
    assert L.coop_bucket_by_owner(None, 10, 100, 0, 0, 0, None, None, None, None, 0, None) == -4    # no owners
    assert L.coop_bucket_by_owner(None, 10, 100, 8, 2, 0, None, None, None, None, 0, None) == -4    # unknown partition
    assert L.coop_bucket_by_owner(None, 10, 0, 8, 0, 0, None, None, None, None, 0, None) == -4      # no vertices
    assert L.coop_bucket_by_owner(None, 10, 100, 8, 0, 0, None, None, None, None, 0, None) == -1    # NULL buffers
    assert L.coop_bucket_by_owner(None, 0, 100, 8, 0, 0, None, None, 0x1000, 0x2000, 16, None) == -4  # workspace too small


def test_arena_bump_allocator():
    L = P.lib()
    a = binding._CArena(0x10000, 1000, 0)
    p1 = L.coop_arena_alloc(C.byref(a), 10, 0)
    p2 = L.coop_arena_alloc(C.byref(a), 300, 1)
    assert p1 == 0x10000 and p2 == 0x10100 and a.used == 768
    assert L.coop_arena_alloc(C.byref(a), 300, 0) is None       # would overflow: NULL, nothing consumed
    assert a.used == 768
    assert L.coop_arena_alloc(None, 8, 0) is None


def test_profile_table():
    L = P.lib()
    n = L.coop_profile_kernels()
    names = [L.coop_profile_name(i).decode() for i in range(n)]
    assert len(set(names)) == n and "gather" in names and "labor_scan" in names
    assert L.coop_profile_name(n) is None
