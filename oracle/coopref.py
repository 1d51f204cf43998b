"""ctypes binding of the CPU oracle (oracle/coopref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module,
and this module never imports the product package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "coopref.c")
_LIB = os.path.join(_HERE, "libcoopref.so")
_OVERRIDE = os.environ.get("COOPREF_LIBRARY_PATH")   # another build of coopref.c (the sanitizer build), loaded as it is

NS, LABOR0, RW = 0, 1, 2
OK, E_NULL, E_RANGE, E_DUPSEED, E_ARG, E_NOMEM = 0, -1, -2, -3, -4, -5


def build(force=False):
    """Compiles coopref.c with the host C compiler (contraction off: every fma is explicit)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra", "-fPIC", "-shared",
             _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Block(C.Structure):
    _fields_ = [("n_dst", C.c_int64), ("n_src", C.c_int64), ("n_edges", C.c_int64),
                ("dst_ids", C.POINTER(C.c_int32)), ("indptr", C.POINTER(C.c_int64)),
                ("col_local", C.POINTER(C.c_int32)), ("col_global", C.POINTER(C.c_int32)),
                ("eid", C.POINTER(C.c_int64)), ("src_ids", C.POINTER(C.c_int32))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not _OVERRIDE:
            build()
        L = C.CDLL(_OVERRIDE or _LIB)
        L.coopref_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        L.coopref_philox4x32_10.restype = None
        L.coopref_mix32.argtypes = [C.c_uint32]
        L.coopref_mix32.restype = C.c_uint32
        L.coopref_layer_keys.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_uint64, C.POINTER(C.c_uint32)]
        L.coopref_layer_keys.restype = None
        L.coopref_variate.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.coopref_variate.restype = C.c_uint32
        for name in ("rcp", "rsqrt", "log", "exp", "qtail"):
            f = getattr(L, "coopref_" + name)
            f.argtypes = [C.c_double]
            f.restype = C.c_double
        L.coopref_phi_inv_u32.argtypes = [C.c_uint32]
        L.coopref_phi_inv_u32.restype = C.c_double
        L.coopref_phi_to_u32.argtypes = [C.c_double]
        L.coopref_phi_to_u32.restype = C.c_uint32
        L.coopref_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                     C.c_void_p, C.c_int, C.c_int, C.c_uint64, C.c_uint32, C.c_uint64,
                                     C.POINTER(_Block)]
        L.coopref_sample.restype = C.c_int
        L.coopref_sample_rw.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                        C.c_void_p, C.c_int, C.c_int32, C.c_int32, C.c_double, C.c_uint64, C.c_uint64,
                                        C.POINTER(_Block)]
        L.coopref_sample_rw.restype = C.c_int
        L.coopref_rw_draw.argtypes = [C.c_uint64, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32]
        L.coopref_rw_draw.restype = C.c_uint32
        L.coopref_free_blocks.argtypes = [C.POINTER(_Block), C.c_int]
        L.coopref_free_blocks.restype = None
        L.coopref_gather.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
        L.coopref_gather.restype = C.c_int
        L.coopref_gather_mean.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.coopref_gather_mean.restype = C.c_int
        L.coopref_cache_create.argtypes = [C.c_int64, C.c_int64]
        L.coopref_cache_create.restype = C.c_void_p
        L.coopref_cache_free.argtypes = [C.c_void_p]
        L.coopref_cache_free.restype = None
        L.coopref_cache_size.argtypes = [C.c_void_p]
        L.coopref_cache_size.restype = C.c_int64
        L.coopref_cache_contains.argtypes = [C.c_void_p, C.c_int32]
        L.coopref_cache_contains.restype = C.c_int
        L.coopref_cache_access.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.coopref_cache_access.restype = C.c_int64
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("coopref error %d" % code)
        self.code = code


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().coopref_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def mix32(x):
    return int(lib().coopref_mix32(int(x) & 0xFFFFFFFF))


def layer_keys(seed, sampler, layer, g):
    K = (C.c_uint32 * 4)()
    lib().coopref_layer_keys(seed, sampler, layer, g, K)
    return [int(x) for x in K]


def variate(seed, sampler, layer, it, kappa, t, s=0):
    return int(lib().coopref_variate(seed, sampler, layer, it, kappa, t, s))


def _arr(ptr, n, dtype):
    if n == 0:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dtype, copy=True)


def rw_draw(seed, layer, it, s, c):
    return int(lib().coopref_rw_draw(seed, layer, it, int(s) & 0xFFFFFFFF, int(c) & 0xFFFFFFFF))


def sample(indptr, indices, seeds, fanouts, sampler, it=0, kappa=1, seed=0, rw=None):
    """Runs L = len(fanouts) sampling layers.  Returns a list of dicts, one per layer, with
    dst_ids, indptr, col_local, col_global, eid, src_ids as numpy arrays.
    sampler RW takes rw = (walk_length, n_walks, restart_p); kappa plays no role there and eid holds visit counts."""
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    seeds = np.ascontiguousarray(seeds, dtype=np.int32)
    fan = np.ascontiguousarray(fanouts, dtype=np.int32)
    L = len(fan)
    blocks = (_Block * max(L, 1))()
    if sampler == RW:
        o, a, p = rw
        rc = lib().coopref_sample_rw(indptr.ctypes.data, indices.ctypes.data, len(indptr) - 1, len(indices),
                                     seeds.ctypes.data, len(seeds), fan.ctypes.data, L, int(o), int(a), float(p), it, seed,
                                     blocks)
    else:
        rc = lib().coopref_sample(indptr.ctypes.data, indices.ctypes.data, len(indptr) - 1, len(indices),
                                  seeds.ctypes.data, len(seeds), fan.ctypes.data, L, sampler, it, kappa, seed,
                                  blocks)
    if rc != OK:
        raise OracleError(rc)
    out = []
    for l in range(L):
        b = blocks[l]
        out.append(dict(
            dst_ids=_arr(b.dst_ids, b.n_dst, np.int32), indptr=_arr(b.indptr, b.n_dst + 1, np.int64),
            col_local=_arr(b.col_local, b.n_edges, np.int32), col_global=_arr(b.col_global, b.n_edges, np.int32),
            eid=_arr(b.eid, b.n_edges, np.int64), src_ids=_arr(b.src_ids, b.n_src, np.int32)))
    lib().coopref_free_blocks(blocks, L)
    return out


def gather(feat, ids):
    """out[i, :] = feat[ids[i], :] for a 2-D C-contiguous array of any dtype."""
    feat = np.ascontiguousarray(feat)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty((len(ids),) + feat.shape[1:], dtype=feat.dtype)
    row_bytes = feat.strides[0]
    rc = lib().coopref_gather(feat.ctypes.data, feat.shape[0], row_bytes, ids.ctypes.data, len(ids),
                              out.ctypes.data)
    if rc != OK:
        raise OracleError(rc)
    return out


def bucket_by_owner(ids, n_vertices, n_parts, scheme, seed=0):
    """(ids grouped by owner, their original positions, group offsets [n_parts + 1]); scheme 0 = ranges, 1 = hashed."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty(len(ids), dtype=np.int32)
    origin = np.empty(len(ids), dtype=np.int32)
    offsets = np.empty(n_parts + 1, dtype=np.int64)
    L = lib()
    L.coopref_bucket_by_owner.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
    L.coopref_bucket_by_owner.restype = C.c_int
    rc = L.coopref_bucket_by_owner(ids.ctypes.data, len(ids), int(n_vertices), int(n_parts), int(scheme), int(seed),
                                   out.ctypes.data, origin.ctypes.data, offsets.ctypes.data)
    if rc != OK:
        raise OracleError(rc)
    return out, origin, offsets


def gather_mean(feat, indptr, col):
    """float64 [n_dst, dim]: mean of feat[col[e], :] over the edges of every destination (0 where there are none)."""
    feat = np.ascontiguousarray(feat)
    assert feat.dtype in (np.float32, np.float16) and feat.ndim == 2
    indptr = np.ascontiguousarray(indptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    n_dst = len(indptr) - 1
    out = np.zeros((n_dst, feat.shape[1]), dtype=np.float64)
    rc = lib().coopref_gather_mean(feat.ctypes.data, feat.shape[0], feat.shape[1], 0 if feat.dtype == np.float32 else 1,
                                   indptr.ctypes.data, col.ctypes.data, n_dst, out.ctypes.data)
    if rc != OK:
        raise OracleError(rc)
    return out


class Cache:
    """Batched LRU vertex cache; access(ids) -> (n_miss, hit mask)."""

    def __init__(self, capacity, n_vertices):
        self._h = lib().coopref_cache_create(capacity, n_vertices)
        if not self._h:
            raise OracleError(E_NOMEM)

    def access(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        hit = np.zeros(len(ids), dtype=np.uint8)
        r = lib().coopref_cache_access(self._h, ids.ctypes.data, len(ids), hit.ctypes.data)
        if r < 0:
            raise OracleError(int(r))
        return int(r), hit.astype(bool)

    def size(self):
        return int(lib().coopref_cache_size(self._h))

    def contains(self, v):
        return bool(lib().coopref_cache_contains(self._h, int(v)))

    def __del__(self):
        if getattr(self, "_h", None):
            lib().coopref_cache_free(self._h)
            self._h = None
