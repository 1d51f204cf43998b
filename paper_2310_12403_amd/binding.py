"""ctypes binding of libcoop.so (see include/coop.h for the contract of every call)."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# (COOP_LIBRARY_PATH: another build of the same sources, e.g. the host-sanitizer build of `python -m paper_2310_12403_amd.build --sanitize`)
_LIB_PATH = os.environ.get("COOP_LIBRARY_PATH") or os.path.join(_HERE, "libcoop.so")

COOP_NS, COOP_LABOR0, COOP_RW = 0, 1, 2
COOP_F32, COOP_F16 = 0, 1
COOP_VALIDATE = 1
COOP_SYMMETRIC = 2
TAG_OUTPUT, TAG_SCRATCH = 0, 1

ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_void_p, C.c_size_t, C.c_int)


class _CBlock(C.Structure):
    _fields_ = [("n_dst", C.c_int64), ("n_src", C.c_int64), ("n_edges", C.c_int64),
                ("dst_ids", C.c_void_p), ("indptr", C.c_void_p), ("col_local", C.c_void_p),
                ("col_global", C.c_void_p), ("eid", C.c_void_p), ("src_ids", C.c_void_p)]


class _CArena(C.Structure):
    _fields_ = [("base", C.c_void_p), ("bytes", C.c_size_t), ("used", C.c_size_t)]


class _CCacheState(C.Structure):
    _fields_ = [("size", C.c_int64), ("clock", C.c_uint64), ("base", C.c_uint64)]


_lib = None


def lib():
    """Loads libcoop.so; fails loudly when it is missing (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libcoop.so is not built: run `python -m paper_2310_12403_amd.build` "
                          "(hipcc, --offload-arch=gfx950) before using paper_2310_12403_amd")
    L = C.CDLL(_LIB_PATH)
    L.coop_strerror.argtypes = [C.c_int]
    L.coop_strerror.restype = C.c_char_p
    L.coop_version.restype = C.c_int
    L.coop_arena_alloc.argtypes = [C.c_void_p, C.c_size_t, C.c_int]
    L.coop_arena_alloc.restype = C.c_void_p
    L.coop_graph_load.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p,
                                  C.POINTER(C.c_void_p)]
    L.coop_graph_load.restype = C.c_int
    L.coop_graph_load_with.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.POINTER(C.c_void_p)]
    L.coop_graph_load_with.restype = C.c_int
    L.coop_graph_free.argtypes = [C.c_void_p]
    L.coop_graph_free.restype = C.c_int
    L.coop_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int, C.c_int, C.c_uint64,
                              C.c_uint32, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_CBlock)]
    L.coop_sample.restype = C.c_int
    L.coop_sample_rw.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(C.c_int32), C.c_int, C.c_int32, C.c_int32, C.c_double,
                                 C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_CBlock)]
    L.coop_sample_rw.restype = C.c_int
    L.coop_copy_ids.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    L.coop_copy_ids.restype = C.c_int
    L.coop_gather.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    L.coop_gather.restype = C.c_int
    L.coop_gather_mean.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    L.coop_gather_mean.restype = C.c_int
    L.coop_gather_status.argtypes = [C.c_void_p]
    L.coop_gather_status.restype = C.c_int
    L.coop_cache_create.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.POINTER(C.c_void_p)]
    L.coop_cache_create.restype = C.c_int
    L.coop_cache_free.argtypes = [C.c_void_p]
    L.coop_cache_gather.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.POINTER(C.c_int64), C.c_void_p]
    L.coop_cache_gather.restype = C.c_int
    L.coop_cache_vertices.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_int64)]
    L.coop_cache_vertices.restype = C.c_int
    L.coop_cache_export.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_CCacheState), C.c_void_p]
    L.coop_cache_export.restype = C.c_int
    L.coop_cache_import.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.POINTER(_CCacheState), C.c_void_p]
    L.coop_cache_import.restype = C.c_int
    L.coop_map_host_pointer.argtypes = [C.c_void_p, C.POINTER(C.c_void_p)]
    L.coop_map_host_pointer.restype = C.c_int
    L.coop_tune.argtypes = [C.c_int, C.c_int64]
    L.coop_tune.restype = C.c_int
    L.coop_profile_enable.argtypes = [C.c_int]
    L.coop_profile_filter.argtypes = [C.c_int]
    L.coop_profile_reset.argtypes = []
    L.coop_profile_kernels.restype = C.c_int
    L.coop_profile_name.argtypes = [C.c_int]
    L.coop_profile_name.restype = C.c_char_p
    L.coop_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _lib = L
    return L


class CoopError(RuntimeError):
    def __init__(self, code):
        super().__init__("libcoop: %s (%d)" % (coop_strerror(code), code))
        self.code = code


def _check(rc):
    if rc != 0:
        raise CoopError(rc)


def coop_strerror(code):
    return lib().coop_strerror(code).decode()


def coop_version():
    return lib().coop_version()


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dev_ptr(t, dtype):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype)
    return C.c_void_p(t.data_ptr())


class Graph:
    """Handle of a CSR graph registered with coop_graph_load; keeps the tensors alive."""

    def __init__(self, handle, indptr, indices):
        self.handle, self.indptr, self.indices = handle, indptr, indices
        self.n_vertices = indptr.numel() - 1
        self.n_edges = indices.numel()

    def close(self):
        if self.handle:
            lib().coop_graph_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def coop_graph_load(indptr, indices, flags=0, stream=None, torch_memory=False):
    """indptr: cuda int64 [n+1]; indices: cuda int32 [nnz] (borrowed for the life of the Graph).
    torch_memory: what the library builds on the graph (the reverse index of a COOP_SYMMETRIC graph) comes from torch's
    allocator through coop_graph_load_with and lives as long as the Graph object."""
    h = C.c_void_p()
    if torch_memory:
        al = _TorchAllocator(indptr.device)
        rc = lib().coop_graph_load_with(_dev_ptr(indptr, torch.int64), _dev_ptr(indices, torch.int32), indptr.numel() - 1,
                                        indices.numel(), flags, al.fn, al.ctx, _stream_ptr(stream), C.byref(h))
        if rc != 0 and al.error is not None:
            raise al.error
        _check(rc)
        g = Graph(h, indptr, indices)
        g._memory = al          # the tensors behind the handle
        return g
    rc = lib().coop_graph_load(_dev_ptr(indptr, torch.int64), _dev_ptr(indices, torch.int32), indptr.numel() - 1,
                               indices.numel(), flags, _stream_ptr(stream), C.byref(h))
    _check(rc)
    return Graph(h, indptr, indices)


class Arena:
    """One preallocated device buffer handed to the library's bump allocator (coop_arena_alloc):
    no allocation, and no Python, runs inside coop_sample.  reset() recycles it."""

    def __init__(self, nbytes, device="cuda"):
        self.buf = torch.empty(int(nbytes), dtype=torch.uint8, device=device)
        base = self.buf.data_ptr()
        self._off = (-base) % 256
        self.c = _CArena(base + self._off, int(nbytes) - self._off, 0)
        self.fn = C.cast(lib().coop_arena_alloc, C.c_void_p)
        self.ctx = C.cast(C.pointer(self.c), C.c_void_p)

    def reset(self):
        self.c.used = 0

    def view(self, ptr, count, dtype):
        if count == 0:
            return torch.empty(0, dtype=dtype, device=self.buf.device)
        off = ptr - self.buf.data_ptr()
        nbytes = count * torch.empty(0, dtype=dtype).element_size()
        return self.buf[off:off + nbytes].view(dtype)


class _TorchAllocator:
    """coop_alloc_fn backed by torch.empty: every buffer is an ordinary torch tensor."""

    def __init__(self, device):
        self.device = device
        self.tensors = {}
        self.error = None

        def _alloc(ctx, nbytes, tag):
            try:
                t = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=self.device)
                p = t.data_ptr()
                p += (-p) % 256
                self.tensors[p] = t
                return p
            except Exception as e:  # never let an exception cross the C boundary
                self.error = e
                return None

        self.fn_obj = ALLOC_FN(_alloc)
        self.fn = C.cast(self.fn_obj, C.c_void_p)
        self.ctx = C.c_void_p()

    def view(self, ptr, count, dtype):
        if count == 0:
            return torch.empty(0, dtype=dtype, device=self.device)
        t = self.tensors[ptr]
        off = ptr - t.data_ptr()
        nbytes = count * torch.empty(0, dtype=dtype).element_size()
        return t[off:off + nbytes].view(dtype)


class Block:
    """One sampled layer.  n_dst / n_src / n_edges are plain ints; dst_ids, indptr, col_local, col_global, eid and
    src_ids are tensors over the memory that the allocator handed out, built on first access (so that a caller
    that only needs the input vertex set pays for one view, not six per layer)."""
    _FIELDS = {"dst_ids": ("n_dst", 0, torch.int32), "indptr": ("n_dst", 1, torch.int64), "col_local": ("n_edges", 0, torch.int32),
               "col_global": ("n_edges", 0, torch.int32), "eid": ("n_edges", 0, torch.int64), "src_ids": ("n_src", 0, torch.int32)}

    def __init__(self, cblock, allocator):
        self.n_dst, self.n_src, self.n_edges = cblock.n_dst, cblock.n_src, cblock.n_edges
        self._ptr = {name: getattr(cblock, name) for name in self._FIELDS}
        self._alloc = allocator

    def __getattr__(self, name):
        fields = type(self)._FIELDS
        if name not in fields:
            raise AttributeError(name)
        count_of, extra, dtype = fields[name]
        t = self._alloc.view(self._ptr[name], getattr(self, count_of) + extra, dtype)
        self.__dict__[name] = t
        return t


def coop_sample(graph, seeds, fanouts, sampler, it=0, kappa=1, seed=0, arena=None, stream=None):
    """Runs L = len(fanouts) sampling layers; returns a list of Block (layer 0 first).
    With `arena` all device memory comes from that preallocated buffer (and scratch shares it)."""
    L = len(fanouts)
    fan = (C.c_int32 * max(L, 1))(*[int(k) for k in fanouts])
    blocks = (_CBlock * max(L, 1))()
    al = arena if arena is not None else _TorchAllocator(seeds.device)
    rc = lib().coop_sample(graph.handle, _dev_ptr(seeds, torch.int32), seeds.numel(), fan, L, sampler, it, kappa, seed,
                           al.fn, al.ctx, _stream_ptr(stream), blocks)
    if rc != 0 and getattr(al, "error", None) is not None:
        raise al.error
    _check(rc)
    return [Block(blocks[l], al) for l in range(L)]


def coop_sample_rw(graph, seeds, fanouts, walk_length, n_walks, restart_p, it=0, seed=0, arena=None, stream=None):
    """Random-walk sampling: as coop_sample, with n_walks walks of walk_length steps per destination and restart
    probability restart_p; a block's eid holds visit counts."""
    L = len(fanouts)
    fan = (C.c_int32 * max(L, 1))(*[int(k) for k in fanouts])
    blocks = (_CBlock * max(L, 1))()
    al = arena if arena is not None else _TorchAllocator(seeds.device)
    rc = lib().coop_sample_rw(graph.handle, _dev_ptr(seeds, torch.int32), seeds.numel(), fan, L, int(walk_length), int(n_walks),
                              float(restart_p), it, seed, al.fn, al.ctx, _stream_ptr(stream), blocks)
    if rc != 0 and getattr(al, "error", None) is not None:
        raise al.error
    _check(rc)
    return [Block(blocks[l], al) for l in range(L)]


COOP_OWNER_RANGE, COOP_OWNER_HASH = 0, 1


def coop_bucket_by_owner(ids, n_vertices, n_parts, scheme=COOP_OWNER_RANGE, seed=0, want_origin=True, workspace=None, stream=None):
    """The ids grouped by owner (stable): returns (ids_out, origin_out or None, offsets int64 [n_parts + 1]), all on the device."""
    L = lib()
    L.coop_bucket_workspace_bytes.argtypes = [C.c_int64, C.c_int]
    L.coop_bucket_workspace_bytes.restype = C.c_size_t
    L.coop_bucket_by_owner.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.coop_bucket_by_owner.restype = C.c_int
    n = ids.numel()
    need = L.coop_bucket_workspace_bytes(n, n_parts)
    if need == 0:
        raise CoopError(-4)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=ids.device)
    assert workspace.numel() * workspace.element_size() >= need
    out = torch.empty_like(ids)
    origin = torch.empty_like(ids) if want_origin else None
    offsets = torch.empty(n_parts + 1, dtype=torch.int64, device=ids.device)
    rc = L.coop_bucket_by_owner(_dev_ptr(ids, torch.int32) if n else None, n, n_vertices, n_parts, scheme, seed,
                                C.c_void_p(out.data_ptr()) if n else None, C.c_void_p(origin.data_ptr()) if want_origin and n else None,
                                C.c_void_p(offsets.data_ptr()), C.c_void_p(workspace.data_ptr()),
                                workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(rc)
    return out, origin, offsets


def coop_bucket_by_owner_static(ids, n_vertices, n_parts, scheme=COOP_OWNER_RANGE, seed=0, out=None, origin=None, offsets=None,
                                stream=None):
    """coop_bucket_by_owner without a workspace and without any allocation inside the library (its scratch is a device array
    of the library).  `out`, `origin`, `offsets` may be preallocated tensors (then nothing at all is allocated); returns
    (ids_out, origin_out, offsets)."""
    L = lib()
    L.coop_bucket_by_owner_static.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]
    L.coop_bucket_by_owner_static.restype = C.c_int
    n = ids.numel()
    if out is None:
        out = torch.empty_like(ids)
    if origin is None:
        origin = torch.empty_like(ids)
    if offsets is None:
        offsets = torch.empty(n_parts + 1, dtype=torch.int64, device=ids.device)
    assert out.numel() >= n and origin.numel() >= n and offsets.numel() >= n_parts + 1
    rc = L.coop_bucket_by_owner_static(_dev_ptr(ids, torch.int32) if n else None, n, n_vertices, n_parts, scheme, seed,
                                       C.c_void_p(out.data_ptr()) if n else None, C.c_void_p(origin.data_ptr()) if n else None,
                                       C.c_void_p(offsets.data_ptr()), _stream_ptr(stream))
    _check(rc)
    return out, origin, offsets


def coop_copy_ids(ids, out=None, stream=None):
    """A plain copy of a device int32 list on the stream."""
    if out is None:
        out = torch.empty_like(ids)
    assert out.numel() == ids.numel()
    _check(lib().coop_copy_ids(_dev_ptr(ids, torch.int32), _dev_ptr(out, torch.int32), ids.numel(), _stream_ptr(stream)))
    return out


_DTYPES = {torch.float32: COOP_F32, torch.float16: COOP_F16}


def coop_gather(feat, ids, out=None, stream=None):
    """out[i, :] = feat[ids[i], :]; feat: [n, dim] fp32/fp16 (device, or pinned host memory mapped to the device)."""
    assert feat.dim() == 2 and feat.is_contiguous() and feat.dtype in _DTYPES
    n, dim = feat.shape
    if out is None:
        out = torch.empty((ids.numel(), dim), dtype=feat.dtype, device=ids.device)
    # `out` may have more rows than there are ids (a buffer sized once and reused): the first ids.numel() rows are written
    assert out.is_contiguous() and out.dtype == feat.dtype and out.dim() == 2 and out.shape[1] == dim and out.shape[0] >= ids.numel()
    rc = lib().coop_gather(C.c_void_p(feat.data_ptr()), n, dim, _DTYPES[feat.dtype], _dev_ptr(ids, torch.int32), ids.numel(),
                           C.c_void_p(out.data_ptr()), _stream_ptr(stream))
    _check(rc)
    return out


def coop_gather_mean(feat, indptr, col_global, out=None, stream=None):
    """out[i, :] = mean of feat[col_global[e], :] over e in [indptr[i], indptr[i+1]) (fp32 accumulation, feat's dtype out)."""
    assert feat.dim() == 2 and feat.is_contiguous() and feat.dtype in _DTYPES
    n, dim = feat.shape
    n_dst = indptr.numel() - 1
    if out is None:
        out = torch.empty((n_dst, dim), dtype=feat.dtype, device=indptr.device)
    assert out.is_contiguous() and out.dtype == feat.dtype and tuple(out.shape) == (n_dst, dim)
    rc = lib().coop_gather_mean(C.c_void_p(feat.data_ptr()), n, dim, _DTYPES[feat.dtype], _dev_ptr(indptr, torch.int64),
                                _dev_ptr(col_global, torch.int32), n_dst, C.c_void_p(out.data_ptr()), _stream_ptr(stream))
    _check(rc)
    return out


def coop_gather_status(stream=None):
    _check(lib().coop_gather_status(_stream_ptr(stream)))


def coop_map_host_pointer(t):
    """Device-side address of a pinned host tensor (raises CoopError if the memory is not mapped)."""
    d = C.c_void_p()
    _check(lib().coop_map_host_pointer(C.c_void_p(t.data_ptr()), C.byref(d)))
    return d.value


class Cache:
    """LRU vertex cache (coop_cache_*).  The backing table may be a cuda tensor or a pinned host tensor."""

    def __init__(self, capacity_rows, n_vertices, dim, dtype, max_ids, device="cuda", stream=None):
        self._alloc = _TorchAllocator(torch.device(device))
        self.capacity, self.n_vertices, self.dim, self.dtype, self.max_ids = capacity_rows, n_vertices, dim, dtype, max_ids
        h = C.c_void_p()
        rc = lib().coop_cache_create(capacity_rows, n_vertices, dim, _DTYPES[dtype], max_ids, self._alloc.fn, self._alloc.ctx,
                                     _stream_ptr(stream), C.byref(h))
        if rc != 0 and self._alloc.error is not None:
            raise self._alloc.error
        _check(rc)
        self.handle = h
        self._tables = {}

    def _table_ptr(self, table):
        assert table.dim() == 2 and table.is_contiguous() and table.dtype == self.dtype and table.shape[1] == self.dim
        if table.is_cuda:
            return table.data_ptr()
        key = table.data_ptr()
        if key not in self._tables:
            assert table.is_pinned(), "a host feature table must be pinned (page-locked)"
            self._tables[key] = coop_map_host_pointer(table)
        return self._tables[key]

    def gather(self, table, ids, out=None, stream=None):
        """Returns (out, n_miss)."""
        if out is None:
            out = torch.empty((ids.numel(), self.dim), dtype=self.dtype, device=ids.device)
        n_miss = C.c_int64()
        rc = lib().coop_cache_gather(self.handle, C.c_void_p(self._table_ptr(table)), table.shape[0], _dev_ptr(ids, torch.int32), ids.numel(),
                                     C.c_void_p(out.data_ptr()), C.byref(n_miss), _stream_ptr(stream))
        _check(rc)
        return out, n_miss.value

    def vertices(self):
        """Sorted tensor of the vertex ids currently cached."""
        p, n = C.c_void_p(), C.c_int64()
        _check(lib().coop_cache_vertices(self.handle, C.byref(p), C.byref(n)))
        v = self._alloc.view(p.value, self.capacity, torch.int32)
        v = v[v >= 0]
        assert v.numel() == n.value
        return torch.sort(v).values

    def export_state(self, stream=None):
        """(vertices int32 [size], stamps int64 [size] (bit pattern of the uint64 stamps), (size, clock, base))."""
        v = torch.empty(max(self.capacity, 1), dtype=torch.int32, device=self._alloc.device)
        st = torch.empty(max(self.capacity, 1), dtype=torch.int64, device=self._alloc.device)
        state = _CCacheState()
        _check(lib().coop_cache_export(self.handle, C.c_void_p(v.data_ptr()), C.c_void_p(st.data_ptr()), C.byref(state),
                                       _stream_ptr(stream)))
        return v[:state.size].clone(), st[:state.size].clone(), (state.size, state.clock, state.base)

    def import_state(self, table, vertices, stamps, state, stream=None):
        cs = _CCacheState(*state)
        _check(lib().coop_cache_import(self.handle, C.c_void_p(self._table_ptr(table)), table.shape[0],
                                       _dev_ptr(vertices, torch.int32), _dev_ptr(stamps, torch.int64), C.byref(cs), _stream_ptr(stream)))

    def close(self):
        if self.handle:
            lib().coop_cache_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def coop_selftest_phi_inv_gap(first=0, count=1 << 32, stream=None):
    """(largest |fp32 Phi^-1 - binary64 Phi^-1| over the uniforms first .. first + count - 1, the smallest uniform that reaches it)."""
    L = lib()
    L.coop_selftest_phi_inv_gap.argtypes = [C.c_uint64, C.c_uint64, C.POINTER(C.c_double), C.POINTER(C.c_uint32), C.c_void_p, C.c_void_p]
    L.coop_selftest_phi_inv_gap.restype = C.c_int
    work = torch.empty(2, dtype=torch.int64, device="cuda")
    gap, arg = C.c_double(), C.c_uint32()
    _check(L.coop_selftest_phi_inv_gap(first, count, C.byref(gap), C.byref(arg), C.c_void_p(work.data_ptr()), _stream_ptr(stream)))
    return gap.value, arg.value


COOP_TUNE_STAGE_CAP = 1
COOP_TUNE_LISTS_PER_WAVE = 2
COOP_TUNE_FUSE_LAYERS = 3
COOP_TUNE_PIECE_LEN = 4
COOP_TUNE_BLEND_CANDIDATES = 5
COOP_TUNE_DEFER_SIZES = 6
COOP_TUNE_UNIQUE = 7
COOP_TUNE_ENUM_DEGREE = 8
COOP_TUNE_NS_LONG_LIST = 9
COOP_TUNE_SPLIT_MIN = 10


def coop_tune(knob, value):
    _check(lib().coop_tune(knob, value))


def profile_enable(on=True):
    lib().coop_profile_enable(1 if on else 0)


def profile_filter(name=None):
    """Times only the named kernel while profiling is on (None: all kernels)."""
    L = lib()
    ids = {L.coop_profile_name(i).decode(): i for i in range(L.coop_profile_kernels())}
    _check(L.coop_profile_filter(-1 if name is None else ids[name]))


def profile_reset():
    lib().coop_profile_reset()


def profile_read_all():
    """{kernel name: (total ms, launches)} for kernels launched while profiling was on."""
    L = lib()
    out = {}
    for i in range(L.coop_profile_kernels()):
        ms, n = C.c_double(), C.c_int64()
        L.coop_profile_read(i, C.byref(ms), C.byref(n))
        if n.value:
            out[L.coop_profile_name(i).decode()] = (ms.value, n.value)
    return out
