"""Seeded synthetic inputs: graphs, features, seed batches.

This module holds none of the sampling method's arithmetic.  It is the only
code that the CPU oracle's tests and the GPU path's tests/bench have in common:
both sides read the arrays produced here.

Graphs stand in for the paper's datasets (Table "dataset": reddit, papers100M,
mag240M ...), which are not available offline; only their shapes are used:
vertex count, edge count, a heavy-tailed degree distribution.

All randomness is a counter-based hash (splitmix64 of the element index), written
with wrapping int64 torch ops, so a given (seed, index) yields the same integer on
CPU and GPU.
"""
import math

import torch

_M64 = (1 << 64) - 1


def _s64(x):
    """Python int -> the int64 with the same low 64 bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x, s):
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def splitmix64(x):
    """splitmix64 finaliser (Steele, Lea, Flood 2014) on an int64 tensor, wrapping arithmetic."""
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


def hash_u53(idx, stream):
    """53 random bits per element of the int64 tensor idx, for the given stream id."""
    key = _s64(0xD1B54A32D192ED03 * (2 * int(stream) + 1))
    return _lsr(splitmix64(splitmix64(idx) ^ key), 11)


def uniform01(idx, stream):
    """float64 uniforms in [0, 1)."""
    return hash_u53(idx, stream).to(torch.float64) * (1.0 / (1 << 53))


def permutation(n, stream, device="cpu"):
    """A fixed pseudo-random permutation of 0..n-1 (argsort of distinct hashes)."""
    idx = torch.arange(n, dtype=torch.int64, device=device)
    h = splitmix64(idx ^ _s64(0xA0761D6478BD642F * (2 * int(stream) + 1)))  # bijection: no ties
    return torch.argsort(h)


# --------------------------------------------------------------------------- #
# edge lists
# --------------------------------------------------------------------------- #
def rmat_edges(scale, n_edges, a=0.57, b=0.19, c=0.19, d=0.05, seed=0, device="cpu", first=0):
    """R-MAT (Chakrabarti, Zhan, Faloutsos 2004): n_edges directed edges on 2^scale vertices."""
    assert abs(a + b + c + d - 1.0) < 1e-9
    e = torch.arange(first, first + n_edges, dtype=torch.int64, device=device)
    src = torch.zeros_like(e)
    dst = torch.zeros_like(e)
    for level in range(scale):
        u = uniform01(e * scale + level, 1000 + seed)
        right = (u >= a) & (u < a + b) | (u >= a + b + c)   # quadrants b, d: column bit set
        down = u >= a + b                                    # quadrants c, d: row bit set
        src = (src << 1) | down.to(torch.int64)
        dst = (dst << 1) | right.to(torch.int64)
    return src, dst


def _chung_lu_offset(n, two_m, alpha):
    """Offset i0 of the weight law w_i ~ (i + i0)^-alpha such that the largest expected degree
    is sqrt(sum of expected degrees) (the usual Chung-Lu cap)."""
    target = math.sqrt(two_m) / two_m   # probability mass of vertex 0

    def mass0(i0):
        if abs(alpha - 1.0) < 1e-12:
            return math.log((i0 + 1.0) / i0) / math.log((n + i0) / i0)
        p = 1.0 - alpha
        return ((i0 + 1.0) ** p - i0 ** p) / ((n + i0) ** p - i0 ** p)

    lo, hi = 1e-9, float(n)
    for _ in range(200):
        mid = math.sqrt(lo * hi)
        if mass0(mid) > target:
            lo = mid
        else:
            hi = mid
    return math.sqrt(lo * hi)


def chung_lu_endpoints(idx, stream, n, alpha, i0):
    """Vertex ranks drawn i.i.d. with probability ~ (rank + i0)^-alpha (inverse CDF of the
    continuous law, floored)."""
    u = uniform01(idx, stream)
    if abs(alpha - 1.0) < 1e-12:
        x = i0 * torch.exp(u * math.log((n + i0) / i0))
    else:
        p = 1.0 - alpha
        lo = i0 ** p
        x = torch.pow(lo + u * ((n + i0) ** p - lo), 1.0 / p)
    return torch.clamp((x - i0).to(torch.int64), 0, n - 1)


# --------------------------------------------------------------------------- #
# CSR construction
# --------------------------------------------------------------------------- #
def csr_from_edges(n, src, dst):
    """Symmetrise, drop self-loops and duplicates, sort: CSR with int64 indptr, int32 indices."""
    keep = src != dst
    src, dst = src[keep], dst[keep]
    keys = torch.cat([src * n + dst, dst * n + src])
    keys = torch.unique(keys)  # sorted
    rows = torch.div(keys, n, rounding_mode="floor")
    indices = (keys - rows * n).to(torch.int32)
    deg = torch.bincount(rows, minlength=n)
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=src.device)
    indptr[1:] = torch.cumsum(deg, 0)
    return indptr, indices


def rmat_csr(scale=14, n_edges=262144, seed=0, device="cpu"):
    """The tiny configuration: R-MAT (0.57, 0.19, 0.19, 0.05), symmetrised and deduplicated."""
    src, dst = rmat_edges(scale, n_edges, seed=seed, device=device)
    return csr_from_edges(1 << scale, src, dst)


def chung_lu_csr(n, m_undirected, exponent, seed=0, device="cpu", chunk=1 << 26, n_parts=None, log=None):
    """Chung-Lu power-law graph: m_undirected edges, both endpoints i.i.d. ~ w, w_i ~ (i+i0)^(-1/(exponent-1)),
    vertex ids randomly relabelled, symmetrised, deduplicated, no self-loops.

    Built in chunks and source-range partitions so that no tensor exceeds about `2*chunk` keys;
    returns (indptr int64 [n+1], indices int32 [nnz]) on `device`."""
    alpha = 1.0 / (exponent - 1.0)
    i0 = _chung_lu_offset(n, 2.0 * m_undirected, alpha)
    relabel = permutation(n, 77 + seed, device)
    if n_parts is None:
        n_parts = max(1, (2 * m_undirected + chunk - 1) // chunk)
    width = (n + n_parts - 1) // n_parts
    bounds = torch.arange(0, n_parts + 1, dtype=torch.int64, device=device) * (width * n)
    runs = [[] for _ in range(n_parts)]
    done = 0
    while done < m_undirected:
        cnt = min(chunk, m_undirected - done)
        e = torch.arange(done, done + cnt, dtype=torch.int64, device=device)
        s = relabel[chung_lu_endpoints(e, 2000 + 2 * seed, n, alpha, i0)]
        d = relabel[chung_lu_endpoints(e, 2001 + 2 * seed, n, alpha, i0)]
        keep = s != d
        s, d = s[keep], d[keep]
        keys = torch.cat([s * n + d, d * n + s])
        del e, s, d, keep
        keys = torch.sort(keys).values
        cut = torch.searchsorted(keys, bounds).tolist()
        for p in range(n_parts):
            if cut[p + 1] > cut[p]:
                runs[p].append(keys[cut[p]:cut[p + 1]].clone())
        del keys
        done += cnt
        if log:
            log("chung_lu: generated %d / %d edges" % (done, m_undirected))
    deg = torch.zeros(n, dtype=torch.int64, device=device)
    indices = torch.empty(2 * m_undirected, dtype=torch.int32, device=device)
    nnz = 0
    for p in range(n_parts):
        if not runs[p]:
            continue
        keys = torch.unique(torch.cat(runs[p]))
        runs[p] = None
        rows = torch.div(keys, n, rounding_mode="floor")
        cols = (keys - rows * n).to(torch.int32)
        lo = p * width
        hi = min(n, lo + width)
        deg[lo:hi] = torch.bincount(rows - lo, minlength=hi - lo)
        indices[nnz:nnz + cols.numel()] = cols
        nnz += cols.numel()
        del keys, rows, cols
        if log:
            log("chung_lu: merged part %d / %d" % (p + 1, n_parts))
    indptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    indptr[1:] = torch.cumsum(deg, 0)
    return indptr, indices[:nnz]


def directed_from_symmetric(indptr, indices, stream=0):
    """A directed graph out of an undirected one stored both ways: of every pair of opposite edges exactly one
    survives, chosen by a hash of the unordered pair, so that N(s) (in-neighbours) and the out-neighbourhood of s
    differ.  Lists stay ascending.  Returns (indptr int64, indices int32) on the input's device."""
    n = indptr.numel() - 1
    deg = indptr[1:] - indptr[:-1]
    rows = torch.repeat_interleave(torch.arange(n, dtype=torch.int64, device=indptr.device), deg)
    cols = indices.to(torch.int64)
    lo, hi = torch.minimum(rows, cols), torch.maximum(rows, cols)
    bit = hash_u53(lo * n + hi, 4000 + stream) & 1          # one coin per unordered pair
    keep = (bit == 1) == (rows < cols)                       # heads: the edge into the larger id survives, tails: the other
    new_deg = torch.bincount(rows[keep], minlength=n)
    out_ptr = torch.zeros(n + 1, dtype=torch.int64, device=indptr.device)
    out_ptr[1:] = torch.cumsum(new_deg, 0)
    return out_ptr, indices[keep].contiguous()


# --------------------------------------------------------------------------- #
# features, seeds
# --------------------------------------------------------------------------- #
def features(n, dim, dtype=torch.float32, seed=0, device="cpu", rows_per_chunk=1 << 22):
    """i.i.d. N(0,1) feature table [n, dim], filled chunk by chunk from a seeded generator."""
    gen = torch.Generator(device=device)
    gen.manual_seed(1234567 + seed)
    out = torch.empty((n, dim), dtype=dtype, device=device)
    for lo in range(0, n, rows_per_chunk):
        hi = min(n, lo + rows_per_chunk)
        out[lo:hi] = torch.randn((hi - lo, dim), dtype=torch.float32, device=device, generator=gen).to(dtype)
    return out


def seed_batches(n, batch, seed=0, device="cpu"):
    """A seeded permutation of V cut into consecutive batches: batch i is perm[i*batch:(i+1)*batch]
    (uniform without replacement; the paper assumes every vertex can be a training vertex)."""
    perm = permutation(n, 555 + seed, device).to(torch.int32)
    nb = n // batch

    def get(i):
        j = i % nb
        return perm[j * batch:(j + 1) * batch]

    return get


# the five benchmark configurations (shapes only)
CONFIGS = {
    "tiny": dict(kind="rmat", scale=14, edges=262144, dim=64, dtype="f32", fanouts=(10, 10, 10), batch=1024,
                 sampler="ns"),
    "products": dict(kind="chung_lu", n=2450000, m=61850000, exponent=2.1, dim=100, dtype="f32",
                     fanouts=(10, 10, 10), batch=16384, sampler="labor0"),
    "reddit": dict(kind="chung_lu", n=232965, m=57300000, exponent=2.3, dim=602, dtype="f32",
                   fanouts=(25, 10, 10), batch=8192, sampler="labor0"),
    "papers100M": dict(kind="chung_lu", n=111059956, m=1620000000, exponent=2.0, dim=128, dtype="f16",
                       fanouts=(10, 10, 10), batch=16384, sampler="labor0"),
    "mag240M": dict(kind="chung_lu", n=244160499, m=1730000000, exponent=2.0, dim=768, dtype="f16",
                    fanouts=(10, 10, 10), batch=32768, sampler="labor0"),
}


def make_graph(name, device="cpu", scale_down=1, seed=None, log=None):
    """Builds the CSR of a named configuration; scale_down > 1 shrinks vertex and edge counts alike."""
    cfg = CONFIGS[name]
    sd = list(CONFIGS).index(name) if seed is None else seed
    if cfg["kind"] == "rmat":
        return rmat_csr(cfg["scale"], cfg["edges"], seed=sd, device=device)
    return chung_lu_csr(cfg["n"] // scale_down, cfg["m"] // scale_down, cfg["exponent"], seed=sd, device=device,
                        log=log)
