"""GPU parity at the benchmark configurations' full sizes (graphs built on the GPU by synth/, the oracle run on
the host copy): products-shaped, reddit-shaped and papers100M-shaped graphs.  Every output array must equal the
oracle's byte for byte; the batch-size sweep is also checked for exact nestedness and sub-additivity."""
import numpy as np
import pytest
import torch

import synth
from oracle import coopref as R

pytestmark = pytest.mark.gpu
NAMES = ("dst_ids", "indptr", "col_global", "eid", "col_local", "src_ids")


@pytest.fixture(scope="module")
def P():
    import paper_2310_12403_amd as P
    return P


def load(P, name):
    indptr, indices = synth.make_graph(name, device="cuda")
    # (the generator's graphs store every edge both ways in sorted lists: registered as such, as bench.py does, so that
    # LABOR-0 with independent variates takes the path that bench.py times)
    g = P.coop_graph_load(indptr, indices, P.COOP_VALIDATE | P.COOP_SYMMETRIC)
    return g, indptr.cpu().numpy(), indices.cpu().numpy()


def compare(P, g, ip, ix, seeds, fanouts, sampler, arena=None, **kw):
    got = P.coop_sample(g, seeds.cuda(), fanouts, sampler, arena=arena, **kw)
    want = R.sample(ip, ix, seeds.cpu().numpy(), fanouts, sampler, **kw)
    for l, (b, w) in enumerate(zip(got, want)):
        for name in NAMES:
            assert np.array_equal(getattr(b, name).cpu().numpy(), w[name]), (l, name)
    return got


def test_products_shaped_labor0_and_sweep(P):
    g, ip, ix = load(P, "products")
    n = len(ip) - 1
    assert n == 2450000 and 1.2e8 < len(ix) < 1.24e8
    perm = synth.permutation(n, 900, device="cuda").to(torch.int32)
    compare(P, g, ip, ix, perm[:16384].contiguous(), (10, 10, 10), R.LABOR0, it=0, kappa=1, seed=0)
    # nested prefixes: S^l of the smaller batch is a subset, |S^l| is monotone and sub-additive (exactly)
    sizes = {}
    for b in (1024, 4096, 16384, 65536):
        blocks = P.coop_sample(g, perm[:b].contiguous(), (10, 10, 10), R.LABOR0, it=0, kappa=1, seed=0)
        sizes[b] = [blk.src_ids for blk in blocks]
    for small, big in ((1024, 4096), (4096, 16384), (16384, 65536)):
        for a, c in zip(sizes[small], sizes[big]):
            assert bool(torch.isin(a, c).all()) and a.numel() <= c.numel() <= 4 * a.numel()
    # two disjoint halves against their union
    A = P.coop_sample(g, perm[:2048].contiguous(), (10, 10, 10), R.LABOR0, it=0, kappa=1, seed=0)
    B = P.coop_sample(g, perm[2048:4096].contiguous(), (10, 10, 10), R.LABOR0, it=0, kappa=1, seed=0)
    for a, b, u in zip(A, B, sizes[4096]):
        union = torch.unique(torch.cat([a.src_ids, b.src_ids]))
        assert torch.equal(union, torch.unique(u))


def test_reddit_shaped_both_samplers_and_wide_rows(P):
    g, ip, ix = load(P, "reddit")
    n = len(ip) - 1
    assert n == 232965
    get = synth.seed_batches(n, 8192, seed=2, device="cuda")
    blocks = compare(P, g, ip, ix, get(0), (25, 10, 10), R.LABOR0, it=3, kappa=1, seed=11)
    compare(P, g, ip, ix, get(1)[:512].contiguous(), (25, 10), R.NS, it=4, kappa=1, seed=11)
    compare(P, g, ip, ix, get(2)[:256].contiguous(), (25, 10), R.LABOR0, it=5, kappa=16, seed=11)
    # fp32 x 602 rows: 2408 bytes, only 8-byte aligned
    feat = synth.features(n, 602, torch.float32, seed=2, device="cuda")
    ids = blocks[-1].src_ids
    rows = P.coop_gather(feat, ids)
    P.coop_gather_status()
    pick = torch.arange(0, ids.numel(), 997, device="cuda")
    assert torch.equal(rows[pick], feat[ids[pick].long()])
    assert rows.cpu().numpy()[:2000].tobytes() == R.gather(feat.cpu().numpy(), ids[:2000].cpu().numpy()).tobytes()


def test_papers100m_shaped_full_batch(P):
    """The benchmark's own workload: one full batch of 16,384 seeds, 3-layer LABOR-0, in the launch configuration that
    bench.py times (arena allocator), all arrays against the oracle; then a dependent batch at kappa = 16."""
    g, ip, ix = load(P, "papers100M")
    n = len(ip) - 1
    assert n == 111059956 and len(ix) > 3.2e9
    get = synth.seed_batches(n, 16384, seed=0, device="cuda")
    arena = P.Arena(4 << 30)
    compare(P, g, ip, ix, get(7), (10, 10, 10), R.LABOR0, it=7, kappa=1, seed=0, arena=arena)
    try:  # the same batch with every list scanned (the long ones cut into pieces), as on a graph not registered as symmetric
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 0)
        arena.reset()
        compare(P, g, ip, ix, get(7), (10, 10, 10), R.LABOR0, it=7, kappa=1, seed=0, arena=arena)
    finally:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 8192)
    compare(P, g, ip, ix, get(8)[:1024].contiguous(), (10, 10), R.LABOR0, it=8 * 16 + 5, kappa=16, seed=0)
    compare(P, g, ip, ix, get(9)[:512].contiguous(), (10, 10), R.NS, it=9, kappa=1, seed=0)
    # dependent batches around group boundaries and at the last iteration of a 512-iteration run
    for it, kappa in ((15, 16), (16, 16), (17, 16), (255, 256), (256, 256), (257, 256), (511, 16), (511, 256)):
        compare(P, g, ip, ix, get(it)[:96].contiguous(), (10, 10), R.LABOR0, it=it, kappa=kappa, seed=0)
    # four times the batch: the last layer's frontier has some twenty million entries, thousands of dedup buckets
    big = synth.seed_batches(n, 65536, seed=1, device="cuda")(0)
    got = compare(P, g, ip, ix, big, (10, 10, 10), R.LABOR0, it=3, kappa=1, seed=0)
    assert got[2].n_dst + got[2].n_edges > 16_000_000
    # random walks at full scale (a smaller batch: the oracle walks 300 steps per destination)
    seeds = get(10)[:2048].contiguous()
    got = P.coop_sample_rw(g, seeds, (10, 10), 3, 100, 0.5, it=10, seed=0, arena=arena)
    want = R.sample(ip, ix, seeds.cpu().numpy(), (10, 10), R.RW, it=10, seed=0, rw=(3, 100, 0.5))
    for l, (b, w) in enumerate(zip(got, want)):
        for name in NAMES:
            assert np.array_equal(getattr(b, name).cpu().numpy(), w[name]), (l, name)


def test_mag240m_shaped_batch_and_host_cache(P):
    """Largest configuration: 244M vertices, ~3.45B edges in HBM, fp16 x 768 rows in pinned host memory behind the
    LRU cache.  One full batch against the oracle, then two consecutive batches through the cache: miss counts
    against the oracle LRU and sampled rows against the host table."""
    g, ip, ix = load(P, "mag240M")
    n = len(ip) - 1
    assert n == 244160499 and len(ix) > 3.4e9
    get = synth.seed_batches(n, 32768, seed=0, device="cuda")
    blocks = compare(P, g, ip, ix, get(3), (10, 10, 10), R.LABOR0, it=3, kappa=1, seed=0)
    del ip, ix
    rows_host = 1 << 20                                    # aliased host table: vertex v reads row v mod 2^20
    table = synth.features(rows_host, 768, torch.float16, seed=9, device="cpu").pin_memory()
    cache = P.Cache(2000000, n, 768, torch.float16, max_ids=8 << 20)
    oracle = R.Cache(2000000, n)
    for it in (3, 4):
        ids = P.coop_sample(g, get(it), (10, 10, 10), R.LABOR0, it=it, kappa=4, seed=0)[-1].src_ids if it != 3 else blocks[-1].src_ids
        out, n_miss = cache.gather(table, ids)
        torch.cuda.synchronize()
        want, _ = oracle.access(ids.cpu().numpy())
        assert n_miss == want
        pick = torch.arange(0, ids.numel(), 4099, device="cuda")
        assert torch.equal(out[pick].cpu(), table[(ids[pick].long() % rows_host).cpu()])
    cache.close()
