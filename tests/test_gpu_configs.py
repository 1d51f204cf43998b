"""GPU parity at the benchmark configurations' full sizes (graphs built on the GPU by synth/, the oracle run on
the host copy): products-shaped, reddit-shaped and papers100M-shaped graphs.  Every output array must equal the
oracle's byte for byte; the batch-size sweep is also checked for exact nestedness and sub-additivity."""
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import synth
from oracle import coopref as R

pytestmark = pytest.mark.gpu
NAMES = ("dst_ids", "indptr", "col_global", "eid", "col_local", "src_ids")

# The oracle is single-threaded and, with dependent variates, evaluates two Phi^-1 and a Phi in binary64 per examined
# neighbour (a full papers100M-shaped batch examines 1.2e9 of them: minutes).  The long oracle runs therefore start in
# threads of their own as soon as the host copy of the graph exists (the C call releases the interpreter lock) and are
# joined where their result is compared; the oracle itself is untouched.
_POOL = ThreadPoolExecutor(max_workers=6)


_CAPTURE = None


@pytest.fixture(autouse=True)
def _progress_lines(request):
    """note() writes past pytest's capture: the long comparisons below report every case as it is done."""
    global _CAPTURE
    _CAPTURE = request.config.pluginmanager.getplugin("capturemanager")
    yield
    _CAPTURE = None


def note(msg):
    line = "[configs %s] %s" % (time.strftime("%H:%M:%S"), msg)
    if _CAPTURE is not None:
        with _CAPTURE.global_and_fixture_disabled():
            print(line, file=sys.stderr, flush=True)
    else:
        print(line, file=sys.stderr, flush=True)


def oracle_async(ip, ix, seeds, fanouts, sampler, **kw):
    seeds_h = np.ascontiguousarray(seeds.cpu().numpy(), dtype=np.int32)
    return _POOL.submit(R.sample, ip, ix, seeds_h, fanouts, sampler, **kw)


def assert_blocks_equal(got, want, tag=""):
    assert len(got) == len(want)
    for l, (b, w) in enumerate(zip(got, want)):
        assert (b.n_dst, b.n_edges, b.n_src) == (len(w["dst_ids"]), len(w["col_global"]), len(w["src_ids"])), (tag, l)
        for name in NAMES:
            assert np.array_equal(getattr(b, name).cpu().numpy(), w[name]), (tag, l, name)


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
    """The reddit-shaped configuration at its stated workload: batch 8,192, fanouts 25/10/10, NS and LABOR-0 (and LABOR-0
    with dependent variates on the same batch), default knobs, every array against the oracle."""
    g, ip, ix = load(P, "reddit")
    n = len(ip) - 1
    assert n == 232965
    get = synth.seed_batches(n, 8192, seed=2, device="cuda")
    ns_want = oracle_async(ip, ix, get(1), (25, 10, 10), R.NS, it=4, kappa=1, seed=11)
    dep_want = oracle_async(ip, ix, get(2), (25, 10, 10), R.LABOR0, it=5, kappa=16, seed=11)
    nsdep_want = oracle_async(ip, ix, get(3)[:2048].contiguous(), (25, 10, 10), R.NS, it=6, kappa=16, seed=11)
    blocks = compare(P, g, ip, ix, get(0), (25, 10, 10), R.LABOR0, it=3, kappa=1, seed=11)
    # fp32 x 602 rows: 2408 bytes, only 8-byte aligned
    feat = synth.features(n, 602, torch.float32, seed=2, device="cuda")
    ids = blocks[-1].src_ids
    rows = P.coop_gather(feat, ids)
    P.coop_gather_status()
    pick = torch.arange(0, ids.numel(), 997, device="cuda")
    assert torch.equal(rows[pick], feat[ids[pick].long()])
    assert rows.cpu().numpy()[:2000].tobytes() == R.gather(feat.cpu().numpy(), ids[:2000].cpu().numpy()).tobytes()
    got = P.coop_sample(g, get(1), (25, 10, 10), R.NS, it=4, kappa=1, seed=11)
    assert got[0].n_dst == 8192 and got[2].n_edges > 1_000_000
    assert_blocks_equal(got, ns_want.result(), "NS 8192 x 25/10/10")
    got = P.coop_sample(g, get(2), (25, 10, 10), R.LABOR0, it=5, kappa=16, seed=11)
    assert_blocks_equal(got, dep_want.result(), "LABOR-0 kappa 16, 8192 x 25/10/10")
    got = P.coop_sample(g, get(3)[:2048].contiguous(), (25, 10, 10), R.NS, it=6, kappa=16, seed=11)
    assert_blocks_equal(got, nsdep_want.result(), "NS kappa 16, 2048 x 25/10/10")


def test_papers100m_shaped_full_batch(P):
    """The benchmark's own workload: full batches of 16,384 seeds, 3-layer LABOR-0 10/10/10, in the launch configuration
    that bench.py times (arena allocator, default knobs), every array against the oracle: independent variates
    (kappa = 1) and dependent ones at kappa = 16 and kappa = 256 inside a group (c = 5/16 and c = 200/256), where the pass
    at layer 1 covers more than 65,536 new destinations for two layers at once (several lists per wave, long lists cut
    into pieces, the three-stage filter in front of the exact blend) and the frontiers go through the partitioned
    dedup.  Then the LRU cache of the configuration (4 M rows) over consecutive dependent batches."""
    g, ip, ix = load(P, "papers100M")
    n = len(ip) - 1
    assert n == 111059956 and len(ix) > 3.2e9
    get = synth.seed_batches(n, 16384, seed=0, device="cuda")
    # dependent variates: nested prefixes of one batch at kappa = 16 (2,048 to the full 16,384 seeds) and the full batch at
    # kappa = 256; the oracle takes from one to several minutes per case, the shorter ones first
    dep = []
    for kappa, it, b in ((16, 8 * 16 + 5, 2048), (16, 8 * 16 + 5, 4096), (16, 8 * 16 + 5, 8192), (16, 8 * 16 + 5, 12288),
                         (16, 8 * 16 + 5, 16384), (256, 256 + 200, 16384)):
        seeds = get(it)[:b].contiguous()
        dep.append((kappa, it, seeds, oracle_async(ip, ix, seeds, (10, 10, 10), R.LABOR0, it=it, kappa=kappa, seed=0)))
    note("papers100M: graph on the host, %d oracle runs with dependent variates started" % len(dep))
    arena = P.Arena(4 << 30)
    compare(P, g, ip, ix, get(7), (10, 10, 10), R.LABOR0, it=7, kappa=1, seed=0, arena=arena)
    try:  # the same batch with every list scanned (the long ones cut into pieces), as on a graph not registered as symmetric
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 0)
        arena.reset()
        compare(P, g, ip, ix, get(7), (10, 10, 10), R.LABOR0, it=7, kappa=1, seed=0, arena=arena)
    finally:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 8192)
    note("papers100M: kappa 1 compared")
    compare(P, g, ip, ix, get(9)[:512].contiguous(), (10, 10), R.NS, it=9, kappa=1, seed=0)
    # dependent batches around group boundaries and at the last iteration of a 512-iteration run
    for it, kappa in ((15, 16), (16, 16), (17, 16), (255, 256), (256, 256), (257, 256), (511, 16), (511, 256)):
        compare(P, g, ip, ix, get(it)[:96].contiguous(), (10, 10), R.LABOR0, it=it, kappa=kappa, seed=0)
    # four times the batch: the last layer's frontier has some twenty million entries, thousands of dedup buckets
    big = synth.seed_batches(n, 65536, seed=1, device="cuda")(0)
    got = compare(P, g, ip, ix, big, (10, 10, 10), R.LABOR0, it=3, kappa=1, seed=0)
    assert got[2].n_dst + got[2].n_edges > 16_000_000
    note("papers100M: 65,536-seed batch compared")
    # random walks at full scale (a smaller batch: the oracle walks 300 steps per destination)
    seeds = get(10)[:2048].contiguous()
    got = P.coop_sample_rw(g, seeds, (10, 10), 3, 100, 0.5, it=10, seed=0, arena=arena)
    want = R.sample(ip, ix, seeds.cpu().numpy(), (10, 10), R.RW, it=10, seed=0, rw=(3, 100, 0.5))
    assert_blocks_equal(got, want, "RW")
    # the configuration's cache: 4 M rows in front of the fp16 x 128 table, consecutive batches of one kappa = 16 group;
    # miss counts against the oracle's LRU fed the same id lists, rows against the table
    feat = synth.features(1 << 22, 128, torch.float16, seed=4, device="cuda")      # (aliased: vertex v reads row v mod 2^22)
    cache = P.Cache(4000000, n, 128, torch.float16, max_ids=8 << 20)
    lru = R.Cache(4000000, n)
    rates = []
    for it in range(32, 38):
        arena.reset()
        ids = P.coop_sample(g, get(it), (10, 10, 10), R.LABOR0, it=it, kappa=16, seed=0, arena=arena)[-1].src_ids
        out, n_miss = cache.gather(feat, ids)
        torch.cuda.synchronize()
        want_miss, _ = lru.access(ids.cpu().numpy())
        assert n_miss == want_miss, it
        pick = torch.arange(0, ids.numel(), 1999, device="cuda")
        assert torch.equal(out[pick], feat[ids[pick].long() % (1 << 22)])
        rates.append(n_miss / ids.numel())
    assert rates[0] == 1.0 and rates[-1] < rates[1] <= 1.0
    cache.close()
    del cache, feat
    # the dependent batches, default knobs, arena allocator (the last two are what `bench.py --kappa 16 / 256` times)
    prev = None
    for kappa, it, seeds, fut in dep:
        arena.reset()
        got = P.coop_sample(g, seeds, (10, 10, 10), R.LABOR0, it=it, kappa=kappa, seed=0, arena=arena)
        if seeds.numel() == 16384:
            assert got[1].n_dst - got[0].n_dst >= 65536 and got[2].n_dst + got[2].n_edges >= 262144
        sets = [b.src_ids.clone() for b in got]
        if prev is not None and prev[0] == kappa:      # nested batches give nested vertex sets, exactly (Sec. 3.2; Thm 3.1's proof)
            for small, big in zip(prev[1], sets):
                assert bool(torch.isin(small, big).all()) and small.numel() < big.numel()
        prev = (kappa, sets)
        assert_blocks_equal(got, fut.result(), "LABOR-0 kappa %d, %d seeds" % (kappa, seeds.numel()))
        note("papers100M: kappa %d, %d seeds, iteration %d compared (|S^3| = %d)" % (kappa, seeds.numel(), it, got[2].n_src))


def test_mag240m_shaped_batch_and_host_cache(P):
    """Largest configuration: 244M vertices, ~3.45B edges in HBM, fp16 x 768 rows in pinned host memory behind the
    configuration's 32M-row LRU cache (49 GB of rows in HBM).  One full batch of 32,768 seeds against the oracle; then,
    for kappa = 1 and kappa = 64, consecutive full batches through a cache of that size: miss counts against the
    oracle's LRU, sampled rows against the host table; a dependent sub-batch of the kappa = 64 group against the oracle."""
    g, ip, ix = load(P, "mag240M")
    n = len(ip) - 1
    assert n == 244160499 and len(ix) > 3.4e9
    get = synth.seed_batches(n, 32768, seed=0, device="cuda")
    sub = get(130)[:1024].contiguous()
    dep_want = oracle_async(ip, ix, sub, (10, 10, 10), R.LABOR0, it=130, kappa=64, seed=0)
    blocks = compare(P, g, ip, ix, get(3), (10, 10, 10), R.LABOR0, it=3, kappa=1, seed=0)
    assert_blocks_equal(P.coop_sample(g, sub, (10, 10, 10), R.LABOR0, it=130, kappa=64, seed=0), dep_want.result(), "kappa 64 sub-batch")
    del ip, ix
    rows_host = 1 << 20                                    # aliased host table: vertex v reads row v mod 2^20
    table = synth.features(rows_host, 768, torch.float16, seed=9, device="cpu").pin_memory()
    arena = P.Arena(8 << 30)
    steady = {}
    for kappa in (1, 64):
        cache = P.Cache(32000000, n, 768, torch.float16, max_ids=8 << 20)
        oracle = R.Cache(32000000, n)
        rates = []
        for it in range(128, 132):                          # (kappa = 64: the first iterations of group 2)
            arena.reset()
            ids = P.coop_sample(g, get(it), (10, 10, 10), R.LABOR0, it=it, kappa=kappa, seed=0, arena=arena)[-1].src_ids
            out, n_miss = cache.gather(table, ids)
            torch.cuda.synchronize()
            want, _ = oracle.access(ids.cpu().numpy())
            assert n_miss == want, (kappa, it)
            pick = torch.arange(0, ids.numel(), 4099, device="cuda")
            assert torch.equal(out[pick].cpu(), table[(ids[pick].long() % rows_host).cpu()])
            rates.append(n_miss / ids.numel())
        steady[kappa] = rates[-1]
        cache.close()
        del cache, oracle
    assert steady[64] < steady[1]     # dependent batches share most of their input vertices (Sec. 3.2)
