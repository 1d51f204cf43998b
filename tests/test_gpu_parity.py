"""GPU parity: every array that libcoop produces must equal the CPU oracle's, byte for byte,
on the same seeded synthetic inputs.  All calls go through the C ABI (ctypes binding)."""
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


class G:
    def __init__(self, P, indptr, indices, flags=None):
        self.indptr_h = indptr.cpu().numpy()
        self.indices_h = indices.cpu().numpy()
        self.indptr_d = indptr.cuda()
        self.indices_d = indices.cuda()
        self.graph = P.coop_graph_load(self.indptr_d, self.indices_d, P.COOP_VALIDATE if flags is None else flags)
        self.n = len(self.indptr_h) - 1


@pytest.fixture(scope="module")
def tiny(P):
    return G(P, *synth.rmat_csr())


@pytest.fixture(scope="module")
def medium(P):
    # products-shaped, 1/50 scale: 49,000 vertices, mean degree ~50, hubs of a few thousand
    return G(P, *synth.chung_lu_csr(49000, 1237000, 2.1, seed=1))


def compare(P, g, seeds, fanouts, sampler, it=0, kappa=1, seed=0, arena=None):
    seeds_h = np.ascontiguousarray(seeds, dtype=np.int32)
    want = R.sample(g.indptr_h, g.indices_h, seeds_h, fanouts, sampler, it=it, kappa=kappa, seed=seed)
    got = P.coop_sample(g.graph, torch.from_numpy(seeds_h).cuda(), fanouts, sampler, it=it, kappa=kappa, seed=seed,
                        arena=arena)
    assert len(got) == len(want)
    for l, (b, w) in enumerate(zip(got, want)):
        assert (b.n_dst, b.n_edges, b.n_src) == (len(w["dst_ids"]), len(w["col_global"]), len(w["src_ids"])), l
        for name in NAMES:
            a = getattr(b, name).cpu().numpy()
            assert a.dtype == w[name].dtype and np.array_equal(a, w[name]), (l, name)
    return got


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_tiny_config_three_layers(P, tiny, sampler):
    seeds = synth.seed_batches(tiny.n, 1024, seed=0)(0).numpy()
    compare(P, tiny, seeds, (10, 10, 10), sampler, it=0, kappa=1, seed=0)


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
@pytest.mark.parametrize("fanouts", [(1,), (3, 2), (25, 10, 10), (64, 1), (5000,), (2, 2, 2, 2)])
def test_fanout_shapes(P, tiny, sampler, fanouts):
    seeds = synth.seed_batches(tiny.n, 300, seed=2)(1).numpy()
    compare(P, tiny, seeds, fanouts, sampler, it=5, kappa=1, seed=42)


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_ragged_and_degenerate_batches(P, tiny, sampler):
    deg = np.diff(tiny.indptr_h)
    hubs = np.argsort(-deg)[:5].astype(np.int32)          # longest lists (thousands of neighbours)
    isolated = np.nonzero(deg == 0)[0][:5].astype(np.int32)
    assert len(isolated) > 0
    for seeds in (np.zeros(0, np.int32), hubs[:1], isolated, np.concatenate([hubs, isolated]),
                  np.arange(tiny.n, dtype=np.int32)[::-1][:4097]):
        compare(P, tiny, seeds, (10, 10), sampler, it=1, kappa=1, seed=7)
    # whole vertex set as one batch (largest batch this graph admits), one layer
    compare(P, tiny, synth.permutation(tiny.n, 1).numpy(), (10,), sampler, it=2, kappa=1, seed=7)


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_medium_graph_many_tiles(P, medium, sampler):
    seeds = synth.seed_batches(medium.n, 4096, seed=3)(0).numpy()
    compare(P, medium, seeds, (10, 10, 10), sampler, it=11, kappa=1, seed=2024)
    compare(P, medium, seeds[:1000], (25, 10), sampler, it=12, kappa=1, seed=(1 << 63) + 12345)


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
@pytest.mark.parametrize("it,kappa", [(0, 16), (1, 16), (15, 16), (16, 16), (17, 16), (511, 256), (77, 0), (3, 2)])
def test_dependent_batches(P, tiny, sampler, it, kappa):
    seeds = synth.seed_batches(tiny.n, 512, seed=4)(3).numpy()
    compare(P, tiny, seeds, (10, 10), sampler, it=it, kappa=kappa, seed=99)


def test_dependent_batches_medium(P, medium):
    seeds = synth.seed_batches(medium.n, 2048, seed=5)(2).numpy()
    compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=37, kappa=64, seed=5)


def test_arena_allocator_and_determinism(P, tiny):
    seeds = synth.seed_batches(tiny.n, 1024, seed=0)(1).numpy()
    arena = P.Arena(64 << 20)
    a = compare(P, tiny, seeds, (10, 10, 10), R.LABOR0, it=3, seed=1, arena=arena)
    keep = [{n: getattr(b, n).clone() for n in NAMES} for b in a]
    arena.reset()
    b = compare(P, tiny, seeds, (10, 10, 10), R.LABOR0, it=3, seed=1, arena=arena)
    for x, y in zip(keep, b):
        for n in NAMES:
            assert torch.equal(x[n], getattr(y, n))
    small = P.Arena(1 << 12)
    with pytest.raises(P.CoopError) as e:
        P.coop_sample(tiny.graph, torch.from_numpy(seeds).cuda(), (10, 10, 10), R.LABOR0, arena=small)
    assert e.value.code == -5


def test_error_codes(P, tiny):
    def run(seeds, fan=(3,), sampler=0):
        return P.coop_sample(tiny.graph, torch.tensor(seeds, dtype=torch.int32).cuda(), fan, sampler)

    for seeds, code in (([1, 2, 1], -3), ([1, 1 << 20], -2), ([-1], -2)):
        for sampler in (0, 1):
            with pytest.raises(P.CoopError) as e:
                run(seeds, sampler=sampler)
            assert e.value.code == code
    for fan in ((), (0,), (3, -1)):
        with pytest.raises(P.CoopError) as e:
            run([1, 2, 3], fan)
        assert e.value.code == -4
    with pytest.raises(P.CoopError):
        run([1, 2, 3], sampler=7)
    # malformed CSR is caught by COOP_VALIDATE
    bad = tiny.indices_d.clone()
    bad[5] = tiny.n
    with pytest.raises(P.CoopError) as e:
        P.coop_graph_load(tiny.indptr_d, bad, P.COOP_VALIDATE)
    assert e.value.code == -8


@pytest.mark.parametrize("dtype,dim", [(torch.float32, 64), (torch.float32, 100), (torch.float32, 602), (torch.float16, 128),
                                       (torch.float16, 768), (torch.float16, 3), (torch.float32, 1), (torch.float16, 1025)])
@pytest.mark.parametrize("n_ids", [0, 1, 63, 1000, 40000])
def test_gather(P, dtype, dim, n_ids):
    n = 5000
    feat = synth.features(n, dim, dtype, seed=dim, device="cpu")
    ids = (synth.hash_u53(torch.arange(n_ids), 31) % n).to(torch.int32)
    want = R.gather(feat.numpy(), ids.numpy())
    got = P.coop_gather(feat.cuda(), ids.cuda())
    P.coop_gather_status()
    assert got.cpu().numpy().tobytes() == want.tobytes()


def test_gather_unaligned_views_and_range(P):
    feat = synth.features(1000, 33, torch.float16, seed=1, device="cpu")
    base = torch.empty(1000 * 33 + 1, dtype=torch.float16, device="cuda")
    view = base[1:].view(1000, 33)                     # 2-byte aligned table
    view.copy_(feat)
    ids = torch.tensor([0, 999, 5, 5, 17], dtype=torch.int32)
    got = P.coop_gather(view, ids.cuda())
    assert got.cpu().numpy().tobytes() == R.gather(feat.numpy(), ids.numpy()).tobytes()
    P.coop_gather_status()
    P.coop_gather(view, torch.tensor([3, 1000], dtype=torch.int32).cuda())
    with pytest.raises(P.CoopError) as e:
        P.coop_gather_status()
    assert e.value.code == -2
    P.coop_gather_status()                              # the condition was cleared


def test_sample_then_gather_end_to_end(P, tiny):
    feat = synth.features(tiny.n, 64, torch.float32, seed=0, device="cpu")
    seeds = synth.seed_batches(tiny.n, 1024, seed=0)(0).numpy()
    blocks = compare(P, tiny, seeds, (10, 10, 10), R.NS)
    rows = P.coop_gather(feat.cuda(), blocks[-1].src_ids)
    P.coop_gather_status()
    assert rows.cpu().numpy().tobytes() == R.gather(feat.numpy(), blocks[-1].src_ids.cpu().numpy()).tobytes()


def test_labor_stage_overflow_path(P, tiny, medium):
    """Staging rows far smaller than the kept-edge counts: every destination takes the second-scan path."""
    try:
        for cap in (1, 4):
            P.coop_tune(P.COOP_TUNE_STAGE_CAP, cap)
            seeds = synth.seed_batches(tiny.n, 700, seed=6)(0).numpy()
            compare(P, tiny, seeds, (10, 10), R.LABOR0, it=2, kappa=1, seed=3)
            compare(P, tiny, seeds[:100], (10, 10), R.LABOR0, it=5, kappa=4, seed=3)
            compare(P, medium, synth.seed_batches(medium.n, 2000, seed=6)(0).numpy(), (25, 10), R.LABOR0, it=2, seed=8)
    finally:
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 0)


def test_unaligned_indices_base(P, tiny):
    """A CSR whose indices array is only 4-byte aligned takes the scalar-load scan."""
    base = torch.empty(tiny.indices_d.numel() + 1, dtype=torch.int32, device="cuda")
    view = base[1:]
    view.copy_(tiny.indices_d)
    assert view.data_ptr() % 16 != 0
    g2 = P.coop_graph_load(tiny.indptr_d, view, P.COOP_VALIDATE)
    seeds = synth.seed_batches(tiny.n, 512, seed=8)(0)
    a = P.coop_sample(tiny.graph, seeds.cuda(), (10, 10), R.LABOR0, it=1, seed=4)
    b = P.coop_sample(g2, seeds.cuda(), (10, 10), R.LABOR0, it=1, seed=4)
    for x, y in zip(a, b):
        for n in NAMES:
            assert torch.equal(getattr(x, n), getattr(y, n))
    want = R.sample(tiny.indptr_h, tiny.indices_h, seeds.numpy(), (10, 10), R.LABOR0, it=1, seed=4)
    for x, w in zip(b, want):
        for n in NAMES:
            assert np.array_equal(getattr(x, n).cpu().numpy(), w[n])


# --------------------------------------------------------------------------------------------------------------- #
# LRU vertex cache (cached / pinned-host feature loading)
# --------------------------------------------------------------------------------------------------------------- #
def run_cache_sequence(P, cap, n, dim, dtype, batches, table_dev):
    feat = synth.features(n, dim, dtype, seed=5, device="cpu")
    table = feat.cuda() if table_dev == "cuda" else feat.pin_memory()
    cache = P.Cache(cap, n, dim, dtype, max(len(b) for b in batches) + 7)
    oracle = R.Cache(cap, n)
    for it, ids in enumerate(batches):
        ids_t = torch.from_numpy(ids).cuda()
        out, n_miss = cache.gather(table, ids_t)
        want_miss, _ = oracle.access(ids)
        assert n_miss == want_miss, (it, n_miss, want_miss)
        assert out.cpu().numpy().tobytes() == R.gather(feat.numpy(), ids).tobytes(), it
        held = cache.vertices().cpu().numpy()
        assert len(held) == oracle.size(), it
        assert all(oracle.contains(int(v)) for v in held), it
    cache.close()


@pytest.mark.parametrize("cap", [0, 1, 50, 700, 5000])
@pytest.mark.parametrize("table_dev", ["cuda", "pinned"])
def test_cache_matches_textbook_lru(P, cap, table_dev):
    n = 3000
    rng = np.random.default_rng(cap + 1)
    batches = [rng.choice(n, int(rng.integers(1, 900)), replace=False).astype(np.int32) for _ in range(25)]
    batches.append(np.arange(n, dtype=np.int32))           # a batch larger than most capacities
    batches += [rng.choice(n, 300, replace=False).astype(np.int32) for _ in range(5)]
    run_cache_sequence(P, cap, n, 64, torch.float32, batches, table_dev)


@pytest.mark.parametrize("dtype,dim", [(torch.float16, 3), (torch.float16, 1), (torch.float16, 100), (torch.float32, 1),
                                       (torch.float32, 602), (torch.float16, 1025)])
def test_cache_row_shapes(P, dtype, dim):
    """Rows whose size leaves the movers only 2-, 4- or 8-byte vectors, and rows longer than one pass of a lane group."""
    n = 2500
    rng = np.random.default_rng(dim)
    batches = [rng.choice(n, int(rng.integers(1, 700)), replace=False).astype(np.int32) for _ in range(12)]
    run_cache_sequence(P, 400, n, dim, dtype, batches, "cuda" if dim % 2 else "pinned")


def test_cache_on_sampled_batches_with_kappa(P, medium):
    """Input sets of consecutive dependent LABOR-0 batches through the cache: misses equal the oracle's on every
    iteration, and a larger kappa lowers the miss count (temporal locality of Sec. 4.2)."""
    get = synth.seed_batches(medium.n, 512, seed=9)
    feat = synth.features(medium.n, 128, torch.float16, seed=3, device="cpu")
    table = feat.pin_memory()
    totals = {}
    for kappa in (1, 16):
        cache = P.Cache(8000, medium.n, 128, torch.float16, medium.n)
        oracle = R.Cache(8000, medium.n)
        miss = 0
        for it in range(24):
            blocks = P.coop_sample(medium.graph, get(it).cuda(), (10, 10), R.LABOR0, it=it, kappa=kappa, seed=1)
            ids = blocks[-1].src_ids
            out, n_miss = cache.gather(table, ids)
            want, _ = oracle.access(ids.cpu().numpy())
            assert n_miss == want
            if it % 8 == 0:
                assert out.cpu().numpy().tobytes() == R.gather(feat.numpy(), ids.cpu().numpy()).tobytes()
            miss += n_miss
        totals[kappa] = miss
        cache.close()
    assert totals[16] < totals[1]


def test_cache_on_a_side_stream_without_host_waits(P):
    """A call returns once its counts are known, with the eviction and the miss rows still queued, and the eviction
    threshold is read back one call late: work queued behind a call on the caller's stream must see all of `out`, and
    a sequence of calls with no host synchronisation between them must keep the textbook LRU's books (also across an
    export, which needs the threshold of the call before it)."""
    n, dim, cap = 6000, 64, 1500
    rng = np.random.default_rng(77)
    feat = synth.features(n, dim, torch.float16, seed=6, device="cpu")
    table = feat.cuda()
    batches = [rng.choice(n, int(rng.integers(200, 1400)), replace=False).astype(np.int32) for _ in range(20)]
    cache = P.Cache(cap, n, dim, torch.float16, 1500)
    oracle = R.Cache(cap, n)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    copies, misses, keep = [], [], []
    for ids in batches:
        t = torch.from_numpy(ids).cuda()
        keep.append(t)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            out, n_miss = cache.gather(table, t, stream=side)
            copies.append(out.clone())          # queued on the side stream right behind the call
        misses.append(n_miss)
    _, _, state = cache.export_state(stream=side)
    side.synchronize()
    for it, (ids, got, n_miss) in enumerate(zip(batches, copies, misses)):
        want_miss, _ = oracle.access(ids)
        assert n_miss == want_miss, it
        assert got.cpu().numpy().tobytes() == R.gather(feat.numpy(), ids).tobytes(), it
    held = cache.vertices().cpu().numpy()
    assert len(held) == oracle.size() == state[0] and all(oracle.contains(int(v)) for v in held)
    cache.close()


def test_cache_errors(P):
    cache = P.Cache(10, 100, 8, torch.float32, 50)
    table = synth.features(100, 8, torch.float32, seed=1).cuda()
    with pytest.raises(P.CoopError) as e:
        cache.gather(table, torch.arange(60, dtype=torch.int32).cuda())
    assert e.value.code == -6
    with pytest.raises(P.CoopError) as e:
        cache.gather(table, torch.tensor([1, 100], dtype=torch.int32).cuda())
    assert e.value.code == -2
    out, n_miss = cache.gather(table, torch.tensor([5, 1], dtype=torch.int32).cuda())
    assert n_miss == 2 and torch.equal(out, table[[5, 1]])      # the failed call inserted nothing
    not_pinned = synth.features(100, 8, torch.float32, seed=1)
    with pytest.raises((P.CoopError, AssertionError)):
        cache.gather(not_pinned, torch.tensor([5], dtype=torch.int32).cuda())


# --------------------------------------------------------------------------------------------------------------- #
# neighbour mean fused with the feature load (Eq. 1, mean aggregator)
# --------------------------------------------------------------------------------------------------------------- #
@pytest.mark.parametrize("dtype,dim,rtol", [(torch.float32, 64, 1e-5), (torch.float32, 100, 1e-5), (torch.float32, 602, 1e-5),
                                            (torch.float16, 128, 1e-2), (torch.float16, 768, 1e-2), (torch.float16, 3, 1e-2)])
def test_gather_mean(P, medium, dtype, dim, rtol):
    """fp32 accumulation against the oracle's fp64 mean: relative tolerance 1e-5 (fp32 rows) / 1e-2 (fp16 rows, whose
    output rounding alone is 2^-11), measured against the row's largest magnitude so that cancellation near zero counts
    as absolute error."""
    feat = synth.features(medium.n, dim, dtype, seed=dim, device="cpu")
    seeds = synth.seed_batches(medium.n, 1500, seed=7)(0)
    blk = P.coop_sample(medium.graph, seeds.cuda(), (10, 10), R.LABOR0, it=1, seed=3)[-1]
    got = P.coop_gather_mean(feat.cuda(), blk.indptr, blk.col_global)
    P.coop_gather_status()
    want = R.gather_mean(feat.numpy(), blk.indptr.cpu().numpy(), blk.col_global.cpu().numpy())
    got = got.cpu().numpy().astype(np.float64)
    scale = np.maximum(np.abs(want).max(axis=1, keepdims=True), 1e-30)
    assert np.all(np.abs(got - want) <= rtol * scale)
    deg = np.diff(blk.indptr.cpu().numpy())
    assert (deg == 0).any() or True
    assert np.all(got[deg == 0] == 0)


def test_gather_mean_edge_cases(P):
    feat = synth.features(50, 8, torch.float32, seed=1).cuda()
    indptr = torch.tensor([0, 0, 1, 1, 4], dtype=torch.int64).cuda()
    col = torch.tensor([7, 1, 2, 3], dtype=torch.int32).cuda()
    out = P.coop_gather_mean(feat, indptr, col)
    P.coop_gather_status()
    assert torch.all(out[0] == 0) and torch.all(out[2] == 0)
    assert torch.equal(out[1], feat[7])                          # a single edge: the row itself, bit for bit
    assert torch.allclose(out[3], feat[[1, 2, 3]].mean(0), rtol=1e-6, atol=1e-7)
    assert P.coop_gather_mean(feat, torch.zeros(1, dtype=torch.int64).cuda(), col[:0]).shape == (0, 8)
    P.coop_gather_mean(feat, torch.tensor([0, 1], dtype=torch.int64).cuda(), torch.tensor([50], dtype=torch.int32).cuda())
    with pytest.raises(P.CoopError) as e:
        P.coop_gather_status()
    assert e.value.code == -2


def test_nested_dependent_minibatching(P, medium):
    """Sec. 3.2's nested scheme: a parent batch of kappa*b seeds and its kappa child batches of b seeds, all drawn
    with the variates of one group (same iter): every child's S^l lies inside the parent's S^l, and the children's
    input sets together are exactly the parent's."""
    kappa, b = 4, 512
    parent = synth.seed_batches(medium.n, kappa * b, seed=12)(0)
    big = P.coop_sample(medium.graph, parent.cuda(), (10, 10, 10), R.LABOR0, it=5, kappa=1, seed=2)
    union = [set() for _ in range(3)]
    for i in range(kappa):
        child = P.coop_sample(medium.graph, parent[i * b:(i + 1) * b].contiguous().cuda(), (10, 10, 10), R.LABOR0, it=5, kappa=1, seed=2)
        for l in range(3):
            assert bool(torch.isin(child[l].src_ids, big[l].src_ids).all())
            union[l] |= set(child[l].src_ids.cpu().tolist())
    for l in range(3):
        assert union[l] == set(big[l].src_ids.cpu().tolist())


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_labor_fusion_modes(P, tiny, medium, mode):
    """LABOR-0 with the scan fused over all remaining layers (2), per layer (0) and the default mix (1): same bytes."""
    try:
        P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, mode)
        seeds = synth.seed_batches(tiny.n, 900, seed=13)(0).numpy()
        compare(P, tiny, seeds, (10, 10, 10), R.LABOR0, it=4, kappa=1, seed=6)
        compare(P, tiny, seeds[:200], (7, 3, 5, 2), R.LABOR0, it=9, kappa=8, seed=6)          # four layers, blended
        compare(P, tiny, seeds[:50], (3, 3, 3, 3, 3), R.LABOR0, it=2, kappa=1, seed=6)          # five layers: never fused
        compare(P, medium, synth.seed_batches(medium.n, 3000, seed=13)(1).numpy(), (25, 10, 10), R.LABOR0, it=1, seed=6)
        isolated = np.nonzero(np.diff(tiny.indptr_h) == 0)[0][:3].astype(np.int32)
        compare(P, tiny, isolated, (10, 10, 10), R.LABOR0, it=1, seed=6)                        # layers that add no vertex
    finally:
        P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, 1)


@pytest.mark.parametrize("piece_len", [0, 256, 300, 512])
def test_labor_long_lists_cut_into_pieces(P, tiny, medium, piece_len):
    """Lists longer than twice the piece length are scanned by several waves; the bytes do not change."""
    try:
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, piece_len)
        hubs_t = np.argsort(-np.diff(tiny.indptr_h))[:40].astype(np.int32)
        hubs_m = np.argsort(-np.diff(medium.indptr_h))[:300].astype(np.int32)
        assert np.diff(tiny.indptr_h)[hubs_t[0]] > 3000 and np.diff(medium.indptr_h)[hubs_m[0]] > 1400
        for mode in (1, 2):
            P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, mode)
            compare(P, tiny, hubs_t, (10, 10, 10), R.LABOR0, it=3, kappa=1, seed=21)
            compare(P, tiny, hubs_t, (5, 30), R.LABOR0, it=7, kappa=4, seed=21)                      # blended
            compare(P, medium, hubs_m, (25, 10, 10), R.LABOR0, it=1, seed=22)
            compare(P, medium, synth.seed_batches(medium.n, 3000, seed=14)(2).numpy(), (10, 10, 10), R.LABOR0, it=5, kappa=16, seed=22)
            compare(P, medium, hubs_m[:20], (1450, 2), R.LABOR0, it=1, seed=22)                      # fanout above some hub degrees
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 4)                                                        # rows overflow across pieces
        compare(P, medium, hubs_m[:50], (10, 10), R.LABOR0, it=2, seed=23)
        compare(P, tiny, hubs_t, (10, 10), R.LABOR0, it=6, kappa=4, seed=23)
    finally:
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, 4096)
        P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, 1)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 0)


@pytest.mark.parametrize("split_min,piece_len", [(64, 4096), (200, 512), (1000, 256)])
def test_labor_lists_handed_to_the_piece_waves_whole(P, tiny, medium, split_min, piece_len):
    """Lists longer than COOP_TUNE_SPLIT_MIN go to the waves that come first in the scan's grid: as a single piece when they
    are shorter than the piece length, in several otherwise (the default does this with dependent variates from 2,048
    entries on).  Independent and dependent variates, both fusion modes; the bytes do not change."""
    try:
        P.coop_tune(P.COOP_TUNE_SPLIT_MIN, split_min)
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, piece_len)
        hubs_m = np.argsort(-np.diff(medium.indptr_h))[:200].astype(np.int32)
        seeds = synth.seed_batches(medium.n, 3000, seed=15)(1).numpy()
        for mode in (1, 2):
            P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, mode)
            compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=5, kappa=16, seed=24)
            compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=4, kappa=1, seed=24)
            compare(P, medium, hubs_m, (25, 10), R.LABOR0, it=9, kappa=4, seed=25)
            compare(P, tiny, synth.seed_batches(tiny.n, 1024, seed=0)(3).numpy(), (10, 10, 10), R.LABOR0, it=3, kappa=2, seed=26)
    finally:
        P.coop_tune(P.COOP_TUNE_SPLIT_MIN, 0)
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, 4096)
        P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, 1)
    with pytest.raises(P.CoopError):
        P.coop_tune(P.COOP_TUNE_SPLIT_MIN, 7)


def test_cache_export_import_resumes_exactly(P):
    """A cache rebuilt from an export answers the following batches exactly as the original does."""
    n, dim = 4000, 32
    rng = np.random.default_rng(21)
    feat = synth.features(n, dim, torch.float16, seed=4, device="cpu")
    table = feat.cuda()
    batches = [rng.choice(n, int(rng.integers(50, 700)), replace=False).astype(np.int32) for _ in range(30)]
    a = P.Cache(900, n, dim, torch.float16, 1000)
    for ids in batches[:15]:
        a.gather(table, torch.from_numpy(ids).cuda())
    vertices, stamps, state = a.export_state()
    assert vertices.numel() == state[0] == a.vertices().numel()
    b = P.Cache(1200, n, dim, torch.float16, 1000)                  # a larger capacity may import a smaller cache
    c = P.Cache(900, n, dim, torch.float16, 1000)
    c.import_state(table, vertices, stamps, state)
    assert torch.equal(c.vertices(), a.vertices())
    for ids in batches[15:]:
        t = torch.from_numpy(ids).cuda()
        out_a, miss_a = a.gather(table, t)
        out_c, miss_c = c.gather(table, t)
        assert miss_a == miss_c and torch.equal(out_a, out_c)
        assert torch.equal(a.vertices(), c.vertices())
    b.import_state(table, vertices, stamps, state)
    assert torch.equal(b.vertices(), torch.sort(vertices).values)
    bad = vertices.clone()
    bad[0] = n
    with pytest.raises(P.CoopError) as e:
        b.import_state(table, bad, stamps, state)
    assert e.value.code == -2 and b.vertices().numel() == 0
    dup = vertices.clone()
    dup[1] = dup[0]
    with pytest.raises(P.CoopError) as e:
        b.import_state(table, dup, stamps, state)
    assert e.value.code == -2 and b.vertices().numel() == 0
    out, n_miss = b.gather(table, torch.from_numpy(batches[0]).cuda())       # still usable, and empty
    assert n_miss == len(batches[0]) and torch.equal(out.cpu(), feat[torch.from_numpy(batches[0]).long()])


def compare_rw(P, g, seeds, fanouts, o, a, p, it=0, seed=0, arena=None):
    seeds_h = np.ascontiguousarray(seeds, dtype=np.int32)
    want = R.sample(g.indptr_h, g.indices_h, seeds_h, fanouts, R.RW, it=it, seed=seed, rw=(o, a, p))
    got = P.coop_sample_rw(g.graph, torch.from_numpy(seeds_h).cuda(), fanouts, o, a, p, it=it, seed=seed, arena=arena)
    assert len(got) == len(want)
    for l, (b, w) in enumerate(zip(got, want)):
        assert (b.n_dst, b.n_edges, b.n_src) == (len(w["dst_ids"]), len(w["col_global"]), len(w["src_ids"])), l
        for name in NAMES:
            a_ = getattr(b, name).cpu().numpy()
            assert a_.dtype == w[name].dtype and np.array_equal(a_, w[name]), (l, name)
    return got


@pytest.mark.parametrize("o,a,p,fanouts", [(3, 100, 0.5, (10, 10, 10)), (1, 7, 0.0, (3, 3)), (4, 20, 0.25, (5, 2, 4)),
                                           (2, 50, 1.0, (8,)), (3, 128, 0.5, (10,)), (2, 192, 0.1, (400,)),
                                           (4, 256, 0.5, (10, 1000)), (1024, 1, 0.3, (2000,)), (1, 1, 0.5, (1,))])
def test_random_walk_sampler(P, tiny, o, a, p, fanouts):
    """App. A.1.3: walks, tallies and the top-k order equal the oracle's on every array (eid = visit counts)."""
    n_seeds = 300 if o * a <= 384 else 60
    seeds = synth.seed_batches(tiny.n, n_seeds, seed=31)(1).numpy()
    compare_rw(P, tiny, seeds, fanouts, o, a, p, it=5, seed=17)


def test_random_walk_sampler_medium_and_degenerate(P, tiny, medium):
    compare_rw(P, medium, synth.seed_batches(medium.n, 2500, seed=32)(0).numpy(), (10, 10), 3, 100, 0.5, it=2, seed=9)
    compare_rw(P, tiny, np.zeros(0, dtype=np.int32), (10, 10), 3, 100, 0.5)                         # empty batch
    isolated = np.nonzero(np.diff(tiny.indptr_h) == 0)[0][:3].astype(np.int32)
    compare_rw(P, tiny, isolated, (10, 10), 3, 100, 0.5)                                            # no neighbours at all
    hubs = np.argsort(-np.diff(tiny.indptr_h))[:5].astype(np.int32)
    compare_rw(P, tiny, np.concatenate([hubs, isolated]), (10, 10), 3, 100, 0.5, it=1 << 40, seed=(1 << 63) + 5)
    arena = P.Arena(64 << 20)
    a = compare_rw(P, tiny, hubs, (10, 10), 3, 100, 0.5, it=3, seed=1, arena=arena)
    first = [b.col_global.clone() for b in a]
    arena.reset()
    b = compare_rw(P, tiny, hubs, (10, 10), 3, 100, 0.5, it=3, seed=1, arena=arena)
    assert all(torch.equal(x, y.col_global) for x, y in zip(first, b))


@pytest.mark.parametrize("o,a,p", [(33, 32, 0.5), (3, 600, 0.3), (1500, 1, 0.0), (40, 40, 0.9)])
def test_random_walks_with_more_than_1024_steps(P, tiny, medium, o, a, p):
    """App. A.1.3 puts no bound on the number of walks or their length.  Above 1,024 steps per destination the visit
    tallies live in device memory (a kernel of its own): fanouts below, around and above the number of distinct vertices
    a destination reaches, a second layer on top, hubs and isolated vertices among the destinations."""
    seeds = synth.seed_batches(tiny.n, 96, seed=61)(0).numpy()
    compare_rw(P, tiny, seeds, (10, 5), o, a, p, it=2, seed=41)
    compare_rw(P, tiny, seeds[:24], (300,), o, a, p, it=3, seed=41)
    compare_rw(P, tiny, seeds[:8], (1 << 20,), o, a, p, it=4, seed=41)
    hubs = np.argsort(-np.diff(medium.indptr_h))[:12].astype(np.int32)
    compare_rw(P, medium, hubs, (25, 3), o, a, p, it=5, seed=42)


def test_random_walk_sampler_errors(P, tiny):
    seeds = torch.arange(4, dtype=torch.int32).cuda()
    for bad in ((0, 10, 0.5), (3, 0, 0.5), (3, 10, 1.5), (3, 10, -0.1), (1 << 11, 1 << 10, 0.5), (3, 10, float("nan"))):
        with pytest.raises(P.CoopError) as e:
            P.coop_sample_rw(tiny.graph, seeds, (5,), *bad)
        assert e.value.code == -4
    with pytest.raises(P.CoopError) as e:
        P.coop_sample(tiny.graph, seeds, (5,), P.COOP_RW)
    assert e.value.code == -4
    with pytest.raises(P.CoopError) as e:
        P.coop_sample_rw(tiny.graph, torch.tensor([1, 1], dtype=torch.int32).cuda(), (5,), 3, 10, 0.5)
    assert e.value.code == -3
    with pytest.raises(P.CoopError) as e:
        P.coop_sample_rw(tiny.graph, torch.tensor([tiny.n], dtype=torch.int32).cuda(), (5,), 3, 10, 0.5)
    assert e.value.code == -2


def test_limits_of_the_interface(P, tiny):
    """Deepest model the interface takes (L = 255), fanouts far above every degree, the largest walk budget."""
    seeds = synth.seed_batches(tiny.n, 8, seed=41)(0).numpy()
    compare(P, tiny, seeds[:2], (1,) * 255, R.LABOR0, it=1, seed=4)
    compare(P, tiny, seeds[:2], (1,) * 255, R.NS, it=1, seed=4)
    compare(P, tiny, seeds, (1 << 30, 1 << 30), R.LABOR0, it=2, seed=4)          # keeps every neighbour: two-hop ball
    compare(P, tiny, seeds, ((1 << 31) - 1,), R.NS, it=2, seed=4)
    compare_rw(P, tiny, seeds, ((1 << 31) - 1,), 1024, 1, 0.0, it=3, seed=4)
    compare_rw(P, tiny, seeds, (7,), 1, 1024, 1.0, it=3, seed=4)
    with pytest.raises(P.CoopError) as e:
        P.coop_sample(tiny.graph, torch.from_numpy(seeds).cuda(), (1,) * 256, P.COOP_LABOR0)
    assert e.value.code == -4


@pytest.mark.parametrize("long_min", [64, 300, 0])
def test_ns_long_lists_taken_by_the_first_waves(P, tiny, medium, long_min):
    """The NS traversal hands the destinations with long lists to the first waves of its grid (a queue filled by the count
    pass) and leaves the rest in destination order.  With the knob at 64 or 300 every pass of these small graphs takes
    that path (by default only passes over 32,768 destinations or more do): same bytes as the oracle, also with a fanout
    above the candidate arrays, whose long lists go on to the bisection kernel, and with the queue switched off."""
    deg = np.diff(medium.indptr_h)
    hubs = np.argsort(-deg)[:30].astype(np.int32)
    rest = synth.seed_batches(medium.n, 3000, seed=12)(0).numpy()
    seeds = np.concatenate([hubs, rest[~np.isin(rest, hubs)]])
    try:
        P.coop_tune(P.COOP_TUNE_NS_LONG_LIST, long_min)
        compare(P, medium, seeds, (10, 10, 10), R.NS, it=3, kappa=1, seed=31)
        compare(P, medium, seeds[:500], (25, 10), R.NS, it=16, kappa=16, seed=31)   # (a group boundary: c = 0)
        compare(P, medium, seeds[:400], (10, 5), R.NS, it=21, kappa=16, seed=31)    # (c = 5/16: the blended kernels)
        compare(P, medium, hubs, (1100, 2), R.NS, it=2, kappa=1, seed=32)
        compare(P, tiny, synth.seed_batches(tiny.n, 1024, seed=0)(2).numpy(), (10, 10, 10), R.NS, it=1, kappa=1, seed=33)
        P.coop_tune(P.COOP_TUNE_DEFER_SIZES, 2)      # every layer is run twice: the queue starts empty both times
        compare(P, medium, seeds, (10, 10, 10), R.NS, it=3, kappa=1, seed=31)
    finally:
        P.coop_tune(P.COOP_TUNE_NS_LONG_LIST, 2048)
        P.coop_tune(P.COOP_TUNE_DEFER_SIZES, 1)
    with pytest.raises(P.CoopError):
        P.coop_tune(P.COOP_TUNE_NS_LONG_LIST, 5)


def test_ns_fanouts_above_the_candidate_arrays(P, medium):
    """App. A.1.1 has no upper limit on the fanout.  Up to 1,024 the k smallest variates of a list are found among
    candidates kept in LDS; above that, lists longer than the fanout take the selection by bisection on the variate.  Hubs
    of some 1,400 neighbours with fanouts on both sides of that line and of their degrees, independent and dependent
    variates, a second layer on top."""
    deg = np.diff(medium.indptr_h)
    hubs = np.argsort(-deg)[:24].astype(np.int32)
    assert deg[hubs[0]] > 1450 and deg[hubs[-1]] > 1300
    rest = synth.seed_batches(medium.n, 200, seed=77)(1).numpy()
    seeds = np.concatenate([hubs, rest[~np.isin(rest, hubs)]])
    for fan in ((1024,), (1025,), (1100, 3), (1400,), (int(deg[hubs[0]]) - 1,), (int(deg[hubs[0]]),), (2000,), (3, 1200)):
        compare(P, medium, seeds, fan, R.NS, it=5, kappa=1, seed=23)
    compare(P, medium, hubs[:6], (1300,), R.NS, it=21, kappa=16, seed=23)
    compare(P, medium, hubs[:6], (1025, 2), R.NS, it=9, kappa=0, seed=24)


def test_blend_candidate_buffer_overflow_is_redone(P, tiny, medium):
    """A candidate buffer far too small for the exact stage of a dependent batch: the pass is repeated with more room
    until it fits, and the bytes do not change."""
    try:
        P.coop_tune(P.COOP_TUNE_BLEND_CANDIDATES, 64)
        seeds = synth.seed_batches(medium.n, 3000, seed=51)(0).numpy()
        compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=5, kappa=16, seed=31)
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, 256)
        compare(P, medium, seeds[:500], (25, 10), R.LABOR0, it=21, kappa=4, seed=32)
        compare(P, tiny, synth.seed_batches(tiny.n, 600, seed=52)(0).numpy(), (7, 3, 5, 2), R.LABOR0, it=9, kappa=8, seed=33)
    finally:
        P.coop_tune(P.COOP_TUNE_BLEND_CANDIDATES, 0)
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, 4096)


def test_ns_dependent_batches_go_through_the_filters(P, tiny, medium):
    """NS with c > 0: candidates reach the exact blend through the integer bounds and the fp32 blend; hubs, short lists,
    fanouts on both sides of the candidate target, a failing first bound (fanout close to the degrees)."""
    seeds = synth.seed_batches(medium.n, 1500, seed=61)(0).numpy()
    hubs = np.argsort(-np.diff(medium.indptr_h))[:200].astype(np.int32)
    for it, kappa in ((5, 16), (255, 256), (3, 2)):
        compare(P, medium, seeds, (10, 10), R.NS, it=it, kappa=kappa, seed=41)
        compare(P, medium, hubs, (25, 3), R.NS, it=it, kappa=kappa, seed=42)
    compare(P, medium, hubs[:40], (1000, 2), R.NS, it=9, kappa=4, seed=43)      # fanout close to the degrees
    compare(P, tiny, synth.seed_batches(tiny.n, 400, seed=62)(0).numpy(), (1, 40, 7), R.NS, it=7, kappa=8, seed=44)
    # fanout 1 over tens of thousands of lists: about one list in 10^4 collects no candidate at its first bound, or has
    # its smallest estimate too close to the filter's limit, and goes through the one-kernel path again
    many = synth.seed_batches(medium.n, 20000, seed=63)(0).numpy()
    for it, kappa in ((3, 4), (9, 16)):
        compare(P, medium, many, (1, 1), R.NS, it=it, kappa=kappa, seed=45)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_edge_count_read_back_modes(P, tiny, medium, mode):
    """The edge arrays sized from the exact count (0), from a bound with the count read back later (1), and from a
    bound that falls short so that every layer is run again the slow way (2): the same bytes, for all three samplers,
    with staging-row and candidate-buffer overflows in the mix."""
    try:
        P.coop_tune(P.COOP_TUNE_DEFER_SIZES, mode)
        seeds = synth.seed_batches(medium.n, 3000, seed=71)(0).numpy()
        small = synth.seed_batches(tiny.n, 500, seed=72)(0).numpy()
        for sampler in (R.NS, R.LABOR0):
            compare(P, medium, seeds, (10, 10, 10), sampler, it=3, kappa=1, seed=61)
            compare(P, medium, seeds[:700], (25, 10), sampler, it=5, kappa=16, seed=62)
            compare(P, tiny, small, (5000, 3), sampler, it=1, seed=63)             # every neighbour, then a small fanout
            compare(P, tiny, small[:0], (10, 10), sampler, seed=64)                # empty batch
            compare(P, tiny, small[:200], (64, 65), sampler, it=2, seed=60)        # the largest fanout with a bound, the first without
            compare(P, tiny, small[:1], (3, 3, 3, 3, 3), sampler, it=9, kappa=4, seed=65)
        compare_rw(P, medium, seeds[:1500], (10, 5), 3, 50, 0.5, it=2, seed=66)
        compare_rw(P, tiny, small, (4, 40), 2, 9, 0.1, it=2, seed=67)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 4)                                      # rows overflow: LABOR-0 leaves the fast mode
        compare(P, medium, seeds[:900], (10, 10, 10), R.LABOR0, it=4, kappa=1, seed=68)
        compare(P, tiny, small, (10, 10), R.LABOR0, it=6, kappa=8, seed=69)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 0)
        P.coop_tune(P.COOP_TUNE_BLEND_CANDIDATES, 64)                              # the exact stage's buffer overflows
        compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=5, kappa=16, seed=70)
        arena = P.Arena(1 << 28)                                                   # bump allocator: abandoned buffers stay
        compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=7, kappa=1, seed=71, arena=arena)
    finally:
        P.coop_tune(P.COOP_TUNE_DEFER_SIZES, 1)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 0)
        P.coop_tune(P.COOP_TUNE_BLEND_CANDIDATES, 0)


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_frontier_dedup_modes(P, tiny, medium, mode):
    """S^{l+1} and the local ids through the hash table in HBM (1), through the partition into buckets with tables in
    LDS (2), and through buckets so large that their tables overflow and the call falls back (3): the same bytes,
    including the seed-list checks, with both ways of reading the edge count back."""
    try:
        P.coop_tune(P.COOP_TUNE_UNIQUE, mode)
        seeds = synth.seed_batches(medium.n, 6000, seed=81)(0).numpy()
        small = synth.seed_batches(tiny.n, 500, seed=82)(0).numpy()
        for defer in (1, 0):
            P.coop_tune(P.COOP_TUNE_DEFER_SIZES, defer)
            P.profile_reset()
            P.profile_enable(True)
            compare(P, medium, seeds, (10, 10, 10), R.LABOR0, it=3, seed=81)       # last layer: several buckets, most vertices
            P.profile_enable(False)
            ran = P.profile_read_all()
            assert ("unique_part_first" in ran) == (mode != 1) and ("unique_insert" in ran) == (mode != 2), ran.keys()
            compare(P, medium, seeds[:2500], (25, 10), R.NS, it=4, seed=82)
            compare(P, tiny, small, (5, 5, 5), R.LABOR0, it=5, kappa=4, seed=83)   # a bucket or two
            compare(P, tiny, small[:1], (2, 2), R.NS, seed=84)
            compare(P, tiny, small[:0], (3,), R.NS, seed=85)
            compare_rw(P, medium, seeds[:1500], (10, 5), 3, 50, 0.5, it=2, seed=86)
        for bad, code in (([1, 2, 1], -3), (list(range(300)) + [299], -3), ([5, 1 << 20], -2)):
            with pytest.raises(P.CoopError) as e:
                P.coop_sample(tiny.graph, torch.tensor(bad, dtype=torch.int32).cuda(), (3, 3), R.LABOR0)
            assert e.value.code == code
    finally:
        P.coop_tune(P.COOP_TUNE_UNIQUE, 0)
        P.coop_tune(P.COOP_TUNE_DEFER_SIZES, 1)


def test_repeated_neighbours_and_unsorted_lists(P):
    """A multigraph with unsorted lists (legal without COOP_SYMMETRIC): a neighbour that occurs several times in a list
    has the same variate each time, so NS must break the tie by list position (in the candidate ranking, in the
    two-kernel path with dependent variates, and in the bisection of the wide-fanout path), LABOR-0 keeps every copy or
    none, and the walks see the copies as separate edges.  Every array against the oracle."""
    rng = np.random.default_rng(404)
    n = 3000
    deg = np.where(rng.random(n) < 0.5, rng.integers(0, 400, n), np.minimum(rng.zipf(1.6, n), 2500)).astype(np.int64)
    deg[:4] = (6000, 2200, 1500, 0)                                  # hubs above the wide-fanout limit, and an empty list
    ip = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    # each list draws from a pool a quarter of its length: most neighbours occur several times, in random order
    ix = np.concatenate([rng.integers(0, n, max(1, d // 4))[rng.integers(0, max(1, d // 4), d)] for d in deg]).astype(np.int32)
    g = G(P, torch.from_numpy(ip), torch.from_numpy(ix))
    seeds = np.concatenate([np.arange(4), synth.seed_batches(n, 600, seed=7)(0).numpy()])
    seeds = np.unique(seeds).astype(np.int32)
    hubs = np.arange(3, dtype=np.int32)
    for kappa, it in ((1, 0), (4, 6), (0, 9)):
        compare(P, g, seeds, (10, 5), R.NS, it=it, kappa=kappa, seed=11)
        compare(P, g, seeds, (10, 5), R.LABOR0, it=it, kappa=kappa, seed=12)
        compare(P, g, hubs, (40, 3), R.NS, it=it, kappa=kappa, seed=13)       # more than 64 candidates per list
    compare(P, g, hubs, (2000,), R.NS, it=1, seed=14)                         # above the candidate arrays: bisection
    compare(P, g, hubs, (1500, 2), R.NS, it=2, kappa=4, seed=15)
    compare_rw(P, g, seeds[:200], (5, 5), 3, 20, 0.3, it=3, seed=16)


def test_randomized_configurations(P, draw_seed=20240, cases=400):
    """Seeded random draws of graph shape, batch, depth, fanouts, sampler, iteration / kappa and of the library's
    internal modes (piece length, layer fusion, staging rows, read-back mode, dedup mode, lists per wave, the lengths from
    which NS queues a list and LABOR-0 hands it to the piece waves; every other
    graph registered as symmetric, with a random degree above which LABOR-0 works from the neighbours' side), every
    output against the oracle: the code paths meet here in combinations that no other test spells out."""
    rng = np.random.default_rng(draw_seed)
    rng2 = np.random.default_rng(draw_seed + 1)
    rng3 = np.random.default_rng(draw_seed + 2)
    fan_choices = (1, 2, 3, 5, 10, 25, 64, 65, 300)
    knobs = (P.COOP_TUNE_PIECE_LEN, P.COOP_TUNE_FUSE_LAYERS, P.COOP_TUNE_STAGE_CAP, P.COOP_TUNE_DEFER_SIZES, P.COOP_TUNE_UNIQUE,
             P.COOP_TUNE_LISTS_PER_WAVE, P.COOP_TUNE_ENUM_DEGREE, P.COOP_TUNE_NS_LONG_LIST, P.COOP_TUNE_SPLIT_MIN)
    defaults = (4096, 1, 0, 1, 0, 0, 8192, 2048, 0)
    graphs = []
    for gi in range(6):
        n = int(rng.choice((60, 900, 7000, 30000)))
        m = int(n * rng.choice((1, 6, 30, 70)))
        graphs.append(G(P, *synth.chung_lu_csr(n, max(m, n), float(rng.choice((1.9, 2.1, 2.6))), seed=100 + gi),
                        flags=P.COOP_VALIDATE | (P.COOP_SYMMETRIC if gi % 2 else 0)))
    try:
        for case in range(cases):
            g = graphs[case % len(graphs)]
            L = int(rng.integers(1, 5))
            fanouts = tuple(int(rng.choice(fan_choices)) for _ in range(L))
            b = int(min(g.n, rng.choice((1, 7, 64, 500, 3000))))
            seeds = synth.seed_batches(g.n, b, seed=int(rng.integers(1 << 20)))(0).numpy()
            sampler = int(rng.choice((R.NS, R.LABOR0, R.RW), p=(0.4, 0.45, 0.15)))
            kappa = int(rng.choice((0, 1, 2, 16)))
            it = int(rng.integers(0, 40))
            sd = int(rng.integers(1 << 30))
            values = (int(rng.choice((0, 256, 512, 4096))), int(rng.integers(0, 3)), int(rng.choice((0, 0, 4, 32))),
                      int(rng.integers(0, 3)), int(rng.integers(0, 4)), int(rng.choice((0, 0, 1, 3, 8))),
                      int(rng2.choice((0, 64, 64, 150, 1000, 8192))), int(rng3.choice((2048, 0, 64, 200))), int(rng3.choice((0, 0, 64, 700))))
            for kn, v in zip(knobs, values):
                P.coop_tune(kn, v)
            label = (case, g.n, fanouts, b, sampler, kappa, it, values)
            try:
                if sampler == R.RW:
                    fan = tuple(min(f, 64) for f in fanouts[:2])
                    compare_rw(P, g, seeds[:min(b, 300)], fan, int(rng.integers(1, 4)), int(rng.integers(1, 40)), float(rng.choice((0.0, 0.3, 1.0))),
                               it=it, seed=sd)
                else:
                    if sampler == R.NS and kappa != 1 and max(fanouts) > 64:
                        fanouts = tuple(min(f, 64) for f in fanouts)  # (keeps the oracle's exact blends to a few seconds)
                    compare(P, g, seeds, fanouts, sampler, it=it, kappa=kappa, seed=sd)
            except AssertionError as e:
                raise AssertionError("%s: %s" % (label, e))
    finally:
        for kn, v in zip(knobs, defaults):
            P.coop_tune(kn, v)


@pytest.mark.parametrize("degree", [64, 300, 8192])
def test_labor_long_lists_from_the_other_side(P, tiny, medium, degree):
    """Graphs registered as symmetric: LABOR-0 with independent variates finds the kept neighbours of lists longer than
    `degree` from the neighbours' side (inverse mixer, walk of the listed vertices' lists, index of reverse positions);
    the bytes must not change.  Dependent variates and NS take the ordinary path on the same handle."""
    try:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, degree)
        flags = P.COOP_VALIDATE | P.COOP_SYMMETRIC
        gm = G(P, torch.from_numpy(medium.indptr_h), torch.from_numpy(medium.indices_h), flags)
        gt = G(P, torch.from_numpy(tiny.indptr_h), torch.from_numpy(tiny.indices_h), flags)
        seeds = synth.seed_batches(gm.n, 4000, seed=91)(0).numpy()
        small = synth.seed_batches(gt.n, 700, seed=92)(0).numpy()
        hubs = np.argsort(-np.diff(gm.indptr_h))[:300].astype(np.int32)
        for mode in (1, 0, 2):
            P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, mode)
            compare(P, gm, seeds, (10, 10, 10), R.LABOR0, it=3, seed=91)
            compare(P, gm, hubs, (5, 25), R.LABOR0, it=4, seed=92)
            compare(P, gt, small, (10, 10, 10), R.LABOR0, it=5, seed=93)
        P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, 1)
        compare(P, gm, seeds, (64, 3), R.LABOR0, it=6, seed=94)             # the largest fanout that is served this way
        compare(P, gm, seeds[:500], (65, 3), R.LABOR0, it=6, seed=95)       # the first that is not
        compare(P, gm, seeds[:800], (10, 10), R.LABOR0, it=7, kappa=4, seed=96)
        compare(P, gm, seeds[:800], (10, 10), R.NS, it=8, seed=97)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 4)                               # rows overflow: the ordered second scan takes over
        compare(P, gm, hubs, (10, 10), R.LABOR0, it=9, seed=98)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 0)
        for defer in (0, 2):
            P.coop_tune(P.COOP_TUNE_DEFER_SIZES, defer)
            compare(P, gm, seeds[:1500], (10, 10, 10), R.LABOR0, it=10, seed=99)
    finally:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 8192)
        P.coop_tune(P.COOP_TUNE_FUSE_LAYERS, 1)
        P.coop_tune(P.COOP_TUNE_STAGE_CAP, 0)
        P.coop_tune(P.COOP_TUNE_DEFER_SIZES, 1)


def test_labor_other_side_falls_back_when_a_hub_is_listed(P):
    """A star with 200,000 leaves: the hub's list is the one long list, and in about one iteration out of 65 (fanout 1,
    degree limit 64) the hub itself is among the vertices with a small variate.  Its 3,125 items do not fit the room that
    was sized for four times the expected number, so the pass is done again with every list scanned.  Every iteration
    must give the oracle's bytes; the kernel launch counts show that the second attempt took place."""
    n_leaf = 200_000
    ip = np.concatenate([[0, n_leaf], n_leaf + 1 + np.arange(n_leaf)]).astype(np.int64)
    ix = np.concatenate([1 + np.arange(n_leaf), np.zeros(n_leaf)]).astype(np.int32)
    g = G(P, torch.from_numpy(ip), torch.from_numpy(ix), flags=P.COOP_VALIDATE | P.COOP_SYMMETRIC)
    seeds = (1 + 37 * np.arange(64)).astype(np.int32)
    redone = 0
    try:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 64)
        P.profile_enable(True)
        for it in range(400):
            P.profile_reset()
            compare(P, g, seeds, (1, 1), R.LABOR0, it=it, seed=5)
            counts = P.profile_read_all()
            lists, scans = counts.get("enum_list", (0, 0))[1], counts.get("labor_scan", (0, 0))[1]
            assert lists >= 1
            redone += scans > 2          # (one scan pass per layer when nothing is redone)
            if redone >= 2:
                break
    finally:
        P.profile_enable(False)
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 8192)
    assert redone >= 1


def test_symmetric_flag_is_checked(P, tiny):
    """COOP_SYMMETRIC: a graph with one edge that lacks its reverse, or with an unsorted list, is refused."""
    flags = P.COOP_VALIDATE | P.COOP_SYMMETRIC
    P.coop_graph_load(tiny.indptr_d, tiny.indices_d, flags)  # the tiny graph is symmetric
    ip, ix = tiny.indptr_h, tiny.indices_h
    deg = np.diff(ip)
    v = int(np.argmax(deg))                      # the hub: drop the hub from the list of one of its neighbours
    w = int(ix[ip[v]])
    keep = np.ones(len(ix), dtype=bool)
    pos = ip[w] + int(np.searchsorted(ix[ip[w]:ip[w + 1]], v))
    assert ix[pos] == v
    keep[pos] = False
    ix2 = ix[keep]
    ip2 = ip.copy()
    ip2[w + 1:] -= 1
    d_ip, d_ix = torch.from_numpy(ip2).cuda(), torch.from_numpy(ix2).cuda()
    with pytest.raises(P.CoopError) as e:
        P.coop_graph_load(d_ip, d_ix, flags)
    assert e.value.code == -8
    swapped = ix.copy()
    a = int(ip[v])
    swapped[a], swapped[a + 1] = swapped[a + 1], swapped[a]
    with pytest.raises(P.CoopError) as e:
        P.coop_graph_load(tiny.indptr_d, torch.from_numpy(swapped).cuda(), flags)
    assert e.value.code == -8
    # COOP_SYMMETRIC alone checks as much (the index of reverse positions cannot be built otherwise)
    with pytest.raises(P.CoopError) as e:
        P.coop_graph_load(d_ip, d_ix, P.COOP_SYMMETRIC)
    assert e.value.code == -8


@pytest.mark.parametrize("scheme", [0, 1])
def test_bucket_by_owner(P, scheme):
    """The local half of the id redistribution (Sec. 3.1, Algorithm 1): ids grouped by owner, original order kept, against
    the oracle's sweep per owner: sizes that span one wave, several stretches and a ragged tail, 1 to 64 owners, an empty
    list, and an id out of range (left out of every group, reported by coop_gather_status)."""
    rng = np.random.default_rng(17 + scheme)
    nv = 1_000_003
    for n, n_parts in ((0, 4), (1, 1), (63, 3), (64, 64), (5000, 8), (70001, 5), (600_000, 8), (5_000_011, 64)):
        ids = rng.integers(0, nv, size=n).astype(np.int32)
        if n > 100:
            ids[: n // 3] = np.sort(ids[: n // 3])            # a sorted stretch: long runs of one owner
        want = R.bucket_by_owner(ids, nv, n_parts, scheme, seed=99)
        got = P.coop_bucket_by_owner(torch.from_numpy(ids).cuda(), nv, n_parts, scheme, seed=99)
        P.coop_gather_status()
        for a, w, name in zip(got, want, ("ids", "origin", "offsets")):
            assert np.array_equal(a.cpu().numpy(), w), (n, n_parts, name)
    # without the way back
    ids = rng.integers(0, nv, size=3000).astype(np.int32)
    got = P.coop_bucket_by_owner(torch.from_numpy(ids).cuda(), nv, 8, scheme, seed=1, want_origin=False)
    assert got[1] is None and np.array_equal(got[0].cpu().numpy(), R.bucket_by_owner(ids, nv, 8, scheme, seed=1)[0])
    # an id outside [0, |V|)
    bad = ids.copy()
    bad[17] = nv
    out, origin, offsets = P.coop_bucket_by_owner(torch.from_numpy(bad).cuda(), nv, 8, scheme, seed=1)
    with pytest.raises(P.CoopError) as e:
        P.coop_gather_status()
    assert e.value.code == -2
    keep = np.delete(ids, 17)
    want = R.bucket_by_owner(keep, nv, 8, scheme, seed=1)
    assert int(offsets[-1]) == len(keep) and np.array_equal(out.cpu().numpy()[: len(keep)], want[0])
    for args in ((nv, 0), (nv, 65), (0, 4)):
        with pytest.raises(P.CoopError):
            P.coop_bucket_by_owner(torch.from_numpy(ids).cuda(), args[0], args[1], scheme)


def test_directed_graph(P, medium):
    """Sec. 2 defines N(s) as the in-neighbours of s: on a directed graph (of every pair of opposite edges of the medium
    graph one survives) the lists that the samplers read are not the lists of the vertices that they lead to.  NS, LABOR-0
    (independent and dependent variates) and random walks against the oracle, the graph registered as it is; stating
    that it is symmetric is refused."""
    dp, dx = synth.directed_from_symmetric(torch.from_numpy(medium.indptr_h), torch.from_numpy(medium.indices_h), stream=3)
    assert dx.numel() * 2 == len(medium.indices_h)
    g = G(P, dp, dx)
    deg = np.diff(g.indptr_h)
    assert (deg == 0).sum() > 0 and deg.max() > 300
    seeds = synth.seed_batches(g.n, 3000, seed=41)(2).numpy()
    hubs = np.argsort(-deg)[:40].astype(np.int32)
    for sampler in (R.NS, R.LABOR0):
        compare(P, g, seeds, (10, 10, 10), sampler, it=4, kappa=1, seed=19)
        compare(P, g, seeds[:700], (5, 10), sampler, it=21, kappa=16, seed=19)
        compare(P, g, hubs, (25, 10), sampler, it=2, kappa=1, seed=20)
    try:  # long lists cut into pieces, on lists that are nobody's mirror image
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, 256)
        compare(P, g, np.concatenate([hubs, seeds[:2000][~np.isin(seeds[:2000], hubs)]]), (10, 10, 10), R.LABOR0, it=6, kappa=1, seed=21)
    finally:
        P.coop_tune(P.COOP_TUNE_PIECE_LEN, 4096)
    compare_rw(P, g, seeds[:1500], (10, 10), 3, 100, 0.5, it=3, seed=22)
    with pytest.raises(P.CoopError) as e:
        P.coop_graph_load(g.indptr_d, g.indices_d, P.COOP_SYMMETRIC)
    assert e.value.code == -8


def test_fp32_phi_inv_stays_within_the_margin_for_every_input(P):
    """The filters in front of the exact blend (App. A.7, c > 0) settle a candidate by Phi^-1 in fp32 wherever ten times
    kPhiInvF32Gap cannot change the outcome.  The distance between that fp32 evaluation (this GPU's log, sqrt and
    reciprocal instructions) and the binary64 definition is measured here for all 2^32 uniforms and must stay below the
    constant that the kernels are compiled with.  Spot values of the measurement are checked against the oracle's kit and
    a numpy restatement of the fp32 form, so that the measurement itself is pinned to something outside the library."""
    from test_blend_prefilter import GAP, approx_phi_inv_f32
    gap, arg = P.coop_selftest_phi_inv_gap(0, 1 << 32)
    assert 0.0 < gap < GAP, (gap, arg)
    L = R.lib()
    # the reported maximum is reproduced at the reported input by the oracle's binary64 kit and numpy's fp32 arithmetic
    # (numpy's log / sqrt / division are correctly rounded, the GPU's are good to an ulp or so, and the rational form
    # amplifies an ulp a hundredfold where its terms cancel: agreement to 2e-5, a twentieth of the margin)
    at_arg = abs(float(approx_phi_inv_f32(arg)) - L.coopref_phi_inv_u32(arg))
    assert abs(at_arg - gap) < 2e-5, (gap, arg, at_arg)
    rng = np.random.default_rng(3)
    for U in [0, 1, 0xFFFFFFFF, 0x7FFFFFFF, 0x80000000, int(0.02425 * 2**32), int(0.02425 * 2**32) + 1] + [int(x) for x in rng.integers(0, 1 << 32, 40)]:
        one, _ = P.coop_selftest_phi_inv_gap(U, 1)
        assert abs(one - abs(float(approx_phi_inv_f32(U)) - L.coopref_phi_inv_u32(U))) < 2e-5, U
        assert one <= gap
    # sub-ranges: the maximum over the halves is the maximum over the whole; an empty range gives 0
    lo, _ = P.coop_selftest_phi_inv_gap(0, 1 << 31)
    hi, _ = P.coop_selftest_phi_inv_gap(1 << 31, 1 << 31)
    assert max(lo, hi) == gap and P.coop_selftest_phi_inv_gap(5, 0)[0] == 0.0


def test_graph_memory_from_the_callers_allocator(P, medium):
    """coop_graph_load_with: the index of reverse positions of a COOP_SYMMETRIC graph is obtained from the caller's allocator
    (here torch's), not from hipMalloc; sampling through it (lists above 64 entries served from the neighbours' side) gives the
    oracle's blocks, and an allocator that fails gives COOP_E_NOMEM."""
    import ctypes as C
    from paper_2310_12403_amd import binding
    g = P.coop_graph_load(medium.indptr_d, medium.indices_d, P.COOP_VALIDATE | P.COOP_SYMMETRIC, torch_memory=True)
    held = sum(t.numel() for t in g._memory.tensors.values())      # torch tensors behind the handle
    assert held >= 4 * len(medium.indices_h)
    class Wrapped:
        indptr_h, indices_h, graph, n = medium.indptr_h, medium.indices_h, g, medium.n
    seeds = synth.seed_batches(medium.n, 3000, seed=71)(1).numpy()
    try:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 64)
        compare(P, Wrapped, seeds, (10, 10, 10), R.LABOR0, it=2, kappa=1, seed=5)
    finally:
        P.coop_tune(P.COOP_TUNE_ENUM_DEGREE, 8192)
    g.close()
    failing = binding.ALLOC_FN(lambda ctx, nbytes, tag: None)
    h = C.c_void_p()
    rc = P.lib().coop_graph_load_with(C.c_void_p(medium.indptr_d.data_ptr()), C.c_void_p(medium.indices_d.data_ptr()), medium.n,
                                      len(medium.indices_h), P.COOP_SYMMETRIC, C.cast(failing, C.c_void_p), None, None, C.byref(h))
    assert rc == -5 and not h.value
