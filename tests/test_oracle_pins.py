"""Pins for the CPU oracle: it is checked against things other than itself.

  - the published Philox4x32-10 known-answer vectors (tests/golden/) and an independent
    pure-Python Philox;
  - a pure-Python brute force of NS / LABOR-0 / Eq. (2) on tiny graphs (sets and loops);
  - structural invariants, the full-fanout = BFS-ball reduction (App. A.1.2, last paragraph),
    exact nestedness (Sec. 3.1 / proof of Thm 3.1), closed-form expectations;
  - scipy's ndtr / ndtri for the Phi kit of App. A.7, and the identities n(0) = n1, n(1) = n2;
  - numpy fancy indexing for the gather, a textbook OrderedDict LRU for the cache.
"""
import collections
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.special import ndtr, ndtri
from scipy import stats

import synth
from oracle import coopref as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M32 = 0xFFFFFFFF


# --------------------------------------------------------------------------- #
# independent pure-Python restatements
# --------------------------------------------------------------------------- #
def py_philox(ctr, key, rounds=10):
    c = [int(x) & M32 for x in ctr]
    k = [int(x) & M32 for x in key]
    for _ in range(rounds):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & M32, (p0 >> 32) ^ c[3] ^ k[1], p0 & M32]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return c


def py_mix32(x):
    x ^= x >> 16
    x = (x * 0x7FEB352D) & M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & M32
    x ^= x >> 16
    return x


def py_unmix32(y):
    """Inverse of py_mix32, step by step (each xor-shift and each odd multiply is invertible)."""
    def unshift(v, s):
        r = v
        for _ in range(32 // s + 1):
            r = v ^ (r >> s)
        return r
    y = unshift(y, 16)
    y = (y * pow(0x846CA68B, -1, 1 << 32)) & M32
    y = unshift(y, 15)
    y = (y * pow(0x7FEB352D, -1, 1 << 32)) & M32
    return unshift(y, 16)


def py_keys(seed, sampler, layer, g):
    return py_philox([g & M32, (g >> 32) & M32, layer | (sampler << 8), 0x434F4F50], [seed & M32, seed >> 32])


def py_uniform(seed, sampler, layer, g, t, s):
    K = py_keys(seed, sampler, layer, g)
    a = py_mix32(t ^ K[0]) ^ K[1]
    if sampler == R.LABOR0:
        return a
    return py_mix32(a ^ py_mix32(s ^ K[2])) ^ K[3]


def brute_sample(indptr, indices, seeds, fanouts, sampler, seed, g):
    """Eq. (2) with sampled neighbourhoods, for c = 0 (variate = first Philox word)."""
    out = []
    dst = [int(x) for x in seeds]
    for layer, k in enumerate(fanouts):
        ptr, cols, eids = [0], [], []
        for s in dst:
            beg, end = int(indptr[s]), int(indptr[s + 1])
            d = end - beg
            nbrs = [int(indices[p]) for p in range(beg, end)]
            if sampler == R.LABOR0:
                keep = [j for j, t in enumerate(nbrs) if py_uniform(seed, sampler, layer, g, t, s) * d <= (k << 32)]
            elif d <= k:
                keep = list(range(d))
            else:
                ranked = sorted((py_uniform(seed, sampler, layer, g, t, s), j) for j, t in enumerate(nbrs))
                keep = sorted(j for _, j in ranked[:k])
            for j in keep:
                cols.append(nbrs[j])
                eids.append(beg + j)
            ptr.append(len(cols))
        src = list(dst)
        seen = set(dst)
        for t in cols:
            if t not in seen:
                seen.add(t)
                src.append(t)
        where = {v: i for i, v in enumerate(src)}
        out.append(dict(dst_ids=dst, indptr=ptr, col_global=cols, eid=eids, src_ids=src,
                        col_local=[where[t] for t in cols]))
        dst = src
    return out


def small_graph(n=80, avg=7, hub=40, seed=3):
    rng = np.random.default_rng(seed)
    m = n * avg // 2
    src = rng.integers(0, n, m)
    dst = rng.integers(0, n, m)
    src = np.concatenate([src, np.zeros(hub, dtype=np.int64)])          # vertex 0 is a hub
    dst = np.concatenate([dst, rng.choice(np.arange(1, n), hub, replace=False)])
    A = sp.coo_matrix((np.ones(len(src)), (src, dst)), shape=(n, n)).tocsr()
    A = A + A.T
    A.setdiag(0)
    A.eliminate_zeros()
    A.sort_indices()
    return A.indptr.astype(np.int64), A.indices.astype(np.int32)


@pytest.fixture(scope="module")
def tiny():
    ip, ix = synth.rmat_csr()
    return ip.numpy(), ix.numpy()


# --------------------------------------------------------------------------- #
# generator
# --------------------------------------------------------------------------- #
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert R.philox4x32_10(w[0:4], w[4:6]) == w[6:10]
        assert py_philox(w[0:4], w[4:6]) == w[6:10]


def test_philox_matches_independent_python():
    rng = np.random.default_rng(1)
    for _ in range(300):
        ctr = rng.integers(0, 2**32, 4).tolist()
        key = rng.integers(0, 2**32, 2).tolist()
        assert R.philox4x32_10(ctr, key) == py_philox(ctr, key)


def test_mixer_is_a_well_mixing_permutation():
    rng = np.random.default_rng(7)
    xs = rng.integers(0, 2**32, 4000).tolist() + [0, 1, M32, 2**31]
    for x in xs:
        y = R.mix32(x)
        assert y == py_mix32(x) and py_unmix32(y) == x          # a bijection: the inverse exists
    # avalanche: flipping any input bit flips every output bit about half the time
    xs = rng.integers(0, 2**32, 20000, dtype=np.uint64)

    def mix_np(x):
        x = x ^ (x >> 16)
        x = (x * 0x7FEB352D) & M32
        x = x ^ (x >> 15)
        x = (x * 0x846CA68B) & M32
        return x ^ (x >> 16)

    base = mix_np(xs)
    assert int(base[5]) == R.mix32(int(xs[5]))
    for i in range(32):
        diff = base ^ mix_np(xs ^ np.uint64(1 << i))
        for o in range(32):
            assert abs(float(((diff >> np.uint64(o)) & np.uint64(1)).mean()) - 0.5) < 0.03


def test_layer_keys_are_philox_words():
    rng = np.random.default_rng(3)
    for _ in range(100):
        seed = int(rng.integers(0, 2**63)) * 2 + 1
        sampler, layer, g = int(rng.integers(0, 2)), int(rng.integers(0, 200)), int(rng.integers(0, 2**62))
        assert R.layer_keys(seed, sampler, layer, g) == py_keys(seed, sampler, layer, g)
    # distinct (seed, sampler, layer, group) give unrelated keys
    ks = {tuple(R.layer_keys(1, sa, la, g)) for sa in (0, 1) for la in range(4) for g in range(50)}
    assert len(ks) == 400


def test_variate_counter_layout():
    rng = np.random.default_rng(2)
    for _ in range(200):
        seed = int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2))
        sampler = int(rng.integers(0, 2))
        layer = int(rng.integers(0, 5))
        it = int(rng.integers(0, 2**40))
        t, s = int(rng.integers(0, 2**31)), int(rng.integers(0, 2**31))
        assert R.variate(seed, sampler, layer, it, 1, t, s) == py_uniform(seed, sampler, layer, it, t, s)
    # LABOR's variate ignores s (one number per source vertex, App. A.1.2)
    assert R.variate(5, R.LABOR0, 1, 9, 1, 123, 7) == R.variate(5, R.LABOR0, 1, 9, 1, 123, 99)
    assert R.variate(5, R.NS, 1, 9, 1, 123, 7) != R.variate(5, R.NS, 1, 9, 1, 123, 99)


# --------------------------------------------------------------------------- #
# brute force on tiny graphs
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
@pytest.mark.parametrize("fanouts", [(3, 2), (1, 5, 2), (64,)])
def test_sample_equals_brute_force(sampler, fanouts):
    indptr, indices = small_graph()
    rng = np.random.default_rng(11)
    for trial in range(3):
        seeds = rng.choice(80, 9, replace=False).astype(np.int32)
        seed, g = 1000 + trial, 5 * trial
        got = R.sample(indptr, indices, seeds, fanouts, sampler, it=g, kappa=1, seed=seed)
        want = brute_sample(indptr, indices, seeds, fanouts, sampler, seed, g)
        for b, w in zip(got, want):
            for name in ("dst_ids", "indptr", "col_global", "eid", "src_ids", "col_local"):
                assert b[name].tolist() == w[name], name


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_repeated_neighbours_against_brute_force(sampler):
    """A multigraph with unsorted lists: a neighbour listed several times has one variate, so NS breaks the tie by list
    position (the brute force sorts (variate, position) pairs) and LABOR-0 keeps every copy or none."""
    rng = np.random.default_rng(23)
    n = 60
    deg = rng.integers(0, 30, n)
    deg[0] = 90
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    indices = np.concatenate([rng.integers(0, n, max(1, d // 4))[rng.integers(0, max(1, d // 4), d)] for d in deg]).astype(np.int32)
    assert any(len(set(indices[indptr[v]:indptr[v + 1]])) < deg[v] // 2 for v in range(n))       # the copies are there
    for trial, fanouts in enumerate([(3, 2), (7,), (2, 2, 2)]):
        seeds = np.concatenate([[0], 1 + rng.choice(n - 1, 8, replace=False)]).astype(np.int32)
        seed, g = 77 + trial, 3 * trial
        got = R.sample(indptr, indices, seeds, fanouts, sampler, it=g, kappa=1, seed=seed)
        want = brute_sample(indptr, indices, seeds, fanouts, sampler, seed, g)
        for b, w in zip(got, want):
            for name in ("dst_ids", "indptr", "col_global", "eid", "src_ids", "col_local"):
                assert b[name].tolist() == w[name], name


def check_invariants(indptr, indices, blocks, seeds, fanouts, sampler):
    deg = np.diff(indptr)
    prev = np.asarray(seeds)
    for b, k in zip(blocks, fanouts):
        assert np.array_equal(b["dst_ids"], prev)
        n_dst, m = len(b["dst_ids"]), len(b["col_global"])
        assert b["indptr"][0] == 0 and b["indptr"][-1] == m and np.all(np.diff(b["indptr"]) >= 0)
        # every sampled edge exists, under its own destination
        assert np.array_equal(indices[b["eid"]], b["col_global"])
        owner = np.repeat(b["dst_ids"], np.diff(b["indptr"]))
        assert np.all(indptr[owner] <= b["eid"]) and np.all(b["eid"] < indptr[owner + 1])
        # adjacency order inside a destination, no edge twice
        for i in range(n_dst):
            seg = b["eid"][b["indptr"][i]:b["indptr"][i + 1]]
            assert np.all(np.diff(seg) > 0)
        cnt = np.diff(b["indptr"])
        if sampler == R.NS:
            assert np.array_equal(cnt, np.minimum(k, deg[b["dst_ids"]]))
        else:
            small = deg[b["dst_ids"]] <= k
            assert np.array_equal(cnt[small], deg[b["dst_ids"]][small])
        # S^{l+1}: S^l first, no duplicates, the union, first-appearance order
        src = b["src_ids"]
        assert np.array_equal(src[:n_dst], b["dst_ids"])
        assert len(np.unique(src)) == len(src)
        assert set(src.tolist()) == set(b["dst_ids"].tolist()) | set(b["col_global"].tolist())
        assert np.array_equal(src[b["col_local"]], b["col_global"])
        cat = np.concatenate([b["dst_ids"], b["col_global"]])
        _, first = np.unique(cat, return_index=True)
        assert np.array_equal(src, cat[np.sort(first)])
        prev = src


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_invariants_tiny_config(tiny, sampler):
    indptr, indices = tiny
    seeds = synth.seed_batches(len(indptr) - 1, 1024, seed=0)(0).numpy()
    blocks = R.sample(indptr, indices, seeds, (10, 10, 10), sampler, it=0, kappa=1, seed=0)
    check_invariants(indptr, indices, blocks, seeds, (10, 10, 10), sampler)


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_full_fanout_is_bfs_ball(tiny, sampler):
    """k >= max degree: both samplers use full neighbourhoods, so S^l is the l-hop ball of Eq. (2)."""
    indptr, indices = tiny
    n = len(indptr) - 1
    k = int(np.diff(indptr).max())
    seeds = np.array([5, 77, 4000, 9001], dtype=np.int32)
    blocks = R.sample(indptr, indices, seeds, (k, k), sampler, it=3, kappa=1, seed=9)
    A = sp.csr_matrix((np.ones(len(indices), dtype=np.int8), indices, indptr), shape=(n, n))
    x = np.zeros(n, dtype=bool)
    x[seeds] = True
    for b in blocks:
        x = x | (A.T @ x.astype(np.int32) > 0)      # S ∪ N(S); the graph is symmetric
        assert set(np.nonzero(x)[0].tolist()) == set(b["src_ids"].tolist())
        assert len(b["col_global"]) == int(np.diff(indptr)[b["dst_ids"]].sum())


@pytest.mark.parametrize("sampler", [R.NS, R.LABOR0])
def test_nestedness_exact(tiny, sampler):
    """The sampled neighbourhood of s depends on (s, layer, seed, iter) only, hence
    (A ∪ B)^l = A^l ∪ B^l as sets, and |S^l| is monotone and sub-additive in the batch."""
    indptr, indices = tiny
    get = synth.seed_batches(len(indptr) - 1, 512, seed=4)
    A, B = get(0).numpy(), get(1).numpy()
    fan = (10, 10, 10)
    kw = dict(it=7, kappa=1, seed=21)
    bA = R.sample(indptr, indices, A, fan, sampler, **kw)
    bB = R.sample(indptr, indices, B, fan, sampler, **kw)
    bAB = R.sample(indptr, indices, np.concatenate([A, B]), fan, sampler, **kw)
    for l in range(3):
        sA, sB, sAB = (set(x[l]["src_ids"].tolist()) for x in (bA, bB, bAB))
        assert sAB == sA | sB
        assert len(sAB) <= len(sA) + len(sB) and len(sAB) >= max(len(sA), len(sB))


def test_work_monotone_and_concave(tiny):
    """Thm 3.1: E|S^l| / |S^0| is nonincreasing; Thm 3.2: E|S^l| is concave in the batch size."""
    indptr, indices = tiny
    n = len(indptr) - 1
    sizes = [256, 512, 1024, 2048, 4096]
    acc = np.zeros((len(sizes), 3))
    for p in range(8):
        perm = synth.permutation(n, 900 + p).numpy().astype(np.int32)
        for i, b in enumerate(sizes):
            blocks = R.sample(indptr, indices, perm[:b], (10, 10, 10), R.LABOR0, it=p, kappa=1, seed=p)
            acc[i] += [len(x["src_ids"]) for x in blocks]
    acc /= 8
    ratio = acc / np.array(sizes)[:, None]
    assert np.all(np.diff(ratio, axis=0) < 0)
    # concavity on the doubling grid: the increment over [b, 2b] is at most twice that over [b/2, b]
    inc = np.diff(acc, axis=0)
    assert np.all(inc[1:] <= 2 * inc[:-1] * 1.02)


# --------------------------------------------------------------------------- #
# closed-form expectations (Monte Carlo over the seed)
# --------------------------------------------------------------------------- #
def test_labor0_and_ns_expectations():
    indptr, indices = small_graph(n=120, avg=12, hub=80, seed=8)
    deg = np.diff(indptr)
    n = len(deg)
    seeds = np.arange(0, 40, dtype=np.int32)        # includes the hub (vertex 0)
    k, trials = 4, 1500
    cnt_sum = np.zeros(len(seeds))
    cnt_sq = np.zeros(len(seeds))
    hit = {R.NS: np.zeros(n), R.LABOR0: np.zeros(n)}
    edges = {R.NS: 0, R.LABOR0: 0}
    for tr in range(trials):
        for sampler in (R.NS, R.LABOR0):
            b = R.sample(indptr, indices, seeds, (k,), sampler, it=tr, kappa=1, seed=77)[0]
            edges[sampler] += len(b["col_global"])
            hit[sampler][np.unique(b["col_global"])] += 1
            if sampler == R.LABOR0:
                c = np.diff(b["indptr"])
                cnt_sum += c
                cnt_sq += c * c
    d = deg[seeds].astype(float)
    mean_want = np.minimum(k, d)
    var_want = np.where(d > k, k * (1 - k / d), 0.0)
    mean = cnt_sum / trials
    var = cnt_sq / trials - mean**2
    # per-seed Binomial(d, k/d): mean k, variance k(1 - k/d)
    assert np.all(np.abs(mean - mean_want) <= 4 * np.sqrt(var_want / trials) + 1e-12)
    assert np.all(np.abs(var - var_want) <= 0.25 * var_want + 1e-12)
    # E|E^0| = sum_s min(k, d_s) for both samplers (exact for NS)
    assert edges[R.NS] == trials * int(mean_want.sum())
    assert abs(edges[R.LABOR0] / trials - mean_want.sum()) <= 4 * math.sqrt(var_want.sum() / trials)
    # P(t sampled): LABOR-0 max_s min(1, k/d_s); NS 1 - prod_s (1 - min(1, k/d_s)), over seeds s adjacent to t
    pi_labor = np.zeros(n)
    pi_ns_c = np.ones(n)
    for s in seeds:
        p = min(1.0, k / deg[s])
        nb = indices[indptr[s]:indptr[s + 1]]
        pi_labor[nb] = np.maximum(pi_labor[nb], p)
        pi_ns_c[nb] *= 1 - p
    for sampler, pi in ((R.LABOR0, pi_labor), (R.NS, 1 - pi_ns_c)):
        f = hit[sampler] / trials
        assert np.all(np.abs(f - pi) <= 4.5 * np.sqrt(pi * (1 - pi) / trials) + 1e-12)
    assert pi_labor.sum() < (1 - pi_ns_c).sum()     # LABOR-0 samples fewer vertices than NS


# --------------------------------------------------------------------------- #
# App. A.7: dependent variates
# --------------------------------------------------------------------------- #
def test_kappa_group_identities(tiny):
    indptr, indices = tiny
    seeds = synth.seed_batches(len(indptr) - 1, 256, seed=1)(2).numpy()
    fan = (5, 5)

    def same(a, b):
        return all(np.array_equal(x[k], y[k]) for x, y in zip(a, b) for k in x)

    for sampler in (R.NS, R.LABOR0):
        base = R.sample(indptr, indices, seeds, fan, sampler, it=3, kappa=1, seed=5)
        assert same(base, R.sample(indptr, indices, seeds, fan, sampler, it=3 * 16, kappa=16, seed=5))
        assert not same(base, R.sample(indptr, indices, seeds, fan, sampler, it=3 * 16 + 1, kappa=16, seed=5))
        zero = R.sample(indptr, indices, seeds, fan, sampler, it=0, kappa=1, seed=5)
        assert same(zero, R.sample(indptr, indices, seeds, fan, sampler, it=123456, kappa=0, seed=5))


def test_blend_formula_against_scipy():
    rng = np.random.default_rng(5)
    worst = 0
    for _ in range(3000):
        seed, t, s = int(rng.integers(0, 2**62)), int(rng.integers(0, 2**31)), int(rng.integers(0, 2**31))
        kappa = int(rng.integers(2, 300))
        i = int(rng.integers(1, kappa))
        g = int(rng.integers(0, 1000))
        sampler, layer = int(rng.integers(0, 2)), int(rng.integers(0, 3))
        u1 = (py_uniform(seed, sampler, layer, g, t, s) + 0.5) / 2**32
        u2 = (py_uniform(seed, sampler, layer, g + 1, t, s) + 0.5) / 2**32
        c = i / kappa
        n = math.cos(c * math.pi / 2) * ndtri(u1) + math.sin(c * math.pi / 2) * ndtri(u2)
        want = ndtr(n) * 2**32
        got = R.variate(seed, sampler, layer, g * kappa + i, kappa, t, s)
        worst = max(worst, abs(got - want))
    assert worst <= 16      # Phi^-1 is good to 1.15e-9 relative: a handful of 2^-32 grid steps


def test_blend_limits_uniformity_and_correlation():
    ts = np.arange(20000)
    K = 1 << 20
    # c -> 1: the variate approaches the next group's uniform (n(1) = n2)
    near = np.array([R.variate(3, R.LABOR0, 0, 5 * K + K - 1, K, int(t)) for t in ts[:3000]], dtype=np.float64)
    nxt = np.array([R.variate(3, R.LABOR0, 0, 6, 1, int(t)) for t in ts[:3000]], dtype=np.float64)
    assert np.max(np.abs(near - nxt)) / 2**32 < 1e-4
    # c -> 0+: close to this group's uniform (n(0) = n1)
    lo = np.array([R.variate(3, R.LABOR0, 0, 5 * K + 1, K, int(t)) for t in ts[:3000]], dtype=np.float64)
    cur = np.array([R.variate(3, R.LABOR0, 0, 5, 1, int(t)) for t in ts[:3000]], dtype=np.float64)
    assert np.max(np.abs(lo - cur)) / 2**32 < 1e-4
    # uniform for every c (n(c) ~ N(0,1)), and corr(n(c1), n(c2)) = cos((c2 - c1) pi / 2) inside a group
    kappa = 8
    r = {i: np.array([R.variate(9, R.NS, 1, 40 + i, kappa, int(t), 17) for t in ts], dtype=np.float64) for i in (1, 3, 6)}
    for i, x in r.items():
        assert stats.kstest((x + 0.5) / 2**32, "uniform").pvalue > 1e-3
    nn = {i: ndtri((x + 0.5) / 2**32) for i, x in r.items()}
    for a, b in ((1, 3), (1, 6), (3, 6)):
        want = math.cos((b - a) / kappa * math.pi / 2)
        got = np.corrcoef(nn[a], nn[b])[0, 1]
        assert abs(got - want) < 4 / math.sqrt(len(ts))


def test_phi_kit_against_scipy():
    L = R.lib()
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.uniform(0.5, 4, 1000), 10.0 ** rng.uniform(-12, 12, 1000)])
    assert max(abs(L.coopref_rcp(x) * x - 1) for x in xs) < 1e-15
    assert max(abs(L.coopref_rsqrt(x) ** 2 * x - 1) for x in xs) < 2e-15
    xs = 10.0 ** rng.uniform(-11, 0, 2000)
    assert max(abs(L.coopref_log(x) - math.log(x)) / max(abs(math.log(x)), 1e-3) for x in xs) < 1e-14
    ys = -rng.uniform(0, 60, 2000)
    assert max(abs(L.coopref_exp(y) / math.exp(y) - 1) for y in ys) < 1e-14
    Us = np.concatenate([rng.integers(0, 2**32, 8000), np.arange(0, 500), 2**32 - 1 - np.arange(0, 500),
                         rng.integers(0, 2**20, 2000), 2**31 + np.arange(-3, 3)])
    for U in Us:
        U = int(U)
        x = L.coopref_phi_inv_u32(U)
        ref = ndtri((U + 0.5) / 2**32)
        assert abs(x - ref) <= 1.2e-9 * abs(ref) + 1e-15
        assert L.coopref_phi_inv_u32(M32 - U) == -x                  # exact mirror symmetry
        assert abs(L.coopref_phi_to_u32(x) - U) <= 2                 # Phi(Phi^-1(u)) = u on the grid
    for a in np.concatenate([rng.uniform(0, 9, 5000), np.linspace(2.9, 3.1, 401), [0.0]]):
        assert abs(L.coopref_qtail(a) / ndtr(-a) - 1) < 1e-10
        lo, hi = L.coopref_phi_to_u32(-a), L.coopref_phi_to_u32(a)
        assert lo + hi == M32 or a == 0.0
    assert L.coopref_phi_to_u32(0.0) == 2**31 - 1
    assert L.coopref_phi_to_u32(-9.5) == 0 and L.coopref_phi_to_u32(9.5) == M32


# --------------------------------------------------------------------------- #
# gather, cache, error paths
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("dtype,dim", [(np.float32, 64), (np.float16, 128), (np.float32, 602), (np.float16, 3)])
def test_gather_is_fancy_indexing(dtype, dim):
    rng = np.random.default_rng(0)
    feat = rng.standard_normal((500, dim)).astype(dtype)
    ids = rng.integers(0, 500, 1234).astype(np.int32)
    out = R.gather(feat, ids)
    assert out.tobytes() == feat[ids].tobytes()
    assert R.gather(feat, np.zeros(0, np.int32)).shape == (0, dim)
    with pytest.raises(R.OracleError):
        R.gather(feat, np.array([500], np.int32))


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_gather_mean_is_segment_mean(dtype):
    """Eq. (1) with a mean aggregator: against numpy's own segmented sum, plus the degenerate rows."""
    rng = np.random.default_rng(3)
    feat = (rng.standard_normal((300, 37)) * 3).astype(dtype)
    if dtype == np.float16:
        feat[0, 0] = np.float16(6e-8)                      # a subnormal half
    deg = rng.integers(0, 9, 120)
    deg[:3] = [0, 1, 0]
    indptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    col = rng.integers(0, 300, indptr[-1]).astype(np.int32)
    col[0] = 0
    got = R.gather_mean(feat, indptr, col)
    rows = feat[col].astype(np.float64)
    want = np.zeros((120, 37))
    nz = deg > 0
    want[nz] = np.add.reduceat(rows, indptr[:-1][nz], axis=0) / deg[nz][:, None]
    assert np.allclose(got, want, rtol=1e-13, atol=1e-300)
    assert np.all(got[0] == 0) and np.all(got[2] == 0)                       # no edges -> zero row
    assert np.array_equal(got[1], feat[col[indptr[1]]].astype(np.float64))   # one edge -> that row, exactly
    with pytest.raises(R.OracleError):
        R.gather_mean(feat, np.array([0, 1], np.int64), np.array([300], np.int32))


def textbook_lru(capacity):
    od = collections.OrderedDict()

    def access(v):
        if v in od:
            od.move_to_end(v)
            return True
        if capacity == 0:
            return False
        if len(od) >= capacity:
            od.popitem(last=False)
        od[v] = True
        return False

    return od, access


@pytest.mark.parametrize("capacity", [0, 1, 7, 50, 400])
def test_cache_is_textbook_lru_on_hits_then_misses(capacity):
    rng = np.random.default_rng(capacity)
    nV = 300
    cache = R.Cache(capacity, nV)
    od, access = textbook_lru(capacity)
    seen = set()
    for it in range(60):
        ids = rng.choice(nV, int(rng.integers(1, 90)), replace=False).astype(np.int32)
        before = set(od.keys())
        n_miss, hit = cache.access(ids)
        assert hit.tolist() == [int(v) in before for v in ids]
        # hits are touched first: only non-hit entries can be evicted by this batch's misses
        for v in ids[hit]:
            assert access(int(v))
        for v in ids[~hit]:
            assert not access(int(v))
        assert n_miss == int((~hit).sum())
        assert cache.size() == len(od)
        assert all(cache.contains(v) == (v in od) for v in range(nV))
        if capacity == 0:
            assert n_miss == len(ids)
        if capacity >= nV:
            assert n_miss == len(set(ids.tolist()) - seen)       # compulsory misses only
        seen |= set(ids.tolist())


def test_error_codes(tiny):
    indptr, indices = tiny
    ok = np.array([1, 2, 3], np.int32)
    for bad_seeds, code in ((np.array([1, 2, 1], np.int32), R.E_DUPSEED), (np.array([1, 1 << 20], np.int32), R.E_RANGE),
                            (np.array([-1], np.int32), R.E_RANGE)):
        with pytest.raises(R.OracleError) as e:
            R.sample(indptr, indices, bad_seeds, (3,), R.NS)
        assert e.value.code == code
    for fan in ((), (0,), (3, -1)):
        with pytest.raises(R.OracleError) as e:
            R.sample(indptr, indices, ok, fan, R.NS)
        assert e.value.code == R.E_ARG
    with pytest.raises(R.OracleError):
        R.sample(indptr, indices, ok, (3,), 7)
    empty = R.sample(indptr, indices, np.zeros(0, np.int32), (3, 3), R.LABOR0)
    assert all(len(b["src_ids"]) == 0 and len(b["col_global"]) == 0 and b["indptr"].tolist() == [0] for b in empty)


# --------------------------------------------------------------------------- #
# Random-walk sampler (App. A.1.3)
# --------------------------------------------------------------------------- #
def py_rw_draw(K, c, s):
    return py_mix32(py_mix32(c ^ K[0]) ^ K[1] ^ py_mix32(s ^ K[2])) ^ K[3]


def brute_rw(indptr, indices, seeds, fanouts, o, a, p, seed, it):
    """a walks of length o per destination, restart with probability p, the k most visited vertices; written from
    the definition with Python containers (Counter, sorted), no shared arithmetic with the C oracle."""
    P = (1 << 32) if p >= 1.0 else int(p * 4294967296.0)
    out = []
    dst = [int(x) for x in seeds]
    for layer, k in enumerate(fanouts):
        K = py_keys(seed, R.RW, layer, it)
        ptr, cols, counts = [0], [], []
        for s in dst:
            nbr = lambda v: [int(x) for x in indices[int(indptr[v]):int(indptr[v + 1])]]
            visits = collections.Counter()
            if nbr(s):
                for w in range(a):
                    cur = s
                    for step in range(o):
                        c = 2 * (w * o + step)
                        base = s if step == 0 or py_rw_draw(K, c + 1, s) < P else cur
                        cand = nbr(base)
                        if not cand:
                            break
                        cur = cand[(py_rw_draw(K, c, s) * len(cand)) >> 32]
                        visits[cur] += 1
            top = sorted(visits.items(), key=lambda vc: (-vc[1], vc[0]))[:k]
            cols += [v for v, _ in top]
            counts += [n for _, n in top]
            ptr.append(len(cols))
        src = list(dst)
        seen = set(dst)
        for t in cols:
            if t not in seen:
                seen.add(t)
                src.append(t)
        where = {v: i for i, v in enumerate(src)}
        out.append(dict(dst_ids=dst, indptr=ptr, col_global=cols, eid=counts, src_ids=src, col_local=[where[t] for t in cols]))
        dst = src
    return out


@pytest.mark.parametrize("o,a,p,fanouts", [(3, 100, 0.5, (10, 10)), (1, 7, 0.0, (3,)), (4, 20, 0.25, (5, 2, 4)), (2, 50, 1.0, (8,)),
                                            (33, 32, 0.5, (6, 3)), (3, 600, 0.3, (40,))])   # (the last two: more than 1,024 steps per destination)
def test_rw_equals_brute_force(o, a, p, fanouts):
    indptr, indices = small_graph()
    seeds = np.array([5, 0, 17, 33, 60, 2], dtype=np.int32)
    got = R.sample(indptr, indices, seeds, fanouts, R.RW, it=11, seed=77, rw=(o, a, p))
    want = brute_rw(indptr, indices, seeds, fanouts, o, a, p, 77, 11)
    for b, w in zip(got, want):
        for name in ("dst_ids", "indptr", "col_global", "eid", "src_ids", "col_local"):
            assert list(b[name]) == list(w[name]), name


def test_rw_draw_layout():
    K = py_keys(9, R.RW, 2, 123456789012)
    for s, c in [(0, 0), (5, 1), (1 << 31, 599), (77, 2 * 1023 + 1)]:
        assert R.rw_draw(9, 2, 123456789012, s, c) == py_rw_draw(K, c, s)
    assert R.layer_keys(9, R.RW, 2, 5) != R.layer_keys(9, R.NS, 2, 5)


def test_rw_invariants_and_reach(tiny):
    """Every kept source lies within o hops of its destination; counts are sorted, positive, sum to at most a*o (to
    exactly a*o when the fanout keeps everything and no walk meets a dead end); a vertex without neighbours keeps none."""
    indptr, indices = tiny
    n = len(indptr) - 1
    A = sp.csr_matrix((np.ones(len(indices), dtype=np.int64), indices, indptr), shape=(n, n))
    o, a = 3, 40
    reach = A.copy()
    step = A.copy()
    for _ in range(o - 1):
        step = (step @ A)
        step.data[:] = 1
        reach = reach + step
    reach = reach.tocsr()
    deg = np.diff(indptr)
    seeds = synth.seed_batches(n, 300, seed=4)(0).numpy()
    iso = np.nonzero(deg == 0)[0][:2].astype(np.int32)
    seeds = np.unique(np.concatenate([seeds, iso])).astype(np.int32)
    for k in (5, 1000):
        b = R.sample(indptr, indices, seeds, (k,), R.RW, it=2, seed=8, rw=(o, a, 0.5))[0]
        for i, s in enumerate(seeds):
            lo, hi = b["indptr"][i], b["indptr"][i + 1]
            cols, cnt = b["col_global"][lo:hi], b["eid"][lo:hi]
            assert hi - lo <= k and len(set(cols)) == len(cols)
            if deg[s] == 0:
                assert hi == lo
                continue
            allowed = set(reach.indices[reach.indptr[s]:reach.indptr[s + 1]])
            assert set(cols) <= allowed
            assert all(c >= 1 for c in cnt) and cnt.sum() <= a * o
            order = sorted(zip(-cnt, cols))
            assert [v for _, v in order] == list(cols)
            if k == 1000:   # symmetric graph: no dead ends, every step visits something
                assert cnt.sum() == a * o
        assert np.array_equal(b["src_ids"][:len(seeds)], seeds)
        assert np.array_equal(b["src_ids"][b["col_local"]], b["col_global"])


def test_rw_restart_probability_and_first_step():
    """Path 0-1-2-3 from s = 1 with o = 2: the second step lands on s itself exactly when the walk does not restart
    (N(0) = {1}, N(2) = {1, 3}); restarts land on 0 or 2.  So visits(0)+visits(2) = a + #restarts, and the number of
    restarts is Binomial(a, p).  Star graph from a leaf with p = 0: the centre is visited exactly a times."""
    indptr = np.array([0, 1, 3, 5, 6], dtype=np.int64)
    indices = np.array([1, 0, 2, 1, 3, 2], dtype=np.int32)
    a = 500
    for p in (0.0, 0.25, 0.5, 1.0):
        tot = 0
        runs = 20
        for it in range(runs):
            b = R.sample(indptr, indices, np.array([1], dtype=np.int32), (10,), R.RW, it=it, seed=3, rw=(2, a, p))[0]
            visits = dict(zip(b["col_global"].tolist(), b["eid"].tolist()))
            assert sum(visits.values()) == 2 * a
            first_and_restarts = visits.get(0, 0) + visits.get(2, 0)
            tot += first_and_restarts - a
            if p == 0.0:
                assert first_and_restarts == a
            if p == 1.0:
                assert first_and_restarts == 2 * a
        mean, sd = runs * a * p, math.sqrt(runs * a * p * (1 - p))
        assert abs(tot - mean) <= 4 * sd + 1e-9
    # first step uniform over N(s): vertex 2 has neighbours {1, 3}
    c1 = 0
    for it in range(20):
        b = R.sample(indptr, indices, np.array([2], dtype=np.int32), (10,), R.RW, it=it, seed=4, rw=(1, a, 0.0))[0]
        visits = dict(zip(b["col_global"].tolist(), b["eid"].tolist()))
        assert sum(visits.values()) == a and set(visits) <= {1, 3}
        c1 += visits.get(1, 0)
    assert abs(c1 - 10 * a) <= 4 * math.sqrt(20 * a * 0.25)
    # star: centre 0, leaves 1..6
    leaves = 6
    ip = np.array([0, leaves] + [leaves + i + 1 for i in range(leaves)], dtype=np.int64)
    ix = np.array(list(range(1, leaves + 1)) + [0] * leaves, dtype=np.int32)
    b = R.sample(ip, ix, np.array([3], dtype=np.int32), (10,), R.RW, it=0, seed=1, rw=(2, 500, 0.0))[0]
    visits = dict(zip(b["col_global"].tolist(), b["eid"].tolist()))
    assert visits[0] == 500 and b["col_global"][0] == 0 and sum(visits.values()) == 1000
    per_leaf = np.array([visits.get(v, 0) for v in range(1, leaves + 1)])
    assert stats.chisquare(per_leaf).pvalue > 1e-4


def test_rw_error_codes_and_kappa_free(tiny):
    indptr, indices = tiny
    seeds = np.array([1, 2, 3], dtype=np.int32)
    for bad in ((0, 10, 0.5), (3, 0, 0.5), (3, 10, 1.5), (3, 10, -0.1), (1 << 11, 1 << 10, 0.5)):
        with pytest.raises(R.OracleError) as e:
            R.sample(indptr, indices, seeds, (5,), R.RW, rw=bad)
        assert e.value.code == R.E_ARG
    with pytest.raises(R.OracleError) as e:
        R.sample(indptr, indices, np.array([1, 1], dtype=np.int32), (5,), R.RW, rw=(3, 10, 0.5))
    assert e.value.code == R.E_DUPSEED
    a = R.sample(indptr, indices, seeds, (5, 5), R.RW, it=3, seed=1, rw=(3, 10, 0.5))
    b = R.sample(indptr, indices, seeds, (5, 5), R.RW, it=4, seed=1, rw=(3, 10, 0.5))
    assert any(not np.array_equal(x["col_global"], y["col_global"]) for x, y in zip(a, b))   # fresh draws per iteration


# ---- ids grouped by owner (Sec. 3.1, Algorithm 1: the local half of the id redistribution) ----------------------------
@pytest.mark.parametrize("n_parts", [1, 3, 8, 64])
def test_bucket_by_owner_ranges_closed_form(n_parts):
    """owner(v) = floor(v P / |V|) = p exactly when ceil(p |V| / P) <= v < ceil((p + 1) |V| / P): the oracle's groups
    against those boundaries, and against a stable argsort of the owners (a library routine)."""
    rng = np.random.default_rng(5)
    nv = 100003
    ids = rng.integers(0, nv, size=20011).astype(np.int32)
    out, origin, offsets = R.bucket_by_owner(ids, nv, n_parts, 0)
    assert offsets[0] == 0 and offsets[-1] == len(ids) and np.all(np.diff(offsets) >= 0)
    assert np.array_equal(out, ids[origin])
    bounds = [-(-p * nv // n_parts) for p in range(n_parts + 1)]   # ceil(p |V| / P)
    for p in range(n_parts):
        grp, org = out[offsets[p]:offsets[p + 1]], origin[offsets[p]:offsets[p + 1]]
        assert np.all((grp >= bounds[p]) & (grp < bounds[p + 1]))
        assert np.all(np.diff(org) > 0)                            # original order kept within the group
    owner = (ids.astype(np.int64) * n_parts) // nv
    assert np.array_equal(origin, np.argsort(owner, kind="stable").astype(np.int32))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(owner, minlength=n_parts))]))


def test_bucket_by_owner_hashed_against_independent_mixer():
    """The random partition: owners recomputed with the pure-Python mixer of this file; groups of about equal size."""
    rng = np.random.default_rng(6)
    nv, n_parts, seed = 50000, 8, (7 << 32) | 12345
    ids = rng.permutation(nv)[:12000].astype(np.int32)
    out, origin, offsets = R.bucket_by_owner(ids, nv, n_parts, 1, seed=seed)
    key = (seed ^ (seed >> 32)) & 0xFFFFFFFF
    owner = np.array([(py_mix32(int(v) ^ key) * n_parts) >> 32 for v in ids], dtype=np.int64)
    assert np.array_equal(origin, np.argsort(owner, kind="stable").astype(np.int32))
    assert np.array_equal(out, ids[origin])
    sizes = np.diff(offsets)
    assert sizes.sum() == len(ids) and np.all(np.abs(sizes - len(ids) / n_parts) < 6 * np.sqrt(len(ids) / n_parts))
    with pytest.raises(R.OracleError):
        R.bucket_by_owner(np.array([nv], dtype=np.int32), nv, n_parts, 0)
    empty = R.bucket_by_owner(np.zeros(0, dtype=np.int32), nv, n_parts, 0)
    assert len(empty[0]) == 0 and np.array_equal(empty[2], np.zeros(n_parts + 1, dtype=np.int64))
