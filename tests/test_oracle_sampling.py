"""Pins for the integer half of the CPU oracle: random source, row sampler, CSR, sampled
blocks, hot-vertex selection. Every check is against something other than the oracle itself:
published known-answer vectors, exhaustive enumeration, library routines, or set arithmetic
on the raw edge list."""
import itertools
import os

import numpy as np
import pytest
import scipy.sparse as sp

import synth_inputs as si
from oracle import oracle as ora

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ random source

def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        vals = [int(x, 16) for x in r if x != "->"]
        assert ora.philox4x32_10(vals[0:4], vals[4:6]) == tuple(vals[6:10])


def test_random64_layout():
    # counter = (v_lo, v_hi, slot, domain<<8|hop), key = (stream_lo, stream_hi); x = out1:out0
    stream, domain, hop, v, slot = 0x0123456789ABCDEF, 1, 2, 0x1_0000_0007, 5
    o = ora.philox4x32_10([v & 0xFFFFFFFF, v >> 32, slot, (domain << 8) | hop],
                          [stream & 0xFFFFFFFF, stream >> 32])
    assert ora.random64(stream, domain, hop, v, slot) == (o[1] << 32) | o[0]


def test_mulhi64_is_floor_of_product():
    rng = np.random.default_rng(0)
    for _ in range(200):
        x = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        n = int(rng.integers(1, 1 << 40))
        assert int(ora.lib().ora_mulhi64(x, n)) == (x * n) >> 64
    assert int(ora.lib().ora_mulhi64((1 << 64) - 1, 7)) == 6
    assert int(ora.lib().ora_mulhi64(0, 7)) == 0


# ------------------------------------------------------------------ Fisher-Yates prefix

def _dense_fisher_yates(d, k, r):
    a = list(range(d))
    for j in range(k):
        a[j], a[r[j]] = a[r[j]], a[j]
    return a[:k]


@pytest.mark.parametrize("d", [1, 2, 3, 4, 5, 6])
def test_fisher_yates_exhaustive(d):
    """Every reachable swap sequence: the sparse-map result equals the dense textbook shuffle,
    and every ordered k-arrangement is produced by exactly one sequence (uniformity)."""
    for k in range(1, d + 1):
        seen = {}
        for r in itertools.product(*[range(j, d) for j in range(k)]):
            got = ora.fisher_yates_prefix(d, k, r)
            assert got == _dense_fisher_yates(d, k, r)
            assert len(set(got)) == k and all(0 <= x < d for x in got)
            seen[tuple(got)] = seen.get(tuple(got), 0) + 1
        n_arr = 1
        for j in range(k):
            n_arr *= d - j
        assert len(seen) == n_arr and set(seen.values()) == {1}


def test_fisher_yates_random_long_chains():
    rng = np.random.default_rng(1)
    for _ in range(300):
        d = int(rng.integers(2, 40))
        k = int(rng.integers(1, d + 1))
        r = [int(rng.integers(j, d)) for j in range(k)]
        assert ora.fisher_yates_prefix(d, k, r) == _dense_fisher_yates(d, k, r)


# ------------------------------------------------------------------ row sampler

def test_sample_row_invariants():
    for d, k in [(0, 5), (1, 5), (5, 5), (6, 5), (7, 1), (1000, 25), (26, 25), (2 ** 33 + 5, 10)]:
        out = ora.sample_row(7, 0, 1, 123, d, k)
        assert len(out) == min(d, k)
        assert len(set(out)) == len(out)
        assert all(0 <= p < d for p in out)
        if d <= k:
            assert out == list(range(d))
        assert out == ora.sample_row(7, 0, 1, 123, d, k)          # equal keys, equal sample
    a = ora.sample_row(7, 0, 1, 123, 10 ** 6, 25)
    assert a != ora.sample_row(8, 0, 1, 123, 10 ** 6, 25)         # stream
    assert a != ora.sample_row(7, 1, 1, 123, 10 ** 6, 25)         # domain
    assert a != ora.sample_row(7, 0, 2, 123, 10 ** 6, 25)         # hop
    assert a != ora.sample_row(7, 0, 1, 124, 10 ** 6, 25)         # vertex


def test_sample_row_first_slot_matches_definition():
    # slot 0 with an untouched array: position = floor(x * d / 2^64)
    for v in range(20):
        d = 1000 + v
        x = ora.random64(3, 0, 0, v, 0)
        assert ora.sample_row(3, 0, 0, v, d, 4)[0] == (x * d) >> 64


def test_sample_row_uniform_inclusion():
    d, k, n = 20, 5, 40000
    cnt = np.zeros(d)
    first = np.zeros(d)
    for s in range(n):
        out = ora.sample_row(s, 0, 0, 77, d, k)
        cnt[out] += 1
        first[out[0]] += 1
    exp = n * k / d
    chi2 = ((cnt - exp) ** 2 / exp).sum()
    assert chi2 < 60.0            # 19 dof; P(chi2 > 60) ~ 4e-6
    exp1 = n / d
    assert ((first - exp1) ** 2 / exp1).sum() < 60.0


# ------------------------------------------------------------------ CSR

def test_csr_matches_library_sort():
    src, dst = si.rmat_edges(300, 4000, seed=3)
    g = ora.build_csr(src, dst, 300)
    order = np.lexsort((src, dst))
    assert np.array_equal(g.col, src[order])
    assert np.array_equal(g.rowptr, np.concatenate([[0], np.cumsum(np.bincount(dst, minlength=300))]))
    m = sp.csr_matrix((np.ones(len(src)), (dst, src)), shape=(300, 300))   # sums duplicates
    for v in range(300):
        row = g.col[g.rowptr[v]:g.rowptr[v + 1]]
        assert np.array_equal(np.unique(row), m[v].indices[np.argsort(m[v].indices)])
        assert len(row) == int(m[v].data.sum())


def test_csr_empty_rows_and_self_loops():
    src = np.array([2, 2, 0, 3, 3], dtype=np.int32)
    dst = np.array([2, 0, 0, 0, 0], dtype=np.int32)
    g = ora.build_csr(src, dst, 5)
    assert g.rowptr.tolist() == [0, 4, 4, 5, 5, 5]
    assert g.col.tolist() == [0, 2, 3, 3, 2]


# ------------------------------------------------------------------ sampled hop

def _in_neighbours(src, dst, v):
    return sorted(src[dst == v].tolist())


def test_hop_full_fanout_is_exact_neighbourhood():
    V = 120
    src, dst = si.random_graph_small(V, 700, seed=5)
    g = ora.build_csr(src, dst, V)
    kmax = int(np.diff(g.rowptr).max())
    seeds = np.array([5, 17, 3, 99, 64], dtype=np.int32)
    sb = ora.sample_blocks(g, seeds, [kmax, kmax + 3], seed=1, step=0)
    frontier = seeds.tolist()
    for blk in sb.blocks:
        assert blk.dst_global.tolist() == frontier
        expect_src = list(frontier)
        for i, v in enumerate(frontier):
            nb = _in_neighbours(src, dst, v)
            got = blk.nbr_global[blk.indptr[i]:blk.indptr[i + 1]].tolist()
            assert got == nb                                   # whole row, CSR order
            for u in nb:
                if u not in expect_src:
                    expect_src.append(u)                       # first-occurrence order
        assert blk.src_global.tolist() == expect_src
        assert np.array_equal(blk.src_global[blk.indices], blk.nbr_global)
        frontier = expect_src
    # two hops with full fanout reach exactly the 2-hop in-neighbourhood (BFS on the edge list)
    reach = set(seeds.tolist())
    level = set(seeds.tolist())
    for _ in range(2):
        level = {int(u) for v in level for u in src[dst == v]}
        reach |= level
    assert set(sb.blocks[-1].src_global.tolist()) == reach


def test_hop_sampled_invariants_and_csc():
    w = si.WORKLOADS["tiny"]
    src, dst = si.rmat_edges(w.n_vertices, w.n_edges, 0)
    g = ora.build_csr(src, dst, w.n_vertices)
    seeds = si.batch_seeds(si.train_split(w.n_vertices), w.batch, 0)
    sb = ora.sample_blocks(g, seeds, w.fanouts, seed=0, step=3)
    deg = np.diff(g.rowptr)
    frontier = seeds
    for h, blk in enumerate(sb.blocks):
        k = w.fanouts[h]
        assert np.array_equal(blk.dst_global, frontier)
        assert np.array_equal(np.diff(blk.indptr), np.minimum(deg[frontier], k))
        assert np.array_equal(blk.src_global[: blk.n_dst], frontier)
        assert len(np.unique(blk.src_global)) == blk.n_src
        assert np.array_equal(blk.src_global[blk.indices], blk.nbr_global)
        # every sampled neighbour is a real in-neighbour; positions in a row are distinct
        for i in range(0, blk.n_dst, 37):
            v = frontier[i]
            row = g.col[g.rowptr[v]:g.rowptr[v + 1]]
            pos = ora.sample_row(0 + 3, 0, h, int(v), len(row), k)
            assert blk.nbr_global[blk.indptr[i]:blk.indptr[i + 1]].tolist() == row[pos].tolist()
        # new ids appear in first-occurrence order
        new = blk.indices[blk.indices >= blk.n_dst]
        _, first = np.unique(new, return_index=True)
        assert np.array_equal(new[np.sort(first)], np.arange(blk.n_dst, blk.n_src))
        # CSC = transpose with edge ids ascending inside each column (scipy as the library)
        a = sp.csr_matrix((np.arange(1, blk.nnz + 1), blk.indices, blk.indptr), shape=(blk.n_dst, blk.n_src))
        assert np.array_equal(blk.csc_indptr, np.concatenate([[0], np.cumsum(np.bincount(blk.indices, minlength=blk.n_src))]))
        order = np.lexsort((np.arange(blk.nnz), blk.indices))
        assert np.array_equal(blk.csc_eid, order)
        rows_of_edge = np.repeat(np.arange(blk.n_dst), np.diff(blk.indptr))
        assert np.array_equal(blk.csc_dst, rows_of_edge[order])
        assert a.nnz == blk.nnz
        frontier = blk.src_global


def test_frontier_deduplication_shape():
    """Fig. 7's example (10000 -> 28706 -> 86175 at fanout 4) shows frontiers are sets: far
    fewer than the 1 + fanout growth. Same order of magnitude on a skewed synthetic graph."""
    src, dst = si.rmat_edges(50_000, 2_000_000, seed=2)
    g = ora.build_csr(src, dst, 50_000)
    seeds = si.train_split(50_000, 0.65, 2)[:2000]
    sb = ora.sample_blocks(g, seeds, [4, 4], seed=0, step=0)
    n1, n2 = sb.blocks[0].n_src, sb.blocks[1].n_src
    assert 2000 < n1 < 2000 * 5 and n1 < n2 < n1 * 5
    assert n2 < 2000 * 25 * 0.9       # de-duplication visibly shrinks the no-dedup bound


# ------------------------------------------------------------------ hot selection and lookup

def test_select_hot_bruteforce_recount():
    V = 400
    src, dst = si.rmat_edges(V, 6000, seed=7)
    g = ora.build_csr(src, dst, V)
    train = si.train_split(V, 0.5, 7)
    fan, B, P, seed = (4, 3, 2), 32, 2, 11
    cache = ora.select_hot(g, train, B, fan, P, 0.1, 2, 8, seed)
    freq = np.zeros(V, dtype=np.int64)
    nb = -(-len(train) // B)
    for p in range(P):
        for b in range(nb):
            batch = train[b * B:(b + 1) * B]
            # hops 0..L-2 only, pre-sampling domain, one stream per (epoch, batch)
            sb = ora.sample_blocks(g, batch, fan[:-1], seed=seed + p * nb + b, step=0, domain=ora.DOMAIN_PRESAMPLE)
            v1 = sb.blocks[-1].src_global
            assert len(np.unique(v1)) == len(v1)
            freq[v1] += 1
    assert np.array_equal(freq, cache.freq)
    n_hot = V // 10
    expect = sorted(range(V), key=lambda v: (-freq[v], v))[:n_hot]
    assert cache.hot_ids.tolist() == expect
    assert np.array_equal(cache.slot_of_vertex[cache.hot_ids], np.arange(n_hot))
    assert (cache.slot_of_vertex >= 0).sum() == n_hot
    assert (cache.version == -1).all() and not cache.emb.any()


def test_select_hot_ties_by_id():
    V = 50
    g = ora.build_csr(np.zeros(0, np.int32), np.zeros(0, np.int32), V)    # no edges: V^1 = seeds
    train = np.arange(V, dtype=np.int32)[::-1].copy()
    cache = ora.select_hot(g, train, 8, (3, 3), 2, 0.2, 1, 4, 0)
    assert cache.hot_ids.tolist() == list(range(10))


def test_cache_lookup_predicate():
    slot = np.full(10, -1, np.int32)
    slot[[2, 4, 6, 8]] = [0, 1, 2, 3]
    c = ora.Cache(np.array([2, 4, 6, 8], np.int32), slot, np.array([-1, 5, 3, 6], np.int32), np.zeros((4, 2)), 2)
    v1 = np.array([8, 1, 2, 4, 6, 9], np.int32)
    comp, hit, hslot = ora.cache_lookup(c, v1, step=6)
    # vertex 8: version 6, age 0 -> hit; 2: empty; 4: age 1 -> hit; 6: age 3 > S -> stale
    assert hit.tolist() == [0, 3] and hslot.tolist() == [3, 1] and comp.tolist() == [1, 2, 4, 5]
    c.staleness = 0
    comp, hit, _ = ora.cache_lookup(c, v1, step=7)
    assert hit.tolist() == [] and comp.tolist() == list(range(6))


def test_bottom_hop_skips_reusable_hot_vertices():
    w = si.WORKLOADS["tiny"]
    src, dst = si.rmat_edges(w.n_vertices, w.n_edges, 0)
    g = ora.build_csr(src, dst, w.n_vertices)
    train = si.train_split(w.n_vertices)
    cache = ora.select_hot(g, train, w.batch, w.fanouts, 1, 0.05, 3, 4, 0)
    cache.version[:] = 0
    seeds = si.batch_seeds(train, w.batch, 1)
    plain = ora.sample_blocks(g, seeds, w.fanouts, 0, 1, None)
    sb = ora.sample_blocks(g, seeds, w.fanouts, 0, 1, cache)
    v1 = plain.blocks[0].src_global
    assert np.array_equal(sb.blocks[0].src_global, v1)
    hot = cache.slot_of_vertex[v1] >= 0
    assert hot.any() and np.array_equal(np.nonzero(hot)[0], sb.hit_pos)
    assert np.array_equal(sb.blocks[1].dst_global, v1[~hot])
    assert len(sb.hit_pos) + len(sb.compute_pos) == len(v1)
    # rows of computed vertices are the same samples as without a cache (pure function of the key)
    pos_in_plain = np.nonzero(~hot)[0]
    for i in range(0, len(pos_in_plain), 50):
        j = pos_in_plain[i]
        a = plain.blocks[1].nbr_global[plain.blocks[1].indptr[j]:plain.blocks[1].indptr[j + 1]]
        b = sb.blocks[1].nbr_global[sb.blocks[1].indptr[i]:sb.blocks[1].indptr[i + 1]]
        assert np.array_equal(a, b)


def test_csr_symmetrise_and_dedup_against_set_arithmetic():
    """The two optional preparations of the edge list: both directions of every edge, and one copy of equal edges."""
    V = 40
    src, dst = si.random_graph_small(V, 400, seed=7)
    assert len({(int(a), int(b)) for a, b in zip(src, dst)}) < 400          # the input has multi-edges
    g = ora.build_csr(src, dst, V, symmetrise=True, dedup=True)
    want = {(int(a), int(b)) for a, b in zip(src, dst)} | {(int(b), int(a)) for a, b in zip(src, dst)}
    got = [(int(g.col[e]), v) for v in range(V) for e in range(g.rowptr[v], g.rowptr[v + 1])]
    assert len(got) == len(want) == g.n_edges and set(got) == want
    for v in range(V):
        row = g.col[g.rowptr[v]:g.rowptr[v + 1]]
        assert (np.diff(row) > 0).all()
    g2 = ora.build_csr(src, dst, V, symmetrise=True)
    assert g2.n_edges == 800
    for v in range(V):
        assert sorted(g2.col[g2.rowptr[v]:g2.rowptr[v + 1]].tolist()) == sorted(
            [int(a) for a, b in zip(src, dst) if b == v] + [int(b) for a, b in zip(src, dst) if a == v])
    g3 = ora.build_csr(src, dst, V, dedup=True)
    assert g3.n_edges == len({(int(a), int(b)) for a, b in zip(src, dst)})
