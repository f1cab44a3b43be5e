"""Pins of the CPU oracle to things other than itself: published known-answer
vectors, closed forms in big-integer arithmetic, exhaustive enumeration,
library routines and the invariants the method must satisfy."""
import itertools
import math
import os
from collections import Counter

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
M64 = (1 << 64) - 1


# ---------------------------------------------------------------- Philox
def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(oracle):
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == want


def test_philox_is_a_bijection_of_the_counter_sample(oracle):
    # distinct counters under one key give distinct blocks (Philox is a keyed bijection)
    seen = set()
    for c0 in range(64):
        for c1 in range(4):
            seen.add(tuple(int(x) for x in oracle.philox4x32_10([c0, c1, 0, 7], [5, 9])))
    assert len(seen) == 256


def test_draw_layout(oracle):
    # draw 2m and 2m+1 are the low and high halves of block m of counter (node, m, hop, tag)
    seed = 0x0123456789ABCDEF
    for node, hop, m in [(0, 0, 0), (17, 1, 3), (2 ** 31 - 1, 2, 11)]:
        blk = oracle.philox4x32_10([node, m, hop, 0x48454C49], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.draw(seed, node, hop, 2 * m) == int(blk[0]) | (int(blk[1]) << 32)
        assert oracle.draw(seed, node, hop, 2 * m + 1) == int(blk[2]) | (int(blk[3]) << 32)


def test_draws_look_uniform(oracle):
    # mean of 20000 bounded draws over [0, 1000) is near 499.5 (sigma of the mean ~ 2.04)
    vals = [oracle.bounded(oracle.draw(99, v, 0, 0), 1000) for v in range(20000)]
    assert abs(np.mean(vals) - 499.5) < 10
    cnt = np.bincount(vals, minlength=1000)
    chi2 = float(((cnt - 20.0) ** 2 / 20.0).sum())
    assert chi2 < 1000 + 6 * math.sqrt(2 * 999)


# ---------------------------------------------------------------- bounded
def test_bounded_closed_form(oracle):
    rng = np.random.default_rng(1)
    xs = [0, 1, M64, M64 - 1, 1 << 63, (1 << 63) - 1] + [int(x) for x in rng.integers(0, 1 << 63, 200)] \
        + [int(x) | (1 << 63) for x in rng.integers(0, 1 << 63, 200)]
    ns = [1, 2, 3, 5, 10, 25, 26, 1000, 40001, (1 << 31) - 1, 1 << 31, (1 << 40) + 7]
    for x in xs:
        for n in ns:
            got = oracle.bounded(x, n)
            assert got == (x * n) >> 64
            assert 0 <= got < n


# ---------------------------------------------------------------- Floyd
def _draw_for(t, n):
    """Smallest 64-bit x with floor(x * n / 2^64) == t."""
    x = -((-t << 64) // n)
    assert (x * n) >> 64 == t
    return x


@pytest.mark.parametrize("d,f", [(2, 1), (3, 2), (4, 2), (5, 2), (5, 3), (6, 3), (6, 5), (7, 4)])
def test_floyd_exhaustive_uniform(oracle, d, f):
    # Feed every tuple (t_0 .. t_{f-1}), t_k in [0, d-f+k].  All tuples are equally likely
    # under uniform draws; a correct sampler maps exactly f! of them to each f-subset.
    ranges = [range(d - f + k + 1) for k in range(f)]
    hits = Counter()
    for ts in itertools.product(*ranges):
        draws = [_draw_for(t, d - f + k + 1) for k, t in enumerate(ts)]
        s = [int(v) for v in oracle.floyd_positions(d, f, draws)]
        assert len(set(s)) == f and all(0 <= v < d for v in s)
        hits[frozenset(s)] += 1
    assert len(hits) == math.comb(d, f)
    assert set(hits.values()) == {math.factorial(f)}


def test_floyd_step_rule(oracle):
    # d = 10, f = 3: steps look at j = 7, 8, 9.  t = (3, 3, 9): second 3 collides -> 8.
    draws = [_draw_for(3, 8), _draw_for(3, 9), _draw_for(9, 10)]
    assert [int(v) for v in oracle.floyd_positions(10, 3, draws)] == [3, 8, 9]
    # a pick equal to an earlier *replacement* also collides: t = (7, 0, 7) with j0 = 7
    draws = [_draw_for(7, 8), _draw_for(0, 9), _draw_for(7, 10)]
    assert [int(v) for v in oracle.floyd_positions(10, 3, draws)] == [7, 0, 9]


def test_floyd_chi_square_over_seeds(oracle):
    # node 0 with degree 6, fanout 3: 20 subsets, 40000 rng seeds
    offsets = np.array([0, 6], np.int64)
    indices = np.arange(100, 106, dtype=np.int32)
    hits = Counter()
    n = 40000
    for s in range(n):
        out = oracle.sample_node(offsets, indices, 0, 0, 3, s * 0x9E3779B97F4A7C15 & M64)
        hits[frozenset(int(x) for x in out)] += 1
    assert len(hits) == 20
    exp = n / 20
    chi2 = sum((c - exp) ** 2 / exp for c in hits.values())
    assert chi2 < 19 + 6 * math.sqrt(2 * 19)       # mean 19, sd ~6.2


def test_omitted_position_uniform_when_d_is_f_plus_1(oracle):
    offsets = np.array([0, 5], np.int64)
    indices = np.arange(5, dtype=np.int32)
    miss = Counter()
    n = 20000
    for s in range(n):
        out = oracle.sample_node(offsets, indices, 0, 1, 4, s + 1)
        miss[(set(range(5)) - set(int(x) for x in out)).pop()] += 1
    exp = n / 5
    chi2 = sum((c - exp) ** 2 / exp for c in miss.values())
    assert len(miss) == 5 and chi2 < 4 + 6 * math.sqrt(8)


# ---------------------------------------------------------------- pure-Python twin
def _py_philox(ctr, key):
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def py_sample_node(offsets, indices, v, hop, f, seed):
    base, d = int(offsets[v]), int(offsets[v + 1] - offsets[v])
    if d <= f:
        return [int(x) for x in indices[base:base + d]]
    chosen = []
    for k in range(f):
        w = _py_philox([v, k >> 1, hop, 0x48454C49], [seed & 0xFFFFFFFF, seed >> 32])
        x = (w[0] | (w[1] << 32)) if k % 2 == 0 else (w[2] | (w[3] << 32))
        j = d - f + k
        t = (x * (j + 1)) >> 64
        chosen.append(j if t in chosen else t)
    return [int(indices[base + s]) for s in chosen]


def py_pipeline(offsets, indices, seeds, fanouts, seed):
    hops = []
    frontier = [int(s) for s in seeds]
    for h, f in enumerate(fanouts):
        indptr, flat = [0], []
        for v in frontier:
            flat += py_sample_node(offsets, indices, v, h, f, seed)
            indptr.append(len(flat))
        hops.append((list(frontier), indptr, flat))
        frontier = list(dict.fromkeys(flat))
    return hops


def _random_graph(rng, n, max_deg):
    deg = rng.integers(0, max_deg + 1, n)
    deg[rng.integers(0, n, max(1, n // 8))] = 0
    offsets = np.zeros(n + 1, np.int64)
    offsets[1:] = np.cumsum(deg)
    rows = [np.sort(rng.choice(n, int(d), replace=False)).astype(np.int32) for d in deg]
    indices = np.concatenate(rows) if rows else np.zeros(0, np.int32)
    return offsets, indices.astype(np.int32)


@pytest.mark.parametrize("gseed", [1, 2, 3])
def test_sampler_equals_python_twin_and_invariants(oracle, gseed):
    rng = np.random.default_rng(gseed)
    n = 60
    offsets, indices = _random_graph(rng, n, 14)
    seeds = rng.integers(0, n, 12).astype(np.int32)        # duplicates likely
    fanouts = [3, 4, 2]
    rs = 0xDEADBEEF00000000 + gseed
    got = oracle.sample(offsets, indices, seeds, fanouts, rs)
    want = py_pipeline(offsets, indices, seeds, fanouts, rs)
    assert len(got) == 3
    for h, ((fr, ip, fl), (wfr, wip, wfl)) in enumerate(zip(got, want)):
        assert fr.tolist() == wfr and ip.tolist() == wip and fl.tolist() == wfl
        f = fanouts[h]
        for i, v in enumerate(fr):
            row = indices[offsets[v]:offsets[v + 1]].tolist()
            mine = fl[ip[i]:ip[i + 1]].tolist()
            assert len(mine) == min(len(row), f)                       # I3
            assert set(mine) <= set(row)                               # I1
            assert len(set(mine)) == len(mine)                         # I2 (rows duplicate-free)
            if len(row) <= f:
                assert mine == row
        if h > 0:
            assert fr.tolist() == list(dict.fromkeys(got[h - 1][2].tolist()))
    assert got[0][0].tolist() == seeds.tolist()
    # I8: same seed -> identical, other seed -> some node with d > f differs
    again = oracle.sample(offsets, indices, seeds, fanouts, rs)
    assert all((a[2] == b[2]).all() for a, b in zip(got, again))
    other = oracle.sample(offsets, indices, seeds, fanouts, rs + 1)
    assert any(a[2].tolist() != b[2].tolist() for a, b in zip(got, other))


def test_duplicate_seeds_get_identical_rows(oracle):
    offsets = np.array([0, 9, 9, 12], np.int64)
    indices = np.arange(12, dtype=np.int32) % 3
    (fr, ip, fl), = oracle.sample(offsets, indices, [0, 2, 0, 1, 0], [4], 77)
    a = fl[ip[0]:ip[1]].tolist()
    assert fl[ip[2]:ip[3]].tolist() == a and fl[ip[4]:ip[5]].tolist() == a
    assert ip.tolist() == [0, 4, 7, 11, 11, 15]


def test_special_graphs(oracle):
    # path 0-1-2-3 (directed both ways), star, fanout equal to / one below the degree
    offsets = np.array([0, 1, 3, 5, 6], np.int64)
    indices = np.array([1, 0, 2, 1, 3, 2], np.int32)
    hops = oracle.sample(offsets, indices, [0], [2, 2], 5)
    assert hops[0][2].tolist() == [1] and hops[1][0].tolist() == [1] and hops[1][2].tolist() == [0, 2]
    star_off = np.array([0, 5, 6, 7, 8, 9, 10], np.int64)
    star_idx = np.array([1, 2, 3, 4, 5, 0, 0, 0, 0, 0], np.int32)
    (fr, ip, fl), = oracle.sample(star_off, star_idx, [0], [5], 1)       # d == f: whole row
    assert fl.tolist() == [1, 2, 3, 4, 5]
    (fr, ip, fl), = oracle.sample(star_off, star_idx, [0], [4], 1)       # d == f + 1
    assert len(set(fl.tolist())) == 4 and set(fl.tolist()) <= {1, 2, 3, 4, 5}
    (fr, ip, fl), = oracle.sample(star_off, star_idx, [0, 3], [0], 1)    # fanout 0: empty hop
    assert fl.size == 0 and ip.tolist() == [0, 0, 0]
    hops = oracle.sample(star_off, star_idx, [], [3, 3], 1)              # no seeds
    assert all(h[0].size == 0 and h[2].size == 0 for h in hops)
    with pytest.raises(ValueError):
        oracle.sample(star_off, star_idx, [6], [1], 1)
    with pytest.raises(ValueError):
        oracle.sample(star_off, star_idx, [-1], [1], 1)


# ---------------------------------------------------------------- dedup
def test_dedup_against_library_routines(oracle):
    rng = np.random.default_rng(3)
    for n_ids, hi in [(0, 10), (1, 10), (50, 7), (5000, 300), (20000, 100000)]:
        ids = rng.integers(0, hi, n_ids).astype(np.int32)
        uniq, inv = oracle.dedup(hi, ids)
        assert uniq.tolist() == list(dict.fromkeys(ids.tolist()))
        vals, first = np.unique(ids, return_index=True)
        assert uniq.tolist() == vals[np.argsort(first)].tolist()
        assert len(uniq) == len(set(ids.tolist()))
        if n_ids:
            assert (uniq[inv] == ids).all()                            # I5
    with pytest.raises(ValueError):
        oracle.dedup(5, np.array([1, 5], np.int32))
    # the scratch is left clean: a second call sees no leftovers
    assert oracle.dedup(10, np.array([3, 3, 4], np.int32))[0].tolist() == [3, 4]
    assert oracle.dedup(10, np.array([4, 3], np.int32))[0].tolist() == [4, 3]


# ---------------------------------------------------------------- cache map, gather, miss list
def test_rank_is_the_inverse_permutation(oracle):
    rng = np.random.default_rng(4)
    order = rng.permutation(1000).astype(np.int32)
    rank = oracle.rank_build(order)
    assert (order[rank] == np.arange(1000)).all() and (rank[order] == np.arange(1000)).all()
    assert (rank == np.argsort(order)).all()
    with pytest.raises(ValueError):
        oracle.rank_build(np.array([0, 1, 1], np.int32))
    with pytest.raises(ValueError):
        oracle.rank_build(np.array([0, 3, 1], np.int32))


@pytest.mark.parametrize("n_hbm,n_host", [(0, 0), (100, 200), (1000, 0), (0, 1000), (300, 700), (1, 1)])
def test_gather_and_miss_list_against_indexing(oracle, n_hbm, n_host):
    rng = np.random.default_rng(5)
    n, row_bytes = 1000, 48
    feats = rng.integers(0, 256, (n, row_bytes), dtype=np.uint8)
    order = rng.permutation(n).astype(np.int32)
    rank = oracle.rank_build(order)
    by_rank = feats[order]
    hbm, host, standin = (np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
                          np.ascontiguousarray(by_rank[n_hbm + n_host:]))
    ids = rng.integers(0, n, 700).astype(np.int32)
    tier, slot = oracle.lookup(ids, rank, n_hbm, n_host)
    r = rank[ids].astype(np.int64)
    want_tier = np.where(r < n_hbm, 0, np.where(r < n_hbm + n_host, 1, 2))
    assert (tier == want_tier).all()
    assert (slot == r - np.choose(want_tier, [0, n_hbm, n_hbm + n_host])).all()
    out = np.full((700, row_bytes), 0xA5, np.uint8)
    mp, mi, ms, stats = oracle.gather(ids, rank, n_hbm, n_host, hbm, host, out)
    hit = want_tier < 2
    assert (out[hit] == feats[ids[hit]]).all()                          # hit rows are features[id]
    assert (out[~hit] == 0xA5).all()                                    # miss rows untouched
    assert mp.tolist() == np.nonzero(~hit)[0].tolist()                  # ascending positions
    assert (mi == ids[~hit]).all() and (ms == slot[~hit]).all()
    assert stats.tolist() == [700, int((want_tier == 0).sum()), int((want_tier == 1).sum()), int((~hit).sum())]
    oracle.gather_miss(mp, ms, standin, out)
    assert (out == feats[ids]).all()                                    # I6


# ---------------------------------------------------------------- hotness, local ids
def test_hotness_against_library_routines(oracle):
    rng = np.random.default_rng(8)
    n = 500
    counts = np.zeros(n, np.int32)
    want = np.zeros(n, np.int64)
    for _ in range(40):
        uniq = rng.choice(n, rng.integers(0, 120), replace=False).astype(np.int32)
        oracle.hotness_add(uniq, counts)
        want += np.bincount(uniq, minlength=n)
    assert (counts == want).all()
    order = oracle.hotness_order(counts)
    assert order.tolist() == sorted(range(n), key=lambda v: (-int(counts[v]), v))
    assert order.tolist() == np.lexsort((np.arange(n), -counts.astype(np.int64))).tolist()
    assert oracle.hotness_order(np.zeros(7, np.int32)).tolist() == list(range(7))


def test_local_ids_against_dictionary(oracle):
    rng = np.random.default_rng(9)
    ids = rng.integers(0, 300, 2000).astype(np.int32)
    uniq, inv = oracle.dedup(300, ids)
    where = {int(v): i for i, v in enumerate(uniq)}
    probe = rng.choice(uniq, 777).astype(np.int32)
    assert oracle.local_ids(300, uniq, probe).tolist() == [where[int(v)] for v in probe]
    assert (oracle.local_ids(300, uniq, ids) == inv).all()             # the inverse map is the special case ids = input
    missing = np.setdiff1d(np.arange(300), uniq)
    if missing.size:
        with pytest.raises(ValueError):
            oracle.local_ids(300, uniq, missing[:1].astype(np.int32))
