"""GPU parity: every output of the HIP path, called through the C ABI, equals the CPU oracle's
bit for bit (the path is integer indexing and byte copies; the tolerance is zero)."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, assert_same, gpu_path, oracle_path, to_bytes, SENTINEL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def helios():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2310_00837_amd import helios as hl
    return hl


@pytest.fixture()
def h(helios):
    ctx = helios.Helios(0)
    yield ctx
    ctx.close()


def _random_graph(rng, n, max_deg, hub_deg=0):
    deg = rng.integers(0, max_deg + 1, n)
    deg[rng.integers(0, n, max(1, n // 8))] = 0
    if hub_deg:
        deg[rng.integers(0, n, 3)] = hub_deg
    offsets = np.zeros(n + 1, np.int64)
    offsets[1:] = np.cumsum(deg)
    rows = [np.sort(rng.choice(n, int(d), replace=False)).astype(np.int32) for d in deg]
    return offsets, np.concatenate(rows).astype(np.int32)


# ------------------------------------------------------------------ sampling
@pytest.mark.parametrize("fanouts", [[3], [5, 5], [8, 9], [16, 17, 2], [25, 10], [33], [64, 2], [65], [200, 3], [0, 4], [4, 0]])
def test_sample_parity_random_graph(h, helios, oracle, fanouts):
    print("fanouts", fanouts, flush=True)
    rng = np.random.default_rng(sum(fanouts) + len(fanouts))
    n = 3000
    off, idx = _random_graph(rng, n, 40, hub_deg=700)
    h.csr_load(torch.from_numpy(off).cuda(), torch.from_numpy(idx).cuda())
    seeds = rng.integers(0, n, 700).astype(np.int32)            # duplicates, several tiles, ragged tail
    for rs in (1, 0xFFFFFFFFFFFFFFFF, 0x123456789ABCDEF0):
        hops = helios.alloc_hops(seeds.size, fanouts, h.device)
        sizes = torch.zeros(2 * len(fanouts), dtype=torch.int64).pin_memory()
        h.sample(torch.from_numpy(seeds).cuda(), fanouts, rs, hops, sizes)
        h.sync()
        want = oracle.sample(off, idx, seeds, fanouts, rs)
        for k, (fr, ip, fl) in enumerate(want):
            assert int(sizes[2 * k]) == fr.size and int(sizes[2 * k + 1]) == fl.size
            assert np.array_equal(hops[k].frontier[:fr.size].cpu().numpy(), fr)
            assert np.array_equal(hops[k].indptr[:fr.size + 1].cpu().numpy(), ip)
            assert np.array_equal(hops[k].flat[:fl.size].cpu().numpy(), fl)


def test_sample_edge_cases(h, helios, oracle):
    # star + isolated nodes; degree == fanout, degree == fanout + 1, empty seed list
    off = np.array([0, 5, 6, 7, 8, 9, 10, 10, 16], np.int64)
    idx = np.array([1, 2, 3, 4, 5, 0, 0, 0, 0, 0, 0, 1, 2, 3, 4, 5], np.int32)
    h.csr_load(torch.from_numpy(off).cuda(), torch.from_numpy(idx).cuda())
    for seeds, fanouts in [([0], [5]), ([0], [4]), ([7, 7, 0, 6], [5, 5]), ([6], [3, 3]), ([], [3, 2]), ([7], [6]), ([7], [1, 1, 1])]:
        print("edge", seeds, fanouts, flush=True)
        s = np.array(seeds, np.int32)
        hops = helios.alloc_hops(s.size, fanouts, h.device)
        sizes = torch.full((2 * len(fanouts),), -7, dtype=torch.int64).pin_memory()
        h.sample(torch.from_numpy(s).cuda(), fanouts, 42, hops, sizes)
        h.sync()
        want = oracle.sample(off, idx, s, fanouts, 42)
        for k, (fr, ip, fl) in enumerate(want):
            assert [int(sizes[2 * k]), int(sizes[2 * k + 1])] == [fr.size, fl.size]
            assert np.array_equal(hops[k].frontier[:fr.size].cpu().numpy(), fr)
            assert np.array_equal(hops[k].indptr[:fr.size + 1].cpu().numpy(), ip)
            assert np.array_equal(hops[k].flat[:fl.size].cpu().numpy(), fl)


# ------------------------------------------------------------------ dedup
@pytest.mark.parametrize("n_ids,hi", [(0, 10), (1, 10), (255, 40), (256, 1000), (257, 50), (5000, 300), (100_000, 20_000),
                                      (300_000, 2_000_000), (70_000, 3)])
def test_dedup_parity(h, oracle, n_ids, hi):
    print("dedup", n_ids, hi, flush=True)
    rng = np.random.default_rng(n_ids + hi)
    n_nodes = max(hi, 1)
    off = torch.zeros(n_nodes + 1, dtype=torch.int64, device="cuda")
    h.csr_load(off, torch.zeros(1, dtype=torch.int32, device="cuda"))
    ids = rng.integers(0, hi, n_ids).astype(np.int32)
    # a power-law mix: many repeats of a few hot IDs, as sampled hubs are
    if n_ids > 1000:
        hot = rng.integers(0, hi, 5).astype(np.int32)
        where = rng.random(n_ids) < 0.3
        ids[where] = hot[rng.integers(0, 5, int(where.sum()))]
    t = torch.from_numpy(ids).cuda()
    uniq = torch.full((max(n_ids, 1),), -9, dtype=torch.int32, device="cuda")
    inv = torch.full((max(n_ids, 1),), -9, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -9, dtype=torch.int64).pin_memory()
    for _ in range(2):                                        # the table is reused by the second call
        h.dedup(t, uniq, inv, nu, n_ids=n_ids)
        h.sync()
        wu, wi = oracle.dedup(n_nodes, ids)
        assert int(nu[0]) == wu.size
        assert np.array_equal(uniq[:wu.size].cpu().numpy(), wu)
        assert np.array_equal(inv[:n_ids].cpu().numpy(), wi)
    h.dedup(t, uniq, None, nu, n_ids=n_ids)                    # inverse is optional
    h.sync()
    assert int(nu[0]) == wu.size


# ------------------------------------------------------------------ lookup + gather + miss list
@pytest.mark.parametrize("row_bytes", [16, 48, 256, 512, 1024, 2048, 4096, 4112])
@pytest.mark.parametrize("tiers", [(0.1, 0.2), (0.0, 0.5), (1.0, 0.0), (0.0, 0.0), (0.0, 1.0)])
def test_gather_parity(h, oracle, row_bytes, tiers):
    print("gather", row_bytes, tiers, flush=True)
    rng = np.random.default_rng(row_bytes)
    n = 5000
    n_hbm, n_host = int(tiers[0] * n), int(tiers[1] * n)
    feats = torch.from_numpy(rng.integers(0, 256, (n, row_bytes), dtype=np.uint8))
    order = torch.from_numpy(rng.permutation(n).astype(np.int32))
    h.csr_load(torch.zeros(n + 1, dtype=torch.int64, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"))
    cache = GpuCache(h, feats, order, n_hbm, n_host)
    by_rank = feats.numpy()[order.numpy()]
    assert np.array_equal(cache.hbm[:n_hbm].cpu().numpy(), by_rank[:n_hbm])
    assert np.array_equal(cache.host[:n_host].numpy(), by_rank[n_hbm:n_hbm + n_host])
    assert np.array_equal(cache.standin[:cache.n_rest].numpy(), by_rank[n_hbm + n_host:])
    rank = oracle.rank_build(order.numpy())
    for n_ids in (0, 1, 777, 4100):
        ids = rng.integers(0, n, n_ids).astype(np.int32)         # duplicates allowed
        out = torch.full((max(n_ids, 1), row_bytes), SENTINEL, dtype=torch.uint8, device="cuda")
        mp = torch.full((max(n_ids, 1),), -9, dtype=torch.int32, device="cuda")
        mi, ms = mp.clone(), mp.clone()
        stats = torch.full((4,), -9, dtype=torch.int64).pin_memory()
        h.gather(torch.from_numpy(ids).cuda(), out, mp, mi, ms, stats, n_ids=n_ids)
        h.sync()
        wout = np.full((n_ids, row_bytes), SENTINEL, np.uint8)
        wmp, wmi, wms, wstats = oracle.gather(ids, rank, n_hbm, n_host, np.ascontiguousarray(by_rank[:n_hbm]),
                                              np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]), wout)
        assert stats.tolist() == wstats.tolist()
        nm = int(wstats[3])
        assert np.array_equal(mp[:nm].cpu().numpy(), wmp) and np.array_equal(mi[:nm].cpu().numpy(), wmi)
        assert np.array_equal(ms[:nm].cpu().numpy(), wms)
        assert np.array_equal(out[:n_ids].cpu().numpy(), wout)         # hit rows copied, miss rows untouched
        h.gather_miss(mp, ms, nm, None, out)
        h.sync()
        assert np.array_equal(out[:n_ids].cpu().numpy(), feats.numpy()[ids])


# ------------------------------------------------------------------ whole path on the small workloads
@pytest.fixture(scope="module")
def workloads():
    made = {}

    def get(cfg):
        if cfg not in made:
            sp = W.spec(cfg)
            g = W.make_graph(sp, 1234, "cpu")
            feats = W.feature_rows(1234, torch.arange(g.n_nodes), sp.dim, sp.dtype)
            made[cfg] = (sp, g, feats)
        return made[cfg]
    return get


@pytest.mark.parametrize("cfg", [0, 1])
def test_whole_path_parity(h, helios, oracle, workloads, cfg):
    sp, g, feats = workloads(cfg)
    print("workload", sp.name, "N", g.n_nodes, "E", g.n_edges, flush=True)
    n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)
    off, idx, order = g.offsets.numpy(), g.indices.numpy(), g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    for b in range(3):
        seeds = W.seed_batch(sp, g, b)
        rs = W.batch_rng_seed(1234, b)
        want = oracle_path(oracle, off, idx, seeds.numpy(), sp.fanouts, rs, rank, n_hbm, n_host, *tabs, sp.row_bytes)
        fused = gpu_path(h, helios, seeds, sp.fanouts, rs, fused=True)
        assert_same(fused, want)
        steps = gpu_path(h, helios, seeds, sp.fanouts, rs, fused=False)
        assert_same(steps, want)
        again = gpu_path(h, helios, seeds, sp.fanouts, rs, fused=True)     # run-twice determinism
        assert_same(again, fused)
        print(" batch", b, "unique", want["unique"].size, "stats", want["stats"].tolist(), flush=True)
    # Zipf seeds (duplicates in the seed list) on the same graph
    z = W.spec(4)
    z.batch = sp.batch
    seeds = W.seed_batch(z, g, 0)
    want = oracle_path(oracle, off, idx, seeds.numpy(), sp.fanouts, 99, rank, n_hbm, n_host, *tabs, sp.row_bytes)
    assert_same(gpu_path(h, helios, seeds, sp.fanouts, 99, fused=True), want)


@pytest.mark.parametrize("fanouts", [[3], [65, 3], [200], [3, 3, 3], [0, 4], [4, 0], [16, 1, 17, 2]])
def test_whole_path_random_graph(h, helios, oracle, fanouts):
    """helios_prepare_batch on a graph with empty rows and hubs, with fan-outs on both sides of every
    group width of the sampling kernel (the lanes that write a sample also feed the de-duplications)."""
    print("whole path, fanouts", fanouts, flush=True)
    rng = np.random.default_rng(100 + sum(fanouts))
    n = 4000
    off, idx = _random_graph(rng, n, 30, hub_deg=900)
    feats = torch.from_numpy(rng.integers(0, 256, (n, 48), dtype=np.uint8))
    order = torch.from_numpy(rng.permutation(n).astype(np.int32))
    n_hbm, n_host = 700, 1100
    h.csr_load(torch.from_numpy(off).cuda(), torch.from_numpy(idx).cuda())
    cache = GpuCache(h, feats, order, n_hbm, n_host)  # noqa: F841
    by_rank = feats.numpy()[order.numpy()]
    rank = oracle.rank_build(order.numpy())
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    for n_seeds in (0, 1, 300, 1500):                   # none; one tile; a ragged second tile; repeated seeds
        seeds = torch.from_numpy(rng.integers(0, n, n_seeds).astype(np.int32))
        want = oracle_path(oracle, off, idx, seeds.numpy(), fanouts, 77, rank, n_hbm, n_host, *tabs, 48)
        assert_same(gpu_path(h, helios, seeds, fanouts, 77, fused=True), want)
        assert_same(gpu_path(h, helios, seeds, fanouts, 77, fused=False), want)


# ------------------------------------------------------------------ error behaviour
def test_errors(h, helios):
    HE = helios.HeliosError
    seeds = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    hops = helios.alloc_hops(2, [2], h.device)
    sizes = torch.zeros(2, dtype=torch.int64).pin_memory()
    with pytest.raises(HE) as e:
        h.sample(seeds, [2], 1, hops, sizes)                         # no graph yet
    assert e.value.code == helios.ESTATE
    off = torch.tensor([0, 3, 3, 6], dtype=torch.int64, device="cuda")
    idx = torch.tensor([1, 2, 0, 0, 1, 2], dtype=torch.int32, device="cuda")
    h.csr_load(off, idx)
    with pytest.raises(HE) as e:
        h.gather(seeds, torch.zeros(2, 16, dtype=torch.uint8, device="cuda"), seeds, seeds, seeds,
                 torch.zeros(4, dtype=torch.int64).pin_memory())
    assert e.value.code == helios.ESTATE
    with pytest.raises(HE) as e:
        h.sample(seeds, [helios.MAX_FANOUT + 1], 1, hops, sizes)
    assert e.value.code == helios.EINVAL
    with pytest.raises(HE) as e:
        h.cache_build(torch.arange(3, dtype=torch.int32, device="cuda"), 1, 1, 24, off, None, None)   # row_bytes % 16
    assert e.value.code == helios.EINVAL
    # a seed that is not a node: reported by the next sync, and the context keeps working
    bad = torch.tensor([0, 3], dtype=torch.int32, device="cuda")
    h.sample(bad, [2], 1, hops, sizes)
    with pytest.raises(HE) as e:
        h.sync()
    assert e.value.code == helios.EDATA
    h.sample(seeds, [2], 1, hops, sizes)
    h.sync()
    assert sizes.tolist() == [2, 2]
    # sample list larger than its buffer: nothing written past it, required size reported
    small = [helios.HopBuffers(hops[0].frontier, hops[0].indptr, torch.full((3,), -5, dtype=torch.int32, device="cuda"))]
    both = torch.tensor([0, 2], dtype=torch.int32, device="cuda")
    guard = small[0].flat
    h.sample(both, [3], 1, small, sizes)
    with pytest.raises(HE) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY and sizes.tolist() == [2, 6]
    assert guard.cpu().tolist() == [1, 2, 0]
    # an order that repeats a node is not a permutation
    h.cache_build(torch.tensor([0, 1, 1], dtype=torch.int32, device="cuda"), 1, 1, 16,
                  torch.zeros(16, dtype=torch.uint8, device="cuda"), torch.zeros(16, dtype=torch.uint8).pin_memory(), None)
    with pytest.raises(HE) as e:
        h.sync()
    assert e.value.code == helios.EDATA
    # miss list too small
    h.cache_build(torch.tensor([2, 0, 1], dtype=torch.int32, device="cuda"), 1, 0, 16,
                  torch.zeros(16, dtype=torch.uint8, device="cuda"), None, None)
    h.sync()
    ids = torch.tensor([0, 1, 2, 0, 1], dtype=torch.int32, device="cuda")
    out = torch.zeros(5, 16, dtype=torch.uint8, device="cuda")
    m = torch.full((2,), -5, dtype=torch.int32, device="cuda")
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    h.gather(ids, out, m, m.clone(), m.clone(), stats)
    with pytest.raises(HE) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY and stats.tolist() == [5, 1, 0, 4]
    assert m.cpu().tolist() == [0, 1]


def test_graph_with_a_neighbour_that_is_no_node(h, helios):
    """An entry of `indices` outside [0, n): the lane that samples it reports it when it feeds the
    de-duplications (HELIOS_EDATA at the next sync); nothing is indexed with it, and the context works on."""
    off = torch.tensor([0, 2, 3, 3], dtype=torch.int64, device="cuda")
    idx = torch.tensor([1, 9, 0], dtype=torch.int32, device="cuda")
    h.csr_load(off, idx)
    seeds = torch.tensor([0], dtype=torch.int32, device="cuda")
    hops = helios.alloc_hops(1, [2, 2], h.device)
    sizes = torch.zeros(4, dtype=torch.int64).pin_memory()
    h.sample(seeds, [2, 2], 5, hops, sizes)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.EDATA
    assert sizes.tolist() == [1, 2, 1, 1]                       # frontier_1 = [1]: the bad value is no frontier node
    assert hops[1].frontier[:1].cpu().tolist() == [1] and hops[1].flat[:1].cpu().tolist() == [0]
    # whole path: same report
    h.cache_build(torch.tensor([2, 0, 1], dtype=torch.int32, device="cuda"), 1, 1, 16,
                  torch.zeros(16, dtype=torch.uint8, device="cuda"), torch.zeros(16, dtype=torch.uint8).pin_memory(),
                  torch.zeros(16, dtype=torch.uint8).pin_memory())
    h.sync()
    with pytest.raises(helios.HeliosError) as e:
        gpu_path(h, helios, seeds.cpu(), [2, 2], 5, fused=True)
    assert e.value.code == helios.EDATA
    # a sound graph afterwards
    h.csr_load(off, torch.tensor([1, 2, 0], dtype=torch.int32, device="cuda"))
    h.sample(seeds, [2, 2], 5, hops, sizes)
    h.sync()
    assert sizes.tolist() == [1, 2, 2, 1]


# ------------------------------------------------------------------ limits and capacities
def test_maximum_fanout_and_hops(h, helios, oracle):
    rng = np.random.default_rng(11)
    n = 6000
    off, idx = _random_graph(rng, n, 30, hub_deg=3000)
    h.csr_load(torch.from_numpy(off).cuda(), torch.from_numpy(idx).cuda())
    hubs = np.nonzero(np.diff(off) == 3000)[0].astype(np.int32)
    seeds = np.concatenate([hubs, rng.integers(0, n, 40).astype(np.int32)])
    for fanouts in ([helios.MAX_FANOUT], [1000, 2], [2] * helios.MAX_HOPS):
        print("limits", fanouts[:3], len(fanouts), flush=True)
        hops = helios.alloc_hops(seeds.size, fanouts, h.device)
        sizes = torch.zeros(2 * len(fanouts), dtype=torch.int64).pin_memory()
        h.sample(torch.from_numpy(seeds).cuda(), fanouts, 7, hops, sizes)
        h.sync()
        for k, (fr, ip, fl) in enumerate(oracle.sample(off, idx, seeds, fanouts, 7)):
            assert [int(sizes[2 * k]), int(sizes[2 * k + 1])] == [fr.size, fl.size]
            assert np.array_equal(hops[k].indptr[:fr.size + 1].cpu().numpy(), ip)
            assert np.array_equal(hops[k].flat[:fl.size].cpu().numpy(), fl)
    with pytest.raises(helios.HeliosError) as e:
        h.sample(torch.from_numpy(seeds).cuda(), [1] * (helios.MAX_HOPS + 1), 7,
                 helios.alloc_hops(seeds.size, [1] * (helios.MAX_HOPS + 1), h.device),
                 torch.zeros(2 * (helios.MAX_HOPS + 1), dtype=torch.int64).pin_memory())
    assert e.value.code == helios.EINVAL


def test_whole_path_capacity_errors(h, helios, workloads):
    """Outputs of helios_prepare_batch that are too small: reported by helios_sync, required sizes
    stored, nothing written past a capacity, and the context works again afterwards."""
    sp, g, feats = workloads(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    seeds = W.seed_batch(sp, g, 0).cuda()
    good = gpu_path(h, helios, seeds, sp.fanouts, 3, fused=True)
    U, n_miss = good["unique"].size, good["miss_pos"].size
    assert n_miss > 4
    dev = h.device
    hops = helios.alloc_hops(seeds.numel(), sp.fanouts, dev)
    cap = seeds.numel() + sum(hb.flat.numel() for hb in hops)
    sizes = torch.zeros(4, dtype=torch.int64).pin_memory()
    nu = torch.zeros(1, dtype=torch.int64).pin_memory()
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    inverse = torch.empty(cap, dtype=torch.int32, device=dev)
    out = torch.full((cap, sp.row_bytes), 0xA5, dtype=torch.uint8, device=dev)
    full = torch.empty(cap, dtype=torch.int32, device=dev)
    # unique list too small
    small_unique = torch.full((U - 10 + 1,), -5, dtype=torch.int32, device=dev)
    h.prepare_batch(seeds, sp.fanouts, 3, hops, sizes, small_unique[:U - 10], inverse, nu, out, full, full.clone(), full.clone(), stats)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY and int(nu[0]) == U
    assert int(small_unique[U - 10]) == -5 and np.array_equal(small_unique[:U - 10].cpu().numpy(), good["unique"][:U - 10])
    # miss list too small
    unique = torch.empty(cap, dtype=torch.int32, device=dev)
    mp = torch.full((n_miss - 3 + 1,), -5, dtype=torch.int32, device=dev)
    h.prepare_batch(seeds, sp.fanouts, 3, hops, sizes, unique, inverse, nu, out, mp[:n_miss - 3], full[:n_miss - 3], full.clone()[:n_miss - 3], stats)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY and int(stats[3]) == n_miss
    assert int(mp[n_miss - 3]) == -5 and np.array_equal(mp[:n_miss - 3].cpu().numpy(), good["miss_pos"][:n_miss - 3])
    # a frontier buffer too small for hop 1
    nf1 = good["hops"][1][0].size
    tight = [hops[0], helios.HopBuffers(torch.full((nf1 - 5,), -5, dtype=torch.int32, device=dev),
                                        torch.empty(nf1 - 5 + 1, dtype=torch.int64, device=dev), hops[1].flat)]
    h.prepare_batch(seeds, sp.fanouts, 3, tight, sizes, unique, inverse, nu, out, full, full.clone(), full.clone(), stats)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY
    # and the context still gives the right answer
    assert_same(gpu_path(h, helios, seeds, sp.fanouts, 3, fused=True), good)


def test_three_batches_in_flight(helios, oracle, workloads):
    """The benchmark's launch configuration: three contexts, each on its own stream with its own
    buffers, all sharing the graph and the cache tables; every batch must still match the oracle."""
    sp, g, feats = workloads(1)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    dev = torch.device("cuda", 0)
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    first = helios.Helios(0)
    first.csr_load(off_d, idx_d)
    cache = GpuCache(first, feats, g.order, n_hbm, n_host)
    lanes = [first]
    for _ in range(2):
        ctx = helios.Helios(0, stream=torch.cuda.Stream(device=dev))
        ctx.csr_load(off_d, idx_d)
        ctx.cache_build(cache.order, n_hbm, n_host, cache.row_bytes, cache.hbm, cache.host, cache.standin)
        ctx.sync()
        lanes.append(ctx)
    torch.cuda.synchronize()
    B = sp.batch
    bufs = []
    for ctx in lanes:
        hops = helios.alloc_hops(B, sp.fanouts, dev)
        cap = B + sum(hb.flat.numel() for hb in hops)
        bufs.append(dict(hops=hops, unique=torch.empty(cap, dtype=torch.int32, device=dev),
                         inverse=torch.empty(cap, dtype=torch.int32, device=dev),
                         out=torch.full((cap, sp.row_bytes), SENTINEL, dtype=torch.uint8, device=dev),
                         mp=torch.empty(cap, dtype=torch.int32, device=dev), mi=torch.empty(cap, dtype=torch.int32, device=dev),
                         ms=torch.empty(cap, dtype=torch.int32, device=dev),
                         sizes=torch.zeros(4, dtype=torch.int64).pin_memory(), nu=torch.zeros(1, dtype=torch.int64).pin_memory(),
                         stats=torch.zeros(4, dtype=torch.int64).pin_memory()))
    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    n_batches = 9
    seeds = [W.seed_batch(sp, g, b).cuda() for b in range(n_batches)]
    torch.cuda.synchronize()

    def check(b):
        ctx, bf = lanes[b % 3], bufs[b % 3]
        ctx.sync()
        want = oracle_path(oracle, g.offsets.numpy(), g.indices.numpy(), seeds[b].cpu().numpy(), sp.fanouts, 100 + b, rank,
                           n_hbm, n_host, *tabs, sp.row_bytes)
        U, nm = int(bf["nu"][0]), int(bf["stats"][3])
        assert bf["stats"].tolist() == want["stats"].tolist()
        assert np.array_equal(bf["unique"][:U].cpu().numpy(), want["unique"])
        assert np.array_equal(bf["mp"][:nm].cpu().numpy(), want["miss_pos"])
        assert np.array_equal(bf["out"][:U].cpu().numpy(), want["out"])
        for k in range(len(sp.fanouts)):
            nfl = int(bf["sizes"][2 * k + 1])
            assert np.array_equal(bf["hops"][k].flat[:nfl].cpu().numpy(), want["hops"][k][2])

    for b in range(n_batches):
        ctx, bf = lanes[b % 3], bufs[b % 3]
        if b >= 3:
            check(b - 3)
            bf["out"].fill_(SENTINEL)
            torch.cuda.synchronize()
        ctx.prepare_batch(seeds[b], sp.fanouts, 100 + b, bf["hops"], bf["sizes"], bf["unique"], bf["inverse"], bf["nu"],
                          bf["out"], bf["mp"], bf["mi"], bf["ms"], bf["stats"])
        ctx.gather_miss(bf["mp"], bf["ms"], bf["mp"].numel(), bf["stats"][3:4], bf["out"])
    for b in range(n_batches - 3, n_batches):
        check(b)
    for ctx in lanes:
        ctx.close()


def test_many_streams_with_large_scans(helios, oracle):
    """Six contexts on six streams, each with scan kernels of about 1500 tiles queued back to back:
    more waiting workgroups than the chip holds at once.  Every tile must still only wait for tiles
    that have started (no HELIOS_EINTERNAL, no hang), and every result must match the oracle."""
    dev = torch.device("cuda", 0)
    n_nodes, n_ids, lanes = 3_000_000, 1_500_000, 6
    rng = np.random.default_rng(21)
    off = torch.zeros(n_nodes + 1, dtype=torch.int64, device=dev)
    idx = torch.zeros(1, dtype=torch.int32, device=dev)
    order = torch.from_numpy(rng.permutation(n_nodes).astype(np.int32)).to(dev)
    table = torch.zeros((1, 16), dtype=torch.uint8, device=dev)
    ctxs, bufs = [], []
    for k in range(lanes):
        ctx = helios.Helios(0, stream=torch.cuda.Stream(device=dev))
        ctx.csr_load(off, idx)
        ctx.cache_build(order, 0, 0, 16, None, None, None)        # every ID is a miss: the miss list is the third scan
        ids = rng.integers(0, n_nodes, n_ids).astype(np.int32)
        ids[rng.random(n_ids) < 0.3] = ids[0]                     # a hot ID, as a sampled hub is
        bufs.append(dict(ids_np=ids, ids=torch.from_numpy(ids).to(dev),
                         uniq=torch.empty(n_ids, dtype=torch.int32, device=dev), inv=torch.empty(n_ids, dtype=torch.int32, device=dev),
                         nu=torch.zeros(1, dtype=torch.int64).pin_memory(), out=torch.zeros((n_ids, 16), dtype=torch.uint8, device=dev),
                         mp=torch.empty(n_ids, dtype=torch.int32, device=dev), mi=torch.empty(n_ids, dtype=torch.int32, device=dev),
                         ms=torch.empty(n_ids, dtype=torch.int32, device=dev), stats=torch.zeros(4, dtype=torch.int64).pin_memory()))
        ctx.reserve(n_ids)
        ctxs.append(ctx)
    for ctx in ctxs:
        ctx.sync()
    torch.cuda.synchronize()
    for rep in range(4):
        for ctx, b in zip(ctxs, bufs):                            # queue everything, then wait
            ctx.dedup(b["ids"], b["uniq"], b["inv"], b["nu"])
            ctx.gather(b["ids"], b["out"], b["mp"], b["mi"], b["ms"], b["stats"])
        for ctx in ctxs:
            ctx.sync()
        print(" rep", rep, "done", flush=True)
    rank = oracle.rank_build(order.cpu().numpy())
    for ctx, b in zip(ctxs, bufs):
        wu, wi = oracle.dedup(n_nodes, b["ids_np"])
        assert int(b["nu"][0]) == wu.size
        assert np.array_equal(b["uniq"][:wu.size].cpu().numpy(), wu) and np.array_equal(b["inv"].cpu().numpy(), wi)
        assert b["stats"].tolist() == [n_ids, 0, 0, n_ids]
        assert np.array_equal(b["mp"].cpu().numpy(), np.arange(n_ids, dtype=np.int32))
        assert np.array_equal(b["ms"].cpu().numpy(), rank[b["ids_np"]])
        ctx.close()
    del table
