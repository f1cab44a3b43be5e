"""GPU parity of the steps around the path: batch generation in local numbering, pre-sampling
hotness and its order, and topology kept in pinned host memory (read by the GPU directly)."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, assert_same, gpu_path, oracle_path, to_bytes

pytestmark = pytest.mark.gpu
SEED = 1234


@pytest.fixture(scope="module")
def helios():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2310_00837_amd import helios as hl
    return hl


@pytest.fixture(scope="module")
def small():
    made = {}

    def get(cfg):
        if cfg not in made:
            sp = W.spec(cfg)
            g = W.make_graph(sp, SEED, "cpu")
            feats = W.feature_rows(SEED, torch.arange(g.n_nodes), sp.dim, sp.dtype)
            made[cfg] = (sp, g, feats)
        return made[cfg]
    return get


def _batch_buffers(helios, h, sp, B):
    dev = h.device
    hops = helios.alloc_hops(B, sp.fanouts, dev)
    cap = B + sum(hb.flat.numel() for hb in hops)
    bufs = dict(hops=hops, cap=cap,
                unique=torch.empty(cap, dtype=torch.int32, device=dev), inverse=torch.empty(cap, dtype=torch.int32, device=dev),
                out=torch.empty((cap, sp.row_bytes), dtype=torch.uint8, device=dev),
                mp=torch.empty(cap, dtype=torch.int32, device=dev), mi=torch.empty(cap, dtype=torch.int32, device=dev),
                ms=torch.empty(cap, dtype=torch.int32, device=dev),
                sizes=torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory(),
                n_unique=torch.zeros(1, dtype=torch.int64).pin_memory(), stats=torch.zeros(4, dtype=torch.int64).pin_memory())
    return bufs


def _prepare(h, sp, seeds, rs, b):
    h.prepare_batch(seeds, sp.fanouts, rs, b["hops"], b["sizes"], b["unique"], b["inverse"], b["n_unique"], b["out"],
                    b["mp"], b["mi"], b["ms"], b["stats"])


@pytest.mark.parametrize("cfg", [0, 1])
def test_blocks_in_local_numbering(helios, oracle, small, cfg):
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    B = sp.batch
    b = _batch_buffers(helios, h, sp, B)
    rows = [torch.full((hb.frontier.numel(),), -7, dtype=torch.int32, device="cuda") for hb in b["hops"]]
    cols = [torch.full((hb.flat.numel(),), -7, dtype=torch.int32, device="cuda") for hb in b["hops"]]
    for batch in range(2):
        seeds = W.seed_batch(sp, g, batch).cuda()
        rs = W.batch_rng_seed(SEED, batch)
        _prepare(h, sp, seeds, rs, b)
        h.make_blocks(b["hops"], rows, cols)
        h.gather_miss(b["mp"], b["ms"], b["mp"].numel(), b["stats"][3:4], b["out"])
        h.sync()
        U = int(b["n_unique"][0])
        uniq = b["unique"][:U].cpu().numpy()
        inv = b["inverse"].cpu().numpy()
        off = seeds.numel()
        for k, hb in enumerate(b["hops"]):
            nf, nfl = int(b["sizes"][2 * k]), int(b["sizes"][2 * k + 1])
            fr, fl = hb.frontier[:nf].cpu().numpy(), hb.flat[:nfl].cpu().numpy()
            assert np.array_equal(rows[k][:nf].cpu().numpy(), oracle.local_ids(g.n_nodes, uniq, fr))
            assert np.array_equal(cols[k][:nfl].cpu().numpy(), oracle.local_ids(g.n_nodes, uniq, fl))
            assert np.array_equal(cols[k][:nfl].cpu().numpy(), inv[off:off + nfl])      # = the slice of the inverse map
            off += nfl
            # the block addresses feature rows: row i of the hop is out[row_local[i]] = feat(frontier[i])
            got = b["out"][rows[k][:nf].long()].cpu().numpy()
            assert np.array_equal(got, to_bytes(feats)[fr])
    # the relabelling reads the batch's own hash table, which a stand-alone de-duplication in between leaves alone
    # (it works on the table of the context's next batch)
    want_rows = [r.clone() for r in rows]
    scratch_u = torch.empty_like(b["unique"])
    scratch_n = torch.zeros(1, dtype=torch.int64).pin_memory()
    h.dedup(seeds, scratch_u, None, scratch_n)
    for r in rows:
        r.fill_(-7)
    h.make_blocks(b["hops"], rows, cols)
    h.sync()
    for k, hb in enumerate(b["hops"]):
        nf = int(b["sizes"][2 * k])
        assert np.array_equal(rows[k][:nf].cpu().numpy(), want_rows[k][:nf].cpu().numpy())
    # before any batch there is nothing to relabel
    fresh = helios.Helios(0)
    fresh.csr_load(g.offsets.cuda(), g.indices.cuda())
    with pytest.raises(helios.HeliosError) as e:
        fresh.make_blocks(b["hops"], rows, cols)
    assert e.value.code == helios.ESTATE
    fresh.close()
    h.close()


@pytest.mark.parametrize("cfg", [0, 1])
def test_blocks_of_queued_plans(helios, oracle, small, cfg):
    """Two recorded plans over two buffer sets on one context, used in turn (the benchmark's launch pattern): the
    blocks of batch A are made after batch B has been launched behind it, from A's own table and buffers."""
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    stream = torch.cuda.Stream()
    h = helios.Helios(0, stream=stream)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    B = sp.batch
    sets = []
    for _ in range(2):
        b = _batch_buffers(helios, h, sp, B)
        b["rows"] = [torch.full((hb.frontier.numel(),), -7, dtype=torch.int32, device="cuda") for hb in b["hops"]]
        b["cols"] = [torch.full((hb.flat.numel(),), -7, dtype=torch.int32, device="cuda") for hb in b["hops"]]
        sets.append(b)
    h.reserve(sets[0]["unique"].numel())
    torch.cuda.synchronize()
    for b in sets:
        b["plan"] = h.plan_create(B, sp.fanouts, b["hops"], b["sizes"], b["unique"], b["inverse"], b["n_unique"], b["out"],
                                  b["mp"], b["mi"], b["ms"], b["stats"])
    n_batches = 7

    def check(b, batch):
        U = int(b["n_unique"][0])
        uniq = b["unique"][:U].cpu().numpy()
        want_u, _ = oracle.dedup(g.n_nodes, np.concatenate(
            [W.seed_batch(sp, g, batch).numpy()] + [hb.flat[:int(b["sizes"][2 * k + 1])].cpu().numpy() for k, hb in enumerate(b["hops"])]))
        assert np.array_equal(uniq, want_u)
        for k, hb in enumerate(b["hops"]):
            nf, nfl = int(b["sizes"][2 * k]), int(b["sizes"][2 * k + 1])
            fr, fl = hb.frontier[:nf].cpu().numpy(), hb.flat[:nfl].cpu().numpy()
            assert np.array_equal(b["rows"][k][:nf].cpu().numpy(), oracle.local_ids(g.n_nodes, uniq, fr)), (batch, k)
            assert np.array_equal(b["cols"][k][:nfl].cpu().numpy(), oracle.local_ids(g.n_nodes, uniq, fl)), (batch, k)

    seeds = [W.seed_batch(sp, g, k).cuda() for k in range(n_batches)]
    sets[0]["plan"].launch(seeds[0], W.batch_rng_seed(SEED, 0))
    for batch in range(1, n_batches + 1):
        prev = sets[(batch - 1) % 2]
        if batch < n_batches:
            sets[batch % 2]["plan"].launch(seeds[batch], W.batch_rng_seed(SEED, batch))     # queued behind the previous batch
        prev["plan"].wait()
        prev["plan"].make_blocks(prev["rows"], prev["cols"])                                   # after the next batch's launch
        torch.cuda.synchronize()
        prev["plan"].wait()                                                                    # would report an ID that is not in the table
        check(prev, batch - 1)
    # two more batches launched since a plan's: its table has been emptied for a later batch
    sets[1]["plan"].launch(seeds[1], 2)
    sets[0]["plan"].launch(seeds[2], 3)
    sets[1]["plan"].make_blocks(sets[1]["rows"], sets[1]["cols"])                              # one batch behind: still fine
    sets[0]["plan"].launch(seeds[3], 4)
    with pytest.raises(helios.HeliosError) as e:
        sets[1]["plan"].make_blocks(sets[1]["rows"], sets[1]["cols"])
    assert e.value.code == helios.ESTATE
    h.sync()
    for b in sets:
        b["plan"].destroy()
    h.close()


@pytest.mark.parametrize("cfg", [0, 1])
def test_presampling_hotness_and_order(helios, oracle, small, cfg):
    """Sec. 3.2.2 "Cache Initialization": hotness counted over pre-sampling batches and the order sorted from it, on
    the 10 k-node and on the 1 M-node workload, against the oracle; the tiers placed by that order serve a batch."""
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    off, idx = g.offsets.numpy(), g.indices.numpy()
    h = helios.Helios(0)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)          # any placement will do for pre-sampling
    b = _batch_buffers(helios, h, sp, sp.batch)
    counts = torch.zeros(g.n_nodes, dtype=torch.int32, device="cuda")
    want_counts = np.zeros(g.n_nodes, np.int32)
    n_batches = 7 if cfg == 0 else 12                            # the train split of workload 0 has 7 full batches
    for batch in range(n_batches):
        seeds = W.seed_batch(sp, g, batch)
        rs = W.batch_rng_seed(SEED, batch)
        _prepare(h, sp, seeds.cuda(), rs, b)
        h.hotness_add(b["unique"], b["unique"].numel(), b["n_unique"], counts)       # count stays on the device
        hops = oracle.sample(off, idx, seeds.numpy(), sp.fanouts, rs)
        uq, _ = oracle.dedup(g.n_nodes, np.concatenate([seeds.numpy()] + [fl for _, _, fl in hops]))
        oracle.hotness_add(uq, want_counts)
    h.sync()
    assert np.array_equal(counts.cpu().numpy(), want_counts)
    order = torch.empty(g.n_nodes, dtype=torch.int32, device="cuda")
    h.hotness_order(counts, order)
    h.sync()
    want_order = oracle.hotness_order(want_counts)
    assert np.array_equal(order.cpu().numpy(), want_order)
    # the pre-sampled order is a valid cache placement: whole path, bit-exact, with tiers filled by it
    cache2 = GpuCache(h, feats, order.cpu(), n_hbm, n_host)  # noqa: F841
    rank = oracle.rank_build(want_order)
    by_rank = to_bytes(feats)[want_order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    seeds = W.seed_batch(sp, g, 3)
    want = oracle_path(oracle, off, idx, seeds.numpy(), sp.fanouts, 5, rank, n_hbm, n_host, *tabs, sp.row_bytes)
    assert_same(gpu_path(h, helios, seeds, sp.fanouts, 5, fused=True), want)
    # hot nodes by pre-sampling beat the in-degree proxy or tie with it on the batches they were counted on
    hit_presampled = int(want["stats"][1])
    del cache
    h.close()
    assert hit_presampled > 0


@pytest.mark.parametrize("cfg", [0, 1])
def test_topology_in_pinned_host_memory(helios, oracle, small, cfg):
    """The graph may stay in CPU memory and be read by the sampling kernel through the mapped
    address (Sec. 3.2.1 keeps the whole topology in the CPU cache)."""
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0)
    off_pin, idx_pin = g.offsets.clone().pin_memory(), g.indices.clone().pin_memory()
    h.csr_load(off_pin, idx_pin)
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    for batch in range(2):
        seeds = W.seed_batch(sp, g, batch)
        rs = W.batch_rng_seed(SEED, batch)
        want = oracle_path(oracle, g.offsets.numpy(), g.indices.numpy(), seeds.numpy(), sp.fanouts, rs, rank, n_hbm,
                           n_host, *tabs, sp.row_bytes)
        assert_same(gpu_path(h, helios, seeds, sp.fanouts, rs, fused=True), want)
    h.close()
