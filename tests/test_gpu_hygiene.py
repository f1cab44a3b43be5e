"""GPU tests of the boundary's error handling around recorded batches, caller-supplied miss lists and
capacity overflows, and of the overlap inside a mini-batch (the host-tier copy of one stage beside
the sampling of the next hop)."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, assert_same, gpu_path, oracle_path, to_bytes, SENTINEL

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


def _buffers(helios, h, sp, B, cap=None):
    dev = h.device
    hops = helios.alloc_hops(B, sp.fanouts, dev)
    cap = B + sum(hb.flat.numel() for hb in hops) if cap is None else cap
    return dict(hops=hops, cap=cap, unique=torch.empty(cap, dtype=torch.int32, device=dev),
                inverse=torch.empty(B + sum(hb.flat.numel() for hb in hops), dtype=torch.int32, device=dev),
                out=torch.full((cap, sp.row_bytes), SENTINEL, dtype=torch.uint8, device=dev),
                mp=torch.full((cap,), -9, dtype=torch.int32, device=dev), mi=torch.full((cap,), -9, dtype=torch.int32, device=dev),
                ms=torch.full((cap,), -9, dtype=torch.int32, device=dev),
                sizes=torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory(),
                n_unique=torch.zeros(1, dtype=torch.int64).pin_memory(), stats=torch.zeros(4, dtype=torch.int64).pin_memory())


def _args(b):
    return (b["hops"], b["sizes"], b["unique"], b["inverse"], b["n_unique"], b["out"], b["mp"], b["mi"], b["ms"], b["stats"])


def test_a_recorded_batch_refuses_a_rebuilt_cache_or_graph(helios, small):
    """A recording holds the cache's tier sizes and table pointers and the graph's pointers: after another
    helios_cache_build (the tier sweep of workload 4 does that) or helios_csr_load it must not replay."""
    sp, g, feats = small(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0, stream=torch.cuda.Stream())
    off, idx = g.offsets.cuda(), g.indices.cuda()
    h.csr_load(off, idx)
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)
    b = _buffers(helios, h, sp, sp.batch)
    h.reserve(b["cap"])
    plan = h.plan_create(sp.batch, sp.fanouts, *_args(b))
    seeds = W.seed_batch(sp, g, 0).cuda()
    plan.launch(seeds, 5)
    plan.wait()
    good_stats = b["stats"].tolist()
    h.cache_build(cache.order, n_hbm // 2, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)     # other tier sizes
    h.sync()
    with pytest.raises(helios.HeliosError) as e:
        plan.launch(seeds, 5)
    assert e.value.code == helios.ESTATE
    # a fresh recording on the rebuilt cache works, the old one stays refused
    plan2 = h.plan_create(sp.batch, sp.fanouts, *_args(b))
    plan2.launch(seeds, 5)
    plan2.wait()
    assert b["stats"].tolist() != good_stats and int(b["stats"][0]) == good_stats[0]
    h.csr_load(off, idx)                                   # the same graph again: still a new generation, and no cache
    for p in (plan, plan2):
        with pytest.raises(helios.HeliosError) as e:
            p.launch(seeds, 5)
        assert e.value.code == helios.ESTATE
    plan.destroy()
    plan2.destroy()
    h.close()


def test_every_plan_reports_its_own_errors(helios, small):
    """Two recordings queued on one context: the one whose unique list is too small reports ECAPACITY at its
    own wait; the other, queued behind it, reports nothing and is correct."""
    sp, g, feats = small(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0, stream=torch.cuda.Stream())
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    seeds = W.seed_batch(sp, g, 0).cuda()
    ref = gpu_path(h, helios, seeds, sp.fanouts, 7, fused=True, serve_misses=False)
    U = ref["unique"].size
    tight, roomy = _buffers(helios, h, sp, sp.batch, cap=U - 9), _buffers(helios, h, sp, sp.batch)
    h.reserve(roomy["cap"])
    p_tight = h.plan_create(sp.batch, sp.fanouts, *_args(tight))
    p_roomy = h.plan_create(sp.batch, sp.fanouts, *_args(roomy))
    for _ in range(2):
        p_tight.launch(seeds, 7)
        p_roomy.launch(seeds, 7)
        p_roomy.wait()                                       # the later batch first: it must not get the earlier one's error
        assert int(roomy["n_unique"][0]) == U
        assert np.array_equal(roomy["unique"][:U].cpu().numpy(), ref["unique"])
        assert np.array_equal(roomy["out"][:U].cpu().numpy(), ref["out_before_miss"])
        with pytest.raises(helios.HeliosError) as e:
            p_tight.wait()
        assert e.value.code == helios.ECAPACITY and int(tight["n_unique"][0]) == U
        p_tight.wait()                                       # reported once
    # helios_sync collects the error words of all plans
    p_tight.launch(seeds, 7)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY
    h.sync()
    p_tight.destroy()
    p_roomy.destroy()
    h.close()


def test_capacity_overflow_with_a_miss_queue_attached(helios, small):
    """An output that does not fit while the batch submits its own misses: nothing is queued from list entries
    that were never written, nothing is written past a capacity, the queue completes and works again."""
    sp, g, feats = small(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0, stream=torch.cuda.Stream())
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    seeds = W.seed_batch(sp, g, 0).cuda()
    ref = gpu_path(h, helios, seeds, sp.fanouts, 3, fused=True)
    U, n_miss = ref["unique"].size, ref["miss_pos"].size
    assert n_miss > 8
    q = helios.MissQueue(h, 16, 256, 2)
    q.attach()
    h.set_param(helios.PARAM_MISSQ_TIMEOUT_US, 20_000_000)
    # (1) the unique list (and with it `out`) is too small: no miss is submitted, the rows that fit are untouched by S6
    b = _buffers(helios, h, sp, sp.batch, cap=U - 10)
    h.prepare_batch(seeds, sp.fanouts, 3, *_args(b))
    q.complete(b["out"])
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY and int(b["n_unique"][0]) == U
    assert np.array_equal(b["unique"].cpu().numpy(), ref["unique"][:U - 10])
    assert q.counters()[2] == 0 and not q.faulted()            # no command was served
    # (2) the miss list is too small: the misses that fit are served, the stats give the required size
    b = _buffers(helios, h, sp, sp.batch)
    k = n_miss - 4
    args = list(_args(b))
    args[6], args[7], args[8] = b["mp"][:k], b["mi"][:k], b["ms"][:k]
    h.prepare_batch(seeds, sp.fanouts, 3, *args)
    q.complete(b["out"])
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY and int(b["stats"][3]) == n_miss
    assert int(b["mp"][k]) == -9 and np.array_equal(b["mp"][:k].cpu().numpy(), ref["miss_pos"][:k])
    got = b["out"][:U].cpu().numpy()
    served = ref["miss_pos"][:k]
    assert np.array_equal(got[served], ref["out"][served])
    assert (got[ref["miss_pos"][k:]] == SENTINEL).all()
    assert q.counters()[2] == k
    # (3) and a batch that fits is right
    b = _buffers(helios, h, sp, sp.batch)
    h.prepare_batch(seeds, sp.fanouts, 3, *_args(b))
    q.complete(b["out"])
    h.sync()
    assert np.array_equal(b["out"][:U].cpu().numpy(), ref["out"])
    q.destroy()
    h.close()


def test_miss_lists_of_the_caller_are_range_checked(helios, small):
    """helios_gather_miss and helios_missq_submit take lists the caller wrote: an entry outside the stand-in table
    or outside `out` is reported (EDATA) and never used as an index; the other entries are served."""
    sp, g, feats = small(0)
    n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    rb = sp.row_bytes
    standin = to_bytes(feats)[g.order.numpy()][n_hbm + n_host:]
    n_out = 40
    pos = torch.tensor([0, 1, -1, 3, n_out, 5, 6, 2 ** 31 - 1], dtype=torch.int32, device="cuda")
    slot = torch.tensor([5, n_rest, 7, -3, 9, 2 ** 31 - 1, 11, 12], dtype=torch.int32, device="cuda")
    ok = [0, 6]                                                # entries whose position and slot are both valid
    for via_queue in (False, True):
        out = torch.full((n_out + 8, rb), SENTINEL, dtype=torch.uint8, device="cuda")        # 8 guard rows
        if via_queue:
            q = helios.MissQueue(h, 4, 8, 1)
            h.set_param(helios.PARAM_MISSQ_TIMEOUT_US, 20_000_000)
            q.submit(pos, slot, pos.numel(), None, n_out)
            q.complete(out)
        else:
            h.gather_miss(pos, slot, pos.numel(), None, out, out_rows=n_out)
        with pytest.raises(helios.HeliosError) as e:
            h.sync()
        assert e.value.code == helios.EDATA
        got = out.cpu().numpy()
        want = np.full_like(got, SENTINEL)
        for k in ok:
            want[int(pos[k])] = standin[int(slot[k])]
        assert np.array_equal(got, want)
        if via_queue:
            assert not q.faulted()
            q.destroy()
    # a clean list afterwards is served without an error
    out = torch.full((n_out, rb), SENTINEL, dtype=torch.uint8, device="cuda")
    h.gather_miss(pos[:1], slot[:1], 1, None, out)
    h.sync()
    assert np.array_equal(out[0].cpu().numpy(), standin[5])
    # host-side checks
    with pytest.raises(helios.HeliosError) as e:
        h.gather_miss(pos, slot, pos.numel(), None, out, out_rows=-1)
    assert e.value.code == helios.EINVAL
    # with every node cached nothing can miss: any entry is outside the (empty) stand-in
    h.cache_build(cache.order, g.n_nodes, 0, rb, torch.zeros((g.n_nodes, rb), dtype=torch.uint8, device="cuda"), None, None)
    h.sync()
    h.gather_miss(pos[:1], slot[:1], 1, None, out)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.EDATA
    h.close()


def test_whole_path_with_an_order_that_is_no_permutation(helios, small):
    """helios_cache_build with a hotness order that repeats a node: reported (EDATA) when the map is built and again by
    every batch that meets a node without a rank; such a node is listed as a miss and its slot is no row of any
    table, so no copy uses it."""
    sp, g, feats = small(0)
    n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
    h = helios.Helios(0)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)
    seeds = W.seed_batch(sp, g, 0).cuda()
    ref = gpu_path(h, helios, seeds, sp.fanouts, 3, fused=True, serve_misses=False)
    bad = cache.order.clone()
    victim = int(ref["unique"][5])                              # a node of the batch loses its rank
    at = int((bad == victim).nonzero()[0])
    bad[at] = bad[(at + 1) % bad.numel()]
    h.cache_build(bad, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.EDATA
    b = _buffers(helios, h, sp, sp.batch)
    h.prepare_batch(seeds, sp.fanouts, 3, *_args(b))
    h.gather_miss(b["mp"], b["ms"], b["mp"].numel(), b["stats"][3:4], b["out"])
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.EDATA
    U = int(b["n_unique"][0])
    assert np.array_equal(b["unique"][:U].cpu().numpy(), ref["unique"])
    nm = int(b["stats"][3])
    mi, ms = b["mi"][:nm].cpu().numpy(), b["ms"][:nm].cpu().numpy()
    assert victim in mi and ms[list(mi).index(victim)] == -1
    assert (b["out"][5].cpu().numpy() == SENTINEL).all()        # the node's row is left alone
    h.close()


@pytest.mark.parametrize("cfg", [1])
def test_host_tier_copy_runs_beside_the_next_hop(helios, oracle, small, cfg):
    """The intra-mini-batch overlap (Sec. 3.3): with the roles of a batch timed by the device clock, the host-tier
    copy of stage 0 starts before the last sampling pass has ended, and the batch is still bit-exact."""
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    stream = torch.cuda.Stream()
    h = helios.Helios(0, stream=stream)
    off, idx = g.offsets.cuda(), g.indices.cuda()
    h.csr_load(off, idx)
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    order = g.order.numpy()
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    rank = oracle.rank_build(order)
    b = _buffers(helios, h, sp, sp.batch)
    h.reserve(b["cap"])
    h.set_timing(1)
    plan = h.plan_create(sp.batch, sp.fanouts, *_args(b))
    for recorded in (False, True, True):
        seeds, rs = W.seed_batch(sp, g, 3).cuda(), W.batch_rng_seed(SEED, 3)
        b["out"].fill_(SENTINEL)
        torch.cuda.synchronize()
        if recorded:
            plan.launch(seeds, rs)
        else:
            h.prepare_batch(seeds, sp.fanouts, rs, *_args(b))
        h.sync()
        roles, per_us = h.batch_ticks()
        assert per_us > 0
        kinds = {(k, s) for k, s, _, a, z in roles if z > a}
        K = len(sp.fanouts)
        assert {(helios.ROLE_SAMPLE, s) for s in range(K)} <= kinds
        assert {(helios.ROLE_COPY_HOST, s) for s in range(K)} <= kinds and (helios.ROLE_COPY_HBM, K - 1) in kinds
        first_link = min(a for k, s, _, a, z in roles if k == helios.ROLE_COPY_HOST and z > a)
        last_sample_end = max(z for k, s, _, a, z in roles if k == helios.ROLE_SAMPLE)
        last_lookup_start = max(a for k, s, _, a, z in roles if k == helios.ROLE_COMPACT_LOOKUP and z > a)
        assert first_link < last_sample_end, "the first host-tier copy should start while the last hop is still being sampled"
        assert first_link < last_lookup_start
        want = oracle_path(oracle, g.offsets.numpy(), g.indices.numpy(), seeds.cpu().numpy(), sp.fanouts, rs, rank, n_hbm,
                           n_host, *tabs, sp.row_bytes)
        U, nm = int(b["n_unique"][0]), int(b["stats"][3])
        got = dict(hops=[(b["hops"][k].frontier[:int(b["sizes"][2 * k])].cpu().numpy(),
                          b["hops"][k].indptr[:int(b["sizes"][2 * k]) + 1].cpu().numpy(),
                          b["hops"][k].flat[:int(b["sizes"][2 * k + 1])].cpu().numpy()) for k in range(K)],
                   unique=b["unique"][:U].cpu().numpy(), inverse=b["inverse"][:want["inverse"].size].cpu().numpy(),
                   stats=b["stats"].numpy().copy(), miss_pos=b["mp"][:nm].cpu().numpy(), miss_id=b["mi"][:nm].cpu().numpy(),
                   miss_slot=b["ms"][:nm].cpu().numpy(), out_before_miss=b["out"][:U].cpu().numpy())
        assert_same(got, want)
    h.set_timing(0)
    plan.destroy()
    h.close()
