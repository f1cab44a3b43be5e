"""Gangs: the mini-batches of several contexts recorded into the same launches.  Every member's batch
must be what helios_prepare_batch gives on that context, i.e. what the CPU oracle gives, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, SENTINEL, assert_same, gangs_in_flight, gpu_path, oracle_path, to_bytes

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


def _oracle_side(oracle, sp, g, feats):
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    return rank, tabs


def _buffers(helios, ctx, sp, cap=None):
    dev = ctx.device
    hops = helios.alloc_hops(sp.batch, sp.fanouts, dev)
    full = sp.batch + sum(hb.flat.numel() for hb in hops)
    cap = full if cap is None else cap
    return helios.BatchBuffers(
        hops=hops, sizes=torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory(),
        unique=torch.empty(cap, dtype=torch.int32, device=dev), inverse=torch.empty(full, dtype=torch.int32, device=dev),
        n_unique=torch.zeros(1, dtype=torch.int64).pin_memory(),
        out=torch.full((cap, sp.row_bytes), SENTINEL, dtype=torch.uint8, device=dev),
        miss_pos=torch.empty(cap, dtype=torch.int32, device=dev), miss_id=torch.empty(cap, dtype=torch.int32, device=dev),
        miss_slot=torch.empty(cap, dtype=torch.int32, device=dev), stats=torch.zeros(4, dtype=torch.int64).pin_memory())


def _result(bs, sp):
    K = len(sp.fanouts)
    sizes, U, nm = bs.sizes, int(bs.n_unique[0]), int(bs.stats[3])
    r = {"hops": []}
    for k in range(K):
        nf, nfl = int(sizes[2 * k]), int(sizes[2 * k + 1])
        hb = bs.hops[k]
        r["hops"].append((hb.frontier[:nf].cpu().numpy(), hb.indptr[:nf + 1].cpu().numpy(), hb.flat[:nfl].cpu().numpy()))
    n_cat = sp.batch + sum(int(sizes[2 * k + 1]) for k in range(K))
    r.update(unique=bs.unique[:U].cpu().numpy(), inverse=bs.inverse[:n_cat].cpu().numpy(), stats=bs.stats.numpy().copy(),
             miss_pos=bs.miss_pos[:nm].cpu().numpy(), miss_id=bs.miss_id[:nm].cpu().numpy(),
             miss_slot=bs.miss_slot[:nm].cpu().numpy(), out_before_miss=bs.out[:U].cpu().numpy())
    return r


@pytest.mark.parametrize("cfg,members,n_gangs", [(0, 1, 1), (0, 2, 2), (0, 4, 2), (1, 3, 2), (1, 4, 1)])
def test_gang_matches_the_oracle(helios, oracle, small, cfg, members, n_gangs):
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    rank, tabs = _oracle_side(oracle, sp, g, feats)
    first = helios.Helios(0)
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    first.csr_load(off_d, idx_d)
    cache = GpuCache(first, feats, g.order, n_hbm, n_host)
    n_jobs = 6 * members
    jobs = [(W.seed_batch(sp, g, b).cuda(), W.batch_rng_seed(SEED, b)) for b in range(n_jobs)]
    got = gangs_in_flight(helios, off_d, idx_d, cache.order, n_hbm, n_host, sp.row_bytes, (cache.hbm, cache.host, cache.standin),
                          sp.batch, sp.fanouts, jobs, members=members, n_gangs=n_gangs)
    for b, res in enumerate(got):
        want = oracle_path(oracle, g.offsets.numpy(), g.indices.numpy(), jobs[b][0].cpu().numpy(), sp.fanouts, jobs[b][1],
                           rank, n_hbm, n_host, *tabs, sp.row_bytes)
        del want["out"]
        assert_same(res, want)
    first.close()


def test_members_report_their_own_errors_and_make_blocks(helios, oracle, small):
    """Three members; the second one's unique list is too small: only that member reports ECAPACITY, the others'
    batches are correct, their hops can be put into local numbering, and the members' contexts still serve direct
    calls between the gang's launches."""
    sp, g, feats = small(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    rank, tabs = _oracle_side(oracle, sp, g, feats)
    off, idx = g.offsets.numpy(), g.indices.numpy()
    st = torch.cuda.Stream()
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    ctxs = []
    cache = None
    for m in range(3):
        h = helios.Helios(0, stream=st)
        h.csr_load(off_d, idx_d)
        if cache is None:
            cache = GpuCache(h, feats, g.order, n_hbm, n_host)
        else:
            h.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
        ctxs.append(h)
    seeds = [W.seed_batch(sp, g, b).cuda() for b in range(6)]
    ref1 = gpu_path(ctxs[1], helios, seeds[1], sp.fanouts, 11, fused=True, serve_misses=False)
    U1 = ref1["unique"].size
    sets = [_buffers(helios, ctxs[0], sp), _buffers(helios, ctxs[1], sp, cap=U1 - 5), _buffers(helios, ctxs[2], sp)]
    for h, bs in zip(ctxs, sets):
        h.reserve(bs.inverse.numel())
        h.sync()
    gang = helios.Gang(ctxs, sp.batch, sp.fanouts, sets)
    rows = [torch.empty(hb.frontier.numel(), dtype=torch.int32, device="cuda") for hb in sets[2].hops]
    cols = [torch.empty(hb.flat.numel(), dtype=torch.int32, device="cuda") for hb in sets[2].hops]
    for rnd in range(3):
        mine = [seeds[(rnd + m) % 6] if m != 1 else seeds[1] for m in range(3)]
        rs = [11 + 100 * rnd + m if m != 1 else 11 for m in range(3)]
        for bs in sets:
            bs.out.fill_(SENTINEL)
        torch.cuda.synchronize()
        gang.launch(mine, rs)
        gang.make_blocks(2, rows, cols)
        status = gang.wait(raise_on_error=False)
        assert status == [helios.OK, helios.ECAPACITY, helios.OK], status
        assert int(sets[1].n_unique[0]) == U1                       # the size it would have needed
        assert gang.wait(raise_on_error=False) == [0, 0, 0]         # reported once
        for m in (0, 2):
            want = oracle_path(oracle, off, idx, mine[m].cpu().numpy(), sp.fanouts, rs[m], rank, n_hbm, n_host, *tabs, sp.row_bytes)
            del want["out"]
            assert_same(_result(sets[m], sp), want)
            if m == 2:
                ctxs[2].sync()
                nfl0 = int(sets[2].sizes[1])
                assert np.array_equal(cols[0][:nfl0].cpu().numpy(), want["inverse"][sp.batch:sp.batch + nfl0])
                assert np.array_equal(rows[0][:sp.batch].cpu().numpy(), want["inverse"][:sp.batch])
        # a direct call on a member's context between two launches of the gang
        eager = gpu_path(ctxs[rnd % 3], helios, seeds[5], sp.fanouts, 77, fused=True)
        assert_same(eager, oracle_path(oracle, off, idx, seeds[5].cpu().numpy(), sp.fanouts, 77, rank, n_hbm, n_host, *tabs, sp.row_bytes))
    # the error also shows up at the member's own helios_sync, and only there
    gang.launch([seeds[0], seeds[1], seeds[2]], [1, 11, 3])
    ctxs[0].sync()
    with pytest.raises(helios.HeliosError) as e:
        ctxs[1].sync()
    assert e.value.code == helios.ECAPACITY
    # a context with a live gang is not destroyed; a rebuilt cache makes the gang refuse
    assert helios._lib.helios_destroy(ctxs[0]._h) == helios.ESTATE
    ctxs[2].cache_build(cache.order, n_hbm // 2, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
    ctxs[2].sync()
    with pytest.raises(helios.HeliosError) as e:
        gang.launch([seeds[0], seeds[1], seeds[2]], [1, 11, 3])
    assert e.value.code == helios.ESTATE
    gang.destroy()
    for h in ctxs:
        h.close()


def test_gang_argument_errors(helios, small):
    sp, g, feats = small(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    st_a, st_b = torch.cuda.Stream(), torch.cuda.Stream()

    def make(stream):
        h = helios.Helios(0, stream=stream)
        h.csr_load(off_d, idx_d)
        return h
    a = make(st_a)
    cache = GpuCache(a, feats, g.order, n_hbm, n_host)
    others = [make(st_a) for _ in range(4)]
    for h in others:
        h.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
    other_stream = make(st_b)
    other_stream.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
    no_cache = make(st_a)
    every = [a] + others + [other_stream, no_cache]
    bufs = {id(h): _buffers(helios, h, sp) for h in every}

    def create(ctxs, n_seeds=sp.batch, fanouts=sp.fanouts):
        return helios.Gang(ctxs, n_seeds, fanouts, [bufs[id(h)] for h in ctxs])

    def refused(code, *args, **kw):
        with pytest.raises(helios.HeliosError) as e:
            create(*args, **kw)
        assert e.value.code == code, (e.value.code, str(e.value))

    refused(helios.EINVAL, [a] + others)                    # five members
    refused(helios.EINVAL, [a, others[0], a])               # the same context twice
    refused(helios.EINVAL, [a, other_stream])               # another stream
    refused(helios.ESTATE, [a, no_cache])                   # a member without a cache
    on_default = helios.Helios(0)
    on_default.csr_load(off_d, idx_d)
    on_default.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
    bufs[id(on_default)] = _buffers(helios, on_default, sp)
    if on_default._stream_ptr == 0:
        refused(helios.EINVAL, [on_default])                # the NULL stream
    others[0].set_param(helios.PARAM_SPLIT_COPIES, 1)
    refused(helios.ESTATE, [a, others[0]])
    others[0].set_param(helios.PARAM_SPLIT_COPIES, 0)
    others[1].set_timing(2)                                 # event timing cannot be recorded
    refused(helios.ESTATE, [a, others[1]])
    others[1].set_timing(0)
    q = helios.MissQueue(others[2], 4, 1024, 1)
    q.attach()
    refused(helios.ESTATE, [a, others[2]])
    q.destroy()
    # after all the refusals a gang of the same contexts still records and runs
    gang = create([a, others[0], others[1], others[2]])
    seeds = [W.seed_batch(sp, g, b).cuda() for b in range(4)]
    gang.launch(seeds, [1, 2, 3, 4])
    assert gang.wait() == [0, 0, 0, 0]
    ref = gpu_path(others[3], helios, seeds[2], sp.fanouts, 3, fused=True, serve_misses=False)
    mine = _result(bufs[id(others[1])], sp)
    assert np.array_equal(mine["unique"], ref["unique"]) and np.array_equal(mine["out_before_miss"], ref["out_before_miss"])
    gang.destroy()
    on_default.close()
    for h in every:
        h.close()


@pytest.mark.parametrize("cfg", [0, 1])
def test_batches_that_serve_their_own_misses(helios, oracle, small, cfg):
    """HELIOS_PARAM_SERVE_MISSES: the whole-path call also copies the rows of its miss list from the stand-in (S6), as
    a role of its last launch.  Directly launched, with split copies, recorded, and in a gang, `out` must be what the
    oracle has after its miss service, and the miss list is still there."""
    sp, g, feats = small(cfg)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    rank, tabs = _oracle_side(oracle, sp, g, feats)
    off, idx = g.offsets.numpy(), g.indices.numpy()
    st = torch.cuda.Stream()
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    ctxs, cache = [], None
    for m in range(3):
        h = helios.Helios(0, stream=st)
        h.csr_load(off_d, idx_d)
        if cache is None:
            cache = GpuCache(h, feats, g.order, n_hbm, n_host)
        else:
            h.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
        h.set_param(helios.PARAM_SERVE_MISSES, 1)
        ctxs.append(h)
    seeds = [W.seed_batch(sp, g, b).cuda() for b in range(4)]
    wants = [oracle_path(oracle, off, idx, seeds[b].cpu().numpy(), sp.fanouts, 40 + b, rank, n_hbm, n_host, *tabs, sp.row_bytes)
             for b in range(4)]
    assert all(int(w["stats"][3]) > 0 for w in wants)              # there are misses to serve

    def served(res, want):
        got = dict(res)
        got["out"] = got.pop("out_before_miss")                    # what the call left in `out` already has the missed rows
        want = dict(want)
        del want["out_before_miss"]
        assert_same(got, want)

    # directly launched, roles and split copies
    served(gpu_path(ctxs[0], helios, seeds[0], sp.fanouts, 40, fused=True, serve_misses=False), wants[0])
    ctxs[0].set_param(helios.PARAM_SPLIT_COPIES, 1)
    served(gpu_path(ctxs[0], helios, seeds[1], sp.fanouts, 41, fused=True, serve_misses=False), wants[1])
    ctxs[0].set_param(helios.PARAM_SPLIT_COPIES, 0)
    # recorded
    bs = _buffers(helios, ctxs[0], sp)
    ctxs[0].reserve(bs.inverse.numel())
    plan = ctxs[0].plan_create(sp.batch, sp.fanouts, bs.hops, bs.sizes, bs.unique, bs.inverse, bs.n_unique, bs.out, bs.miss_pos,
                               bs.miss_id, bs.miss_slot, bs.stats)
    for b in (2, 3):
        bs.out.fill_(SENTINEL)
        torch.cuda.synchronize()
        plan.launch(seeds[b], 40 + b)
        plan.wait()
        served(_result(bs, sp), wants[b])
    plan.destroy()
    # in a gang
    sets = [_buffers(helios, h, sp) for h in ctxs]
    for h, b_ in zip(ctxs, sets):
        h.reserve(b_.inverse.numel())
        h.sync()
    gang = helios.Gang(ctxs, sp.batch, sp.fanouts, sets)
    for rnd in range(2):
        for b_ in sets:
            b_.out.fill_(SENTINEL)
        torch.cuda.synchronize()
        pick = [(rnd + m) % 4 for m in range(3)]
        gang.launch([seeds[b] for b in pick], [40 + b for b in pick])
        assert gang.wait() == [0, 0, 0]
        for m, b in enumerate(pick):
            served(_result(sets[m], sp), wants[b])
    gang.destroy()
    # not together with an attached miss queue; not without a stand-in table
    q = helios.MissQueue(ctxs[1], 4, 4096, 1)
    q.attach()
    with pytest.raises(helios.HeliosError) as e:
        gpu_path(ctxs[1], helios, seeds[0], sp.fanouts, 40, fused=True, serve_misses=False)
    assert e.value.code == helios.ESTATE
    q.destroy()
    ctxs[2].cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, None)
    with pytest.raises(helios.HeliosError) as e:
        gpu_path(ctxs[2], helios, seeds[0], sp.fanouts, 40, fused=True, serve_misses=False)
    assert e.value.code == helios.ESTATE
    for h in ctxs:
        h.close()


def test_gang_of_small_and_odd_batches(helios, oracle, small):
    """Three hops, a handful of seeds with repeats, a fan-out above the group width of the others, an empty hop: the
    members of a gang take the same steps whatever their data, and each still equals the oracle."""
    sp, g, feats = small(0)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    rank, tabs = _oracle_side(oracle, sp, g, feats)
    off, idx = g.offsets.numpy(), g.indices.numpy()
    st = torch.cuda.Stream()
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    ctxs, cache = [], None
    for m in range(2):
        h = helios.Helios(0, stream=st)
        h.csr_load(off_d, idx_d)
        if cache is None:
            cache = GpuCache(h, feats, g.order, n_hbm, n_host)
        else:
            h.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
        ctxs.append(h)
    hub = int(g.order[0])
    for n_seeds, fanouts in ((5, [3, 70, 2]), (1, [4, 0, 3]), (0, [3, 2]), (7, [2, 2, 2])):
        class Shape:
            batch = n_seeds
            row_bytes = sp.row_bytes
        Shape.fanouts = fanouts
        sets = [_buffers(helios, h, Shape) for h in ctxs]
        for h, bs in zip(ctxs, sets):
            h.reserve(bs.inverse.numel())
            h.sync()
        gang = helios.Gang(ctxs, n_seeds, fanouts, sets)
        for rnd in range(2):
            seed_lists = [torch.tensor(([hub, 17, hub, 4242, 17, 9, 9999] * 2)[m + rnd:m + rnd + n_seeds], dtype=torch.int32).cuda()
                          for m in range(2)]
            rs = [900 + 10 * rnd + m for m in range(2)]
            for bs in sets:
                bs.out.fill_(SENTINEL)
            torch.cuda.synchronize()
            gang.launch(seed_lists, rs)
            assert gang.wait() == [0, 0]
            for m in range(2):
                want = oracle_path(oracle, off, idx, seed_lists[m].cpu().numpy(), fanouts, rs[m], rank, n_hbm, n_host, *tabs, sp.row_bytes)
                del want["out"]
                assert_same(_result(sets[m], Shape), want)
        if n_seeds == 7:
            # more launches than the ring of per-batch variables has slots, queued without a wait in between
            for k in range(300):
                gang.launch(seed_lists, [5000 + k, 6000 + k])
            assert gang.wait() == [0, 0]
            for m in range(2):
                want = oracle_path(oracle, off, idx, seed_lists[m].cpu().numpy(), fanouts, [5299, 6299][m], rank, n_hbm, n_host, *tabs,
                                   sp.row_bytes)
                got = _result(sets[m], Shape)
                for key in ("unique", "inverse", "stats", "miss_pos", "miss_id", "miss_slot"):
                    assert np.array_equal(got[key], want[key]), key
        gang.destroy()
    for h in ctxs:
        h.close()


def test_roles_of_a_gang_are_timed_per_member(helios, oracle, small):
    """Timing level 1 is part of a gang's recording: every member gets the ticks of its own roles, the results stay
    those of the oracle, and the members' roles of one launch run at the same time."""
    sp, g, feats = small(1)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    rank, tabs = _oracle_side(oracle, sp, g, feats)
    off, idx = g.offsets.numpy(), g.indices.numpy()
    st = torch.cuda.Stream()
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    ctxs, cache = [], None
    for m in range(3):
        h = helios.Helios(0, stream=st)
        h.csr_load(off_d, idx_d)
        if cache is None:
            cache = GpuCache(h, feats, g.order, n_hbm, n_host)
        else:
            h.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm, cache.host, cache.standin)
        h.set_timing(1)
        ctxs.append(h)
    sets = [_buffers(helios, h, sp) for h in ctxs]
    for h, bs in zip(ctxs, sets):
        h.reserve(bs.inverse.numel())
        h.sync()
    gang = helios.Gang(ctxs, sp.batch, sp.fanouts, sets)
    for rnd in range(2):
        seeds = [W.seed_batch(sp, g, 3 * rnd + m).cuda() for m in range(3)]
        rs = [W.batch_rng_seed(SEED, 3 * rnd + m) for m in range(3)]
        for bs in sets:
            bs.out.fill_(SENTINEL)
        torch.cuda.synchronize()
        gang.launch(seeds, rs)
        assert gang.wait() == [0, 0, 0]
        for m in range(3):
            want = oracle_path(oracle, off, idx, seeds[m].cpu().numpy(), sp.fanouts, rs[m], rank, n_hbm, n_host, *tabs, sp.row_bytes)
            del want["out"]
            assert_same(_result(sets[m], sp), want)
        per_member = []
        for h in ctxs:
            roles, per_us = h.batch_ticks()
            live = {(kind, stage): (a, z) for kind, stage, wgs, a, z in roles if z > a}
            assert per_us > 0
            for key in ((helios.ROLE_SAMPLE, 0), (helios.ROLE_SAMPLE, 1), (helios.ROLE_COMPACT_LOOKUP, 0), (helios.ROLE_COMPACT_LOOKUP, 1),
                        (helios.ROLE_COPY_HBM, 1), (helios.ROLE_COPY_HOST, 0), (helios.ROLE_COPY_HOST, 1), (helios.ROLE_INVERSE, 1)):
                assert key in live, (key, sorted(live))
            per_member.append(live)
        # the last host-tier copies of the three members share a launch: each starts before the others end
        spans = [pm[(helios.ROLE_COPY_HOST, 1)] for pm in per_member]
        assert max(a for a, _ in spans) < min(z for _, z in spans)
    gang.destroy()
    for h in ctxs:
        h.close()
