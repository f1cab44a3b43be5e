"""The asynchronous miss queue (submission kernel -> service threads -> completion kernel) must
leave in `out` exactly what the oracle's miss gather leaves: rows of misses equal features[id],
every other row untouched.  How the commands are spread over the queues and in which order they
complete is the queue's own business and is not compared."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, SENTINEL, assert_same, oracle_path, to_bytes

pytestmark = pytest.mark.gpu
SEED = 1234


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


def _small_cache(h, rng, n, row_bytes, n_hbm, n_host):
    feats = torch.from_numpy(rng.integers(0, 256, (n, row_bytes), dtype=np.uint8))
    order = torch.from_numpy(rng.permutation(n).astype(np.int32))
    h.csr_load(torch.zeros(n + 1, dtype=torch.int64, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"))
    cache = GpuCache(h, feats, order, n_hbm, n_host)
    return feats, order, cache


@pytest.mark.parametrize("row_bytes", [16, 512, 2048, 4112])
@pytest.mark.parametrize("shape", [(1, 4096, 1), (7, 600, 2), (64, 64, 3), (300, 14, 4), (4096, 1, 2)])
def test_missq_rounds_match_the_oracle(h, helios, oracle, row_bytes, shape):
    n_queues, depth, threads = shape
    print("missq", row_bytes, shape, flush=True)
    rng = np.random.default_rng(row_bytes + n_queues)
    n, n_hbm, n_host = 6000, 600, 1200
    feats, order, cache = _small_cache(h, rng, n, row_bytes, n_hbm, n_host)
    by_rank = feats.numpy()[order.numpy()]
    rank = oracle.rank_build(order.numpy())
    q = helios.MissQueue(h, n_queues, depth, threads)
    h.set_param(helios.PARAM_MISSQ_TIMEOUT_US, 20_000_000)
    rounds = misses = 0
    for n_ids in (4000, 0, 1, 333, 4000):                       # the queues are reused round after round
        ids = rng.integers(0, n, n_ids).astype(np.int32)
        if n_ids == 1:
            ids[:] = order.numpy()[-1]                          # a single miss
        out = torch.full((max(n_ids, 1), row_bytes), SENTINEL, dtype=torch.uint8, device="cuda")
        mp = torch.full((max(n_ids, 1),), -9, dtype=torch.int32, device="cuda")
        mi, ms = mp.clone(), mp.clone()
        stats = torch.full((4,), -9, dtype=torch.int64).pin_memory()
        h.gather(torch.from_numpy(ids).cuda(), out, mp, mi, ms, stats, n_ids=n_ids)
        q.submit(mp, ms, mp.numel(), stats[3:4], out.shape[0])
        q.complete(out)
        h.sync()
        wout = np.full((n_ids, row_bytes), SENTINEL, np.uint8)
        wmp, wmi, wms, wstats = oracle.gather(ids, rank, n_hbm, n_host, np.ascontiguousarray(by_rank[:n_hbm]),
                                              np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]), wout)
        assert int(wstats[3]) <= n_queues * depth
        oracle.gather_miss(wmp, wms, np.ascontiguousarray(by_rank[n_hbm + n_host:]), wout)
        assert stats.tolist() == wstats.tolist()
        assert np.array_equal(out[:n_ids].cpu().numpy(), wout)
        assert np.array_equal(wout, feats.numpy()[ids])
        assert not q.faulted()
        rounds, misses = rounds + 1, misses + int(wstats[3])
    opened, served, commands = q.counters()
    assert opened == rounds and commands == misses and served in (rounds - 1, rounds)   # the last round may still be closing
    q.destroy()


def _batch_buffers(helios, sp, dev):
    B = sp.batch
    hops = helios.alloc_hops(B, sp.fanouts, dev)
    cap = B + sum(hb.flat.numel() for hb in hops)
    bf = dict(hops=hops, cap=cap,
              unique=torch.empty(cap, dtype=torch.int32, device=dev), inverse=torch.empty(cap, dtype=torch.int32, device=dev),
              out=torch.full((cap, sp.row_bytes), SENTINEL, dtype=torch.uint8, device=dev),
              mp=torch.empty(cap, dtype=torch.int32, device=dev), mi=torch.empty(cap, dtype=torch.int32, device=dev),
              ms=torch.empty(cap, dtype=torch.int32, device=dev),
              sizes=torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory(),
              nu=torch.zeros(1, dtype=torch.int64).pin_memory(), stats=torch.zeros(4, dtype=torch.int64).pin_memory())
    return bf


def _collect(bf, sp):
    K = len(sp.fanouts)
    sizes, U = bf["sizes"], int(bf["nu"][0])
    res = {"hops": []}
    for k in range(K):
        nf, nfl = int(sizes[2 * k]), int(sizes[2 * k + 1])
        hb = bf["hops"][k]
        res["hops"].append((hb.frontier[:nf].cpu().numpy(), hb.indptr[:nf + 1].cpu().numpy(), hb.flat[:nfl].cpu().numpy()))
    n_cat = sp.batch + sum(int(sizes[2 * k + 1]) for k in range(K))
    nm = int(bf["stats"][3])
    res.update(unique=bf["unique"][:U].cpu().numpy(), inverse=bf["inverse"][:n_cat].cpu().numpy(),
               stats=bf["stats"].numpy().copy(), miss_pos=bf["mp"][:nm].cpu().numpy(), miss_id=bf["mi"][:nm].cpu().numpy(),
               miss_slot=bf["ms"][:nm].cpu().numpy(), out=bf["out"][:U].cpu().numpy())
    return res


@pytest.mark.parametrize("cfg", [0, 1])
def test_batches_submit_their_own_misses(helios, oracle, cfg):
    """With a queue attached, directly launched and recorded batches put their misses on the queue
    right after the lookup; after helios_missq_complete every output equals the oracle's."""
    sp = W.spec(cfg)
    g = W.make_graph(sp, SEED, "cpu")
    feats = W.feature_rows(SEED, torch.arange(g.n_nodes), sp.dim, sp.dtype)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    dev = torch.device("cuda", 0)
    stream = torch.cuda.Stream(device=dev)
    h = helios.Helios(0, stream=stream)
    h.csr_load(g.offsets.cuda(), g.indices.cuda())
    cache = GpuCache(h, feats, g.order, n_hbm, n_host)  # noqa: F841
    torch.cuda.synchronize()
    bf = _batch_buffers(helios, sp, dev)
    h.reserve(bf["cap"])
    q = helios.MissQueue(h, 128, (bf["cap"] + 127) // 128, 3)
    h.set_param(helios.PARAM_MISSQ_TIMEOUT_US, 20_000_000)
    q.attach()
    torch.cuda.synchronize()
    plan = h.plan_create(sp.batch, sp.fanouts, bf["hops"], bf["sizes"], bf["unique"], bf["inverse"], bf["nu"], bf["out"],
                         bf["mp"], bf["mi"], bf["ms"], bf["stats"])
    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    off, idx = g.offsets.numpy(), g.indices.numpy()
    for b in range(6):
        seeds = W.seed_batch(sp, g, b).cuda()
        rs = W.batch_rng_seed(SEED, b)
        bf["out"].fill_(SENTINEL)
        torch.cuda.synchronize()
        if b % 3 == 2:
            h.prepare_batch(seeds, sp.fanouts, rs, bf["hops"], bf["sizes"], bf["unique"], bf["inverse"], bf["nu"],
                            bf["out"], bf["mp"], bf["mi"], bf["ms"], bf["stats"])
        else:
            plan.launch(seeds, rs)
        q.complete(bf["out"])
        h.sync()
        want = oracle_path(oracle, off, idx, seeds.cpu().numpy(), sp.fanouts, rs, rank, n_hbm, n_host, *tabs, sp.row_bytes)
        del want["out_before_miss"]
        assert_same(_collect(bf, sp), want)
        print(" batch", b, "recorded" if b % 3 != 2 else "direct", "misses", int(bf["stats"][3]), flush=True)
    # a batch must be completed before the next one is launched
    seeds = W.seed_batch(sp, g, 0).cuda()
    plan.launch(seeds, 1)
    with pytest.raises(helios.HeliosError) as e:
        plan.launch(seeds, 2)
    assert e.value.code == helios.ESTATE
    q.complete(bf["out"])
    h.sync()
    # a recorded batch runs only with the queue it was recorded with
    q.detach()
    with pytest.raises(helios.HeliosError) as e:
        plan.launch(seeds, 3)
    assert e.value.code == helios.ESTATE
    plan.destroy()
    q.destroy()
    h.close()


def test_missq_capacity_and_state_errors(h, helios, oracle):
    rng = np.random.default_rng(5)
    n, row_bytes = 3000, 64
    feats, order, cache = _small_cache(h, rng, n, row_bytes, 0, 0)          # everything misses
    HE = helios.HeliosError
    q = helios.MissQueue(h, 8, 16, 2)                                        # room for 128 misses a round
    with pytest.raises(HE) as e:
        q.complete(torch.zeros(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == helios.ESTATE
    ids = rng.permutation(n)[:500].astype(np.int32)
    out = torch.full((500, row_bytes), SENTINEL, dtype=torch.uint8, device="cuda")
    mp = torch.empty(500, dtype=torch.int32, device="cuda")
    mi, ms = mp.clone(), mp.clone()
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    h.gather(torch.from_numpy(ids).cuda(), out, mp, mi, ms, stats)
    q.submit(mp, ms, 500, stats[3:4], out.shape[0])
    with pytest.raises(HE) as e:
        q.submit(mp, ms, 500, stats[3:4], out.shape[0])
    assert e.value.code == helios.ESTATE
    q.complete(out)
    with pytest.raises(HE) as e:
        h.sync()
    assert e.value.code == helios.ECAPACITY
    got = out.cpu().numpy()
    assert np.array_equal(got[:128], feats.numpy()[ids[:128]])               # the first 128 were served
    assert (got[128:] == SENTINEL).all()
    # the queue works again with a list that fits
    out.fill_(SENTINEL)
    q.submit(mp, ms, 100, None, out.shape[0])
    q.complete(out)
    h.sync()
    got = out.cpu().numpy()
    assert np.array_equal(got[:100], feats.numpy()[ids[:100]]) and (got[100:] == SENTINEL).all()
    # a queue belongs to the cache it was made for
    h.cache_build(cache.order, 0, 0, row_bytes, None, None, cache.standin)
    h.sync()
    with pytest.raises(HE) as e:
        q.submit(mp, ms, 100, None, out.shape[0])
    assert e.value.code == helios.ESTATE
    q.destroy()
    for bad in ((0, 4, 1), (5000, 4, 1), (4, 0, 1), (4, 4, 65)):
        with pytest.raises(HE) as e:
            helios.MissQueue(h, *bad)
        assert e.value.code == helios.EINVAL


def test_missq_time_limit(h, helios):
    """A service that never answers (no service threads): every wave of the completion kernel
    gives up after the time limit and ends, helios_sync reports it, nothing is written."""
    rng = np.random.default_rng(6)
    n, row_bytes = 1000, 128
    feats, order, cache = _small_cache(h, rng, n, row_bytes, 0, 0)
    q = helios.MissQueue(h, 16, 64, 0)
    h.set_param(helios.PARAM_MISSQ_TIMEOUT_US, 3000)
    ids = torch.arange(700, dtype=torch.int32, device="cuda")
    out = torch.full((700, row_bytes), SENTINEL, dtype=torch.uint8, device="cuda")
    mp = torch.empty(700, dtype=torch.int32, device="cuda")
    mi, ms = mp.clone(), mp.clone()
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    h.gather(ids, out, mp, mi, ms, stats)
    q.submit(mp, ms, 700, stats[3:4], out.shape[0])
    q.complete(out)
    with pytest.raises(helios.HeliosError) as e:
        h.sync()
    assert e.value.code == helios.EINTERNAL
    assert (out.cpu().numpy() == SENTINEL).all()
    q.destroy()
    h.sync()                                                     # the context itself is fine
