"""The whole path on many small, randomly shaped workloads (graph size and skew, hops, fan-outs around the
group widths, batch sizes, seeds with repeats, row sizes, tier splits including empty tiers), each through the
directly launched call, a recorded batch, and a gang, against the CPU oracle.  The shapes come from a fixed list of
seeds, so every run sees the same cases."""
import random

import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, SENTINEL, assert_same, gpu_path, oracle_path, to_bytes

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def helios():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2310_00837_amd import helios as hl
    return hl


def _shape(case: int):
    rnd = random.Random(7700 + case)
    n_nodes = rnd.choice([64, 300, 1500, 6000, 20000])
    avg_deg = rnd.choice([1.5, 4, 12, 30])
    n_hops = rnd.choice([1, 2, 2, 3, 4])
    fanouts = [rnd.choice([0, 1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100]) for _ in range(n_hops)]
    batch = rnd.choice([1, 2, 17, 64, 255, 256, 257, 600])
    dim, dtype = rnd.choice([(4, torch.float32), (8, torch.float16), (24, torch.float32), (64, torch.float32),
                             (128, torch.float32), (200, torch.float32), (1024, torch.float16), (1028, torch.float32)])
    row_bytes = dim * (4 if dtype == torch.float32 else 2)
    while batch * int(np.prod([max(f, 1) for f in fanouts])) * row_bytes > (96 << 20):   # keep the worst-case buffers small
        fanouts[rnd.randrange(n_hops)] = rnd.choice([1, 2, 3, 5])
    split = rnd.choice([(0.1, 0.2), (0.0, 0.5), (0.5, 0.0), (0.0, 0.0), (1.0, 0.0), (0.0, 1.0), (0.3, 0.7), (0.02, 0.03)])
    gamma = rnd.choice([2.1, 2.5, 3.0])
    repeats = rnd.random() < 0.4
    return dict(n_nodes=n_nodes, n_edges=int(n_nodes * avg_deg), n_hops=n_hops, fanouts=fanouts, batch=batch, dim=dim,
                dtype=dtype, split=split, gamma=gamma, repeats=repeats, rnd=rnd)


@pytest.mark.parametrize("case", range(36))
def test_random_shape(helios, oracle, case):
    sh = _shape(case)
    sp = W.WorkloadSpec(f"random-{case}", sh["n_nodes"], sh["n_edges"], sh["dim"], sh["dtype"], sh["batch"], sh["fanouts"], 0.5,
                        ("frac", sh["split"][0]), ("frac", sh["split"][1]), gamma=sh["gamma"])
    g = W.make_graph(sp, 900 + case, "cpu")
    feats = W.feature_rows(900 + case, torch.arange(g.n_nodes), sp.dim, sp.dtype)
    n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
    rnd = sh["rnd"]
    B = min(sp.batch, g.n_nodes)

    def seeds_of(k):
        if sh["repeats"]:
            pool = [rnd.randrange(g.n_nodes) for _ in range(max(1, B // 3))]
            return torch.tensor([rnd.choice(pool) for _ in range(B)], dtype=torch.int32)
        return torch.tensor(rnd.sample(range(g.n_nodes), B), dtype=torch.int32)

    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    off, idx = g.offsets.numpy(), g.indices.numpy()
    st = torch.cuda.Stream()
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    members = 1 + case % 4
    ctxs, cache = [], None
    for m in range(members):
        h = helios.Helios(0, stream=st)
        h.csr_load(off_d, idx_d)
        if cache is None:
            cache = GpuCache(h, feats, g.order, n_hbm, n_host)
        else:
            h.cache_build(cache.order, n_hbm, n_host, sp.row_bytes, cache.hbm if n_hbm else None, cache.host if n_host else None,
                          cache.standin if n_rest else None)
        ctxs.append(h)
    # directly launched: the three calls one after the other, and the whole-path call
    s0 = seeds_of(0)
    want = oracle_path(oracle, off, idx, s0.numpy(), sp.fanouts, 31 + case, rank, n_hbm, n_host, *tabs, sp.row_bytes)
    assert_same(gpu_path(ctxs[0], helios, s0, sp.fanouts, 31 + case, fused=False, serve_misses=n_rest > 0), want)
    assert_same(gpu_path(ctxs[0], helios, s0, sp.fanouts, 31 + case, fused=True, serve_misses=n_rest > 0), want)

    dev = ctxs[0].device

    def buffers():
        hops = helios.alloc_hops(B, sp.fanouts, dev)
        full = B + sum(hb.flat.numel() for hb in hops)
        return helios.BatchBuffers(
            hops=hops, sizes=torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory(),
            unique=torch.empty(full, dtype=torch.int32, device=dev), inverse=torch.empty(full, dtype=torch.int32, device=dev),
            n_unique=torch.zeros(1, dtype=torch.int64).pin_memory(),
            out=torch.full((full, sp.row_bytes), SENTINEL, dtype=torch.uint8, device=dev),
            miss_pos=torch.empty(full, dtype=torch.int32, device=dev), miss_id=torch.empty(full, dtype=torch.int32, device=dev),
            miss_slot=torch.empty(full, dtype=torch.int32, device=dev), stats=torch.zeros(4, dtype=torch.int64).pin_memory())

    def result(bs):
        K = len(sp.fanouts)
        sizes, U, nm = bs.sizes, int(bs.n_unique[0]), int(bs.stats[3])
        r = {"hops": []}
        for k in range(K):
            nf, nfl = int(sizes[2 * k]), int(sizes[2 * k + 1])
            hb = bs.hops[k]
            r["hops"].append((hb.frontier[:nf].cpu().numpy(), hb.indptr[:nf + 1].cpu().numpy(), hb.flat[:nfl].cpu().numpy()))
        n_cat = B + sum(int(sizes[2 * k + 1]) for k in range(K))
        r.update(unique=bs.unique[:U].cpu().numpy(), inverse=bs.inverse[:n_cat].cpu().numpy(), stats=bs.stats.numpy().copy(),
                 miss_pos=bs.miss_pos[:nm].cpu().numpy(), miss_id=bs.miss_id[:nm].cpu().numpy(),
                 miss_slot=bs.miss_slot[:nm].cpu().numpy(), out_before_miss=bs.out[:U].cpu().numpy())
        return r

    # recorded, replayed twice
    bs = buffers()
    ctxs[0].reserve(bs.inverse.numel())
    plan = ctxs[0].plan_create(B, sp.fanouts, bs.hops, bs.sizes, bs.unique, bs.inverse, bs.n_unique, bs.out, bs.miss_pos, bs.miss_id,
                               bs.miss_slot, bs.stats)
    for k in (1, 2):
        sk = seeds_of(k)
        bs.out.fill_(SENTINEL)
        torch.cuda.synchronize()
        plan.launch(sk.cuda(), 500 + k)
        plan.wait()
        w = oracle_path(oracle, off, idx, sk.numpy(), sp.fanouts, 500 + k, rank, n_hbm, n_host, *tabs, sp.row_bytes)
        del w["out"]
        assert_same(result(bs), w)
    plan.destroy()
    # a gang of 1..4 members, launched twice
    sets = [buffers() for _ in ctxs]
    for h, b_ in zip(ctxs, sets):
        h.reserve(b_.inverse.numel())
        h.sync()
    gang = helios.Gang(ctxs, B, sp.fanouts, sets)
    for rnd_no in range(2):
        sl = [seeds_of(10 + rnd_no * 4 + m) for m in range(members)]
        rs = [700 + rnd_no * 10 + m for m in range(members)]
        for b_ in sets:
            b_.out.fill_(SENTINEL)
        torch.cuda.synchronize()
        gang.launch([s.cuda() for s in sl], rs)
        assert gang.wait() == [0] * members
        for m in range(members):
            w = oracle_path(oracle, off, idx, sl[m].numpy(), sp.fanouts, rs[m], rank, n_hbm, n_host, *tabs, sp.row_bytes)
            del w["out"]
            assert_same(result(sets[m]), w)
    gang.destroy()
    for h in ctxs:
        h.close()
