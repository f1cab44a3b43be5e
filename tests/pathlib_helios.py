"""Shared helpers of the GPU parity tests: run the path through the C ABI (via the thin
binding) and through the CPU oracle on the same inputs, and compare every output array."""
import numpy as np
import torch

SENTINEL = 0xA5


def to_bytes(t: torch.Tensor) -> np.ndarray:
    """[rows, dim] tensor of any dtype -> numpy uint8 [rows, row_bytes] (host copy)."""
    t = t.detach().cpu().contiguous()
    return t.view(torch.uint8).reshape(t.shape[0], -1).numpy() if t.numel() else \
        np.zeros((0, t.shape[1] * t.element_size()), np.uint8)


class GpuCache:
    """Tier tables of a small workload, built from a full feature table through helios_cache_fill."""

    def __init__(self, h, feats: torch.Tensor, order: torch.Tensor, n_hbm: int, n_host: int):
        n, dim = feats.shape
        self.row_bytes = dim * feats.element_size()
        dev = h.device
        self.order = order.to(dev)
        src = feats.to(dev)
        n_rest = n - n_hbm - n_host
        self.hbm = torch.empty((max(n_hbm, 1), dim), dtype=feats.dtype, device=dev)
        self.host = torch.empty((max(n_host, 1), dim), dtype=feats.dtype).pin_memory()
        self.standin = torch.empty((max(n_rest, 1), dim), dtype=feats.dtype).pin_memory()
        h.cache_fill(src, self.order, 0, n_hbm, self.hbm)
        h.cache_fill(src, self.order, n_hbm, n_host, self.host)
        h.cache_fill(src, self.order, n_hbm + n_host, n_rest, self.standin)
        h.sync()
        self.n_hbm, self.n_host, self.n_rest = n_hbm, n_host, n_rest
        h.cache_build(self.order, n_hbm, n_host, self.row_bytes, self.hbm, self.host, self.standin)
        h.sync()


def gpu_path(h, helios, seeds: torch.Tensor, fanouts, rng_seed: int, fused: bool, serve_misses: bool = True):
    """Returns a dict of numpy arrays with every output of the path."""
    dev = h.device
    seeds = seeds.to(dev)
    B = seeds.numel()
    hops = helios.alloc_hops(B, fanouts, dev)
    K = len(fanouts)
    cat_cap = B + sum(hb.flat.numel() for hb in hops)
    sizes = torch.zeros(2 * K, dtype=torch.int64).pin_memory()
    n_unique = torch.zeros(1, dtype=torch.int64).pin_memory()
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    unique = torch.empty(max(cat_cap, 1), dtype=torch.int32, device=dev)
    inverse = torch.empty(max(cat_cap, 1), dtype=torch.int32, device=dev)
    out = torch.full((max(cat_cap, 1), h.row_bytes), SENTINEL, dtype=torch.uint8, device=dev)
    mp = torch.empty(max(cat_cap, 1), dtype=torch.int32, device=dev)
    mi = torch.empty_like(mp)
    ms = torch.empty_like(mp)
    if fused:
        h.prepare_batch(seeds, fanouts, rng_seed, hops, sizes, unique, inverse, n_unique, out, mp, mi, ms, stats)
        h.sync()
    else:
        h.sample(seeds, fanouts, rng_seed, hops, sizes)
        h.sync()
        parts = [seeds] + [hops[k].flat[:int(sizes[2 * k + 1])] for k in range(K)]
        cat = torch.cat(parts)
        h.dedup(cat, unique, inverse, n_unique)
        h.sync()
        h.gather(unique, out, mp, mi, ms, stats, n_ids=int(n_unique[0]))
        h.sync()
    res = {"hops": []}
    for k in range(K):
        nf, nfl = int(sizes[2 * k]), int(sizes[2 * k + 1])
        res["hops"].append((hops[k].frontier[:nf].cpu().numpy(), hops[k].indptr[:nf + 1].cpu().numpy(),
                            hops[k].flat[:nfl].cpu().numpy()))
    U = int(n_unique[0])
    n_cat = B + sum(int(sizes[2 * k + 1]) for k in range(K))
    nm = int(stats[3])
    res.update(unique=unique[:U].cpu().numpy(), inverse=inverse[:n_cat].cpu().numpy(), stats=stats.numpy().copy(),
               miss_pos=mp[:nm].cpu().numpy(), miss_id=mi[:nm].cpu().numpy(), miss_slot=ms[:nm].cpu().numpy(),
               out_before_miss=out[:U].cpu().numpy())
    if serve_misses:
        h.gather_miss(mp, ms, mp.numel(), stats[3:4], out)
        h.sync()
        res["out"] = out[:U].cpu().numpy()
    return res


def lanes_in_flight(helios, offsets, indices, order, n_hbm, n_host, row_bytes, tabs_dev, batch, fanouts, jobs,
                    n_lanes: int = 3, recorded: bool = True, per_lane: int = 1, tune=None):
    """bench.py's launch configuration: n_lanes contexts, each on its own stream with (recorded=True) a
    recorded batch per buffer set, sharing the graph and the cache tables.  per_lane == 1: a lane is
    synchronised before it gets its next batch, and the miss list is served (result key "out").
    per_lane == 2: every lane has two buffer sets, a batch is queued behind the lane's running one and
    each is waited for by helios_plan_wait; misses are not served (result key "out_before_miss").
    jobs: list of (seeds on the GPU, rng_seed).  Returns one result dict per job, as gpu_path does."""
    import torch as T
    assert per_lane == 1 or recorded
    dev = offsets.device
    lanes, units = [], []
    for _ in range(n_lanes):
        ctx = helios.Helios(dev.index or 0, stream=T.cuda.Stream(device=dev))
        ctx.csr_load(offsets, indices)
        ctx.cache_build(order, n_hbm, n_host, row_bytes, *tabs_dev)
        ctx.sync()
        if tune is not None:
            tune(ctx)                             # launch parameters, set before anything is recorded
        lanes.append(ctx)
    for w in range(per_lane):
        for ctx in lanes:
            hops = helios.alloc_hops(batch, fanouts, dev)
            cap = batch + sum(hb.flat.numel() for hb in hops)
            ctx.reserve(cap)
            units.append(dict(ctx=ctx, hops=hops, unique=T.empty(cap, dtype=T.int32, device=dev),
                              inverse=T.empty(cap, dtype=T.int32, device=dev),
                              out=T.full((cap, row_bytes), SENTINEL, dtype=T.uint8, device=dev),
                              mp=T.empty(cap, dtype=T.int32, device=dev), mi=T.empty(cap, dtype=T.int32, device=dev),
                              ms=T.empty(cap, dtype=T.int32, device=dev),
                              sizes=T.zeros(2 * len(fanouts), dtype=T.int64).pin_memory(),
                              nu=T.zeros(1, dtype=T.int64).pin_memory(), stats=T.zeros(4, dtype=T.int64).pin_memory(),
                              plan=None))
    T.cuda.synchronize()
    if recorded:
        for bf in units:
            bf["plan"] = bf["ctx"].plan_create(batch, fanouts, bf["hops"], bf["sizes"], bf["unique"], bf["inverse"],
                                               bf["nu"], bf["out"], bf["mp"], bf["mi"], bf["ms"], bf["stats"])
        T.cuda.synchronize()
    K = len(fanouts)

    def collect(bf):
        if per_lane > 1:
            bf["plan"].wait()
        else:
            bf["ctx"].sync()
        sizes, U, nm = bf["sizes"], int(bf["nu"][0]), int(bf["stats"][3])
        res = {"hops": []}
        for k in range(K):
            nf, nfl = int(sizes[2 * k]), int(sizes[2 * k + 1])
            hb = bf["hops"][k]
            res["hops"].append((hb.frontier[:nf].cpu().numpy(), hb.indptr[:nf + 1].cpu().numpy(), hb.flat[:nfl].cpu().numpy()))
        n_cat = batch + sum(int(sizes[2 * k + 1]) for k in range(K))
        res.update(unique=bf["unique"][:U].cpu().numpy(), inverse=bf["inverse"][:n_cat].cpu().numpy(),
                   stats=bf["stats"].numpy().copy(), miss_pos=bf["mp"][:nm].cpu().numpy(),
                   miss_id=bf["mi"][:nm].cpu().numpy(), miss_slot=bf["ms"][:nm].cpu().numpy())
        res["out" if per_lane == 1 else "out_before_miss"] = bf["out"][:U].cpu().numpy()
        return res

    results = [None] * len(jobs)
    n_units = len(units)
    for j, (seeds, rs) in enumerate(jobs):
        bf = units[j % n_units]
        if j >= n_units:
            results[j - n_units] = collect(bf)
            with T.cuda.stream(T.cuda.ExternalStream(bf["ctx"]._stream_ptr, device=dev)):
                bf["out"].fill_(SENTINEL)                 # in stream order: the lane may be running its other set
        if recorded:
            bf["plan"].launch(seeds, rs)
        else:
            bf["ctx"].prepare_batch(seeds, fanouts, rs, bf["hops"], bf["sizes"], bf["unique"], bf["inverse"], bf["nu"],
                                    bf["out"], bf["mp"], bf["mi"], bf["ms"], bf["stats"])
        if per_lane == 1:
            bf["ctx"].gather_miss(bf["mp"], bf["ms"], bf["mp"].numel(), bf["stats"][3:4], bf["out"])
    for j in range(max(0, len(jobs) - n_units), len(jobs)):
        results[j] = collect(units[j % n_units])
    for ctx in lanes:
        ctx.sync()
    for bf in units:
        if bf["plan"] is not None:
            bf["plan"].destroy()
    for ctx in lanes:
        ctx.close()
    return results


def gangs_in_flight(helios, offsets, indices, order, n_hbm, n_host, row_bytes, tabs_dev, batch, fanouts, jobs,
                    members: int = 3, n_gangs: int = 2, tune=None, served: bool = False):
    """bench.py's gang configuration: n_gangs streams, on each a gang of `members` contexts with one buffer set
    per member; the jobs go out `members` at a time, to the gangs in turn, and a gang is waited for
    (helios_gang_wait) before it gets its next batches.  Misses are not served (result key "out_before_miss"), unless
    served: then every batch serves its own (HELIOS_PARAM_SERVE_MISSES; result key "out").
    jobs: list of (seeds on the GPU, rng_seed), a multiple of `members`.  Returns one result dict per job."""
    import torch as T
    assert len(jobs) % members == 0
    dev = offsets.device
    gangs = []
    K = len(fanouts)
    for _ in range(n_gangs):
        st = T.cuda.Stream(device=dev)
        ctxs, sets = [], []
        for _ in range(members):
            ctx = helios.Helios(dev.index or 0, stream=st)
            ctx.csr_load(offsets, indices)
            ctx.cache_build(order, n_hbm, n_host, row_bytes, *tabs_dev)
            if tune is not None:
                tune(ctx)
            if served:
                ctx.set_param(helios.PARAM_SERVE_MISSES, 1)
            hops = helios.alloc_hops(batch, fanouts, dev)
            cap = batch + sum(hb.flat.numel() for hb in hops)
            ctx.reserve(cap)
            ctx.sync()
            ctxs.append(ctx)
            sets.append(helios.BatchBuffers(
                hops=hops, sizes=T.zeros(2 * K, dtype=T.int64).pin_memory(), unique=T.empty(cap, dtype=T.int32, device=dev),
                inverse=T.empty(cap, dtype=T.int32, device=dev), n_unique=T.zeros(1, dtype=T.int64).pin_memory(),
                out=T.full((cap, row_bytes), SENTINEL, dtype=T.uint8, device=dev),
                miss_pos=T.empty(cap, dtype=T.int32, device=dev), miss_id=T.empty(cap, dtype=T.int32, device=dev),
                miss_slot=T.empty(cap, dtype=T.int32, device=dev), stats=T.zeros(4, dtype=T.int64).pin_memory()))
        T.cuda.synchronize()
        gangs.append(dict(stream=st, ctxs=ctxs, sets=sets, gang=helios.Gang(ctxs, batch, fanouts, sets), jobs=None))
    T.cuda.synchronize()

    def collect(gd):
        st = gd["gang"].wait()
        assert all(code == 0 for code in st), st
        res = []
        for bs in gd["sets"]:
            sizes, U, nm = bs.sizes, int(bs.n_unique[0]), int(bs.stats[3])
            r = {"hops": []}
            for k in range(K):
                nf, nfl = int(sizes[2 * k]), int(sizes[2 * k + 1])
                hb = bs.hops[k]
                r["hops"].append((hb.frontier[:nf].cpu().numpy(), hb.indptr[:nf + 1].cpu().numpy(), hb.flat[:nfl].cpu().numpy()))
            n_cat = batch + sum(int(sizes[2 * k + 1]) for k in range(K))
            r.update(unique=bs.unique[:U].cpu().numpy(), inverse=bs.inverse[:n_cat].cpu().numpy(),
                     stats=bs.stats.numpy().copy(), miss_pos=bs.miss_pos[:nm].cpu().numpy(),
                     miss_id=bs.miss_id[:nm].cpu().numpy(), miss_slot=bs.miss_slot[:nm].cpu().numpy())
            r["out" if served else "out_before_miss"] = bs.out[:U].cpu().numpy()
            res.append(r)
        return res

    results = [None] * len(jobs)
    for r in range(len(jobs) // members):
        gd = gangs[r % n_gangs]
        if gd["jobs"] is not None:
            first = gd["jobs"]
            results[first:first + members] = collect(gd)
            with T.cuda.stream(gd["stream"]):
                for bs in gd["sets"]:
                    bs.out.fill_(SENTINEL)
        mine = jobs[r * members:(r + 1) * members]
        gd["gang"].launch([j[0] for j in mine], [j[1] for j in mine])
        gd["jobs"] = r * members
    for gd in gangs:
        if gd["jobs"] is not None:
            first = gd["jobs"]
            results[first:first + members] = collect(gd)
    for gd in gangs:
        gd["gang"].destroy()
        for ctx in gd["ctxs"]:
            ctx.close()
    return results


def oracle_path(oracle, off, idx, seeds, fanouts, rng_seed, rank, n_hbm, n_host, hbm_tab, host_tab, standin_tab,
                row_bytes):
    hops = oracle.sample(off, idx, seeds, fanouts, rng_seed)
    cat = np.concatenate([np.asarray(seeds, np.int32)] + [fl for _, _, fl in hops])
    uniq, inv = oracle.dedup(off.size - 1, cat)
    out = np.full((uniq.size, row_bytes), SENTINEL, np.uint8)
    mp, mi, ms, stats = oracle.gather(uniq, rank, n_hbm, n_host, hbm_tab, host_tab, out)
    before = out.copy()
    oracle.gather_miss(mp, ms, standin_tab, out)
    return dict(hops=hops, unique=uniq, inverse=inv, stats=stats, miss_pos=mp, miss_id=mi, miss_slot=ms,
                out_before_miss=before, out=out)


def assert_same(got, want):
    assert len(got["hops"]) == len(want["hops"])
    for k, (g, w) in enumerate(zip(got["hops"], want["hops"])):
        for name, a, b in zip(("frontier", "indptr", "flat"), g, w):
            assert a.shape == b.shape, f"hop {k} {name}: {a.shape} vs {b.shape}"
            assert np.array_equal(a, b), f"hop {k} {name} differs"
    for key in ("unique", "inverse", "stats", "miss_pos", "miss_id", "miss_slot", "out_before_miss", "out"):
        if key in got and key in want:
            assert got[key].shape == want[key].shape, f"{key}: {got[key].shape} vs {want[key].shape}"
            assert np.array_equal(got[key], want[key]), f"{key} differs"
