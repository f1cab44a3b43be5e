"""Benchmark of the Helios mini-batch preparation path on one MI355X.

A step is one pass of the whole path (k-hop sampling, de-duplication, cache lookup, gather of
both cached tiers, miss list: a recorded helios_prepare_batch) over one batch of seeds of a
synthetic workload whose graph, feature tables and seeds are resident before the timed region
(graph, cache map and HBM tier in HBM; host tier and storage stand-in in pinned host memory,
where the method keeps them).  In the timed region the batches run in gangs: the mini-batches
of four contexts share every launch (helios_gang_*), three such gangs in flight; the same
K steps by separate recordings on three streams are reported under "lanes".  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..4] [--hbm-frac P]

Default workload: benchmark configs[3] (50 M nodes, 1 B edges, 2 KB rows, 3 hops), the largest
one-GPU workload; the same line carries a shorter block for configs[2] (the paper's PA shape)
under "also" unless --also -1.

    python bench.py --only roofline ...   runs only the set-up and the region the two "roofline"
                                          objects come from (what profiles/kernel_trace_* trace)
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
ROLE_NAMES = {1: "sample", 2: "compact_hop", 3: "compact_lookup", 4: "copy_host", 5: "copy_hbm", 6: "inverse", 7: "copy_standin"}


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def optional(what: str, fn):
    """A secondary region of the benchmark: if it raises, the line still carries the headline figures."""
    try:
        return fn()
    except Exception as e:                      # noqa: BLE001 (reported in the line)
        log(f"{what} failed: {e!r}")
        return {"error": repr(e)}


def measure_host_link(torch, gib: float = 1.0) -> float:
    """Pinned host -> device copy rate in GB/s (best of 5), the denominator of the host-tier gather."""
    n = int(gib * (1 << 30))
    src = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    src.fill_(1)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    best = 0.0
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dst.copy_(src, non_blocking=True)
        e1.record()
        e1.synchronize()
        best = max(best, n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    return best


def measure_plain_copy(torch, h) -> float:
    """A plain 1 GiB device copy with the row copy's accesses (known traffic: 1 GiB read + 1 GiB written), GB/s."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    src.fill_(3)
    best = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        h.calibration_copy(src, dst)
        e1.record()
        e1.synchronize()
        best = max(best, 2.0 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    return best


def large_list(torch, helios, dev, rb: int, table_gb: float, seed: int):
    """The HBM-tier copy where it is bound by bandwidth: helios_gather of 1 M random IDs (fewer for rows
    above 1 KB) that all hit an HBM tier of table_gb, far larger than the last-level cache; the copy kernel
    is launched with HIP events that take its own begin and end (as a kernel trace reports them)."""
    n_tab = int(table_gb * 1e9) // rb
    n_ids = 1_000_000 if rb <= 1024 else 500_000
    if n_tab < 2 * n_ids:
        return None
    table = torch.empty((n_tab, rb), dtype=torch.uint8, device=dev)
    table.fill_(5)
    order_l = torch.arange(n_tab, device=dev, dtype=torch.int32)       # the IDs are random, so are the rows
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    ids = torch.randint(0, n_tab, (n_ids,), device=dev, dtype=torch.int32, generator=gen)
    out = torch.empty((n_ids, rb), dtype=torch.uint8, device=dev)
    mp = torch.empty(16, dtype=torch.int32, device=dev)
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    ctx = helios.Helios(0, stream=torch.cuda.Stream(device=dev))
    ctx.csr_load(torch.zeros(n_tab + 1, dtype=torch.int64, device=dev), torch.zeros(1, dtype=torch.int32, device=dev))
    ctx.cache_build(order_l, n_tab, 0, rb, table, None, None)
    ctx.set_timing(2)
    times = []
    for _ in range(7):
        ctx.gather(ids, out, mp, mp.clone(), mp.clone(), stats)
        ctx.sync()
        times.append(ctx.gather_times()[2])
    ctx.close()
    ms = statistics.median(times[2:])
    gbs = 2.0 * n_ids * rb / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    return {"rows": n_ids, "row_bytes": rb, "table_GB": n_tab * rb / 1e9, "kernel_us": ms * 1e3, "achieved": gbs,
            "frac": gbs / HBM_PEAK_GBS,
            "note": "gather_rows_kernel alone on a list long enough to be bound by bandwidth; median of 5 launches, HIP "
                    "events on the kernel"}


def counted_traffic(rb: int, rows_per_launch: float):
    """HBM bytes per launch of the HBM-tier copy from the committed counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
    scaled by the calibration copy): those runs are taken on a long list of rows of the same size (the profiler does not
    survive the set-up of the large workloads), so the counted bytes per row are scaled to this launch's row count."""
    name = {2048: "hbm_traffic_and_l2_gather_rows_large_list_2KB_rows.txt",
            512: "hbm_traffic_and_l2_gather_rows_large_list_512B_rows.txt"}.get(rb)
    path = os.path.join(ROOT, "profiles", name) if name else None
    if not path or not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("TRAFFIC_JSON:"):
            try:
                t = json.loads(line[len("TRAFFIC_JSON:"):])
            except Exception:
                return None
            k = rows_per_launch / t["rows_per_launch"]
            return {"unit": "bytes per launch of the HBM-tier row copy", "fetched": t["fetched"] * k, "written": t["written"] * k,
                    "algorithmic_read": rows_per_launch * (rb + 8), "algorithmic_written": rows_per_launch * rb,
                    "rows_per_launch": rows_per_launch,
                    "source": "counted on %d rows of %d B with the same kernel (profiles/%s), scaled to this launch's rows"
                              % (t["rows_per_launch"], rb, name)}
    return None


def run_workload(args, cfg: int, hbm_frac, K: int, Wm: int, link_gbs: float, full: bool):
    """Sets workload `cfg` up, runs the timed regions, returns the result dict (full: with every region and the
    CPU-oracle leg; else the headline figures only)."""
    import numpy as np
    import torch

    from paper_2310_00837_amd import helios, workload as W
    dev = torch.device("cuda", 0)
    sp = W.spec(cfg, hbm_frac)
    only = args.only

    # ---------------- inputs (untimed)
    t0 = time.time()
    big = sp.n_nodes > 5_000_000
    gen_dev = dev if big else "cpu"
    g = W.make_graph(sp, args.seed, gen_dev, progress=log if big else None)
    log(f"{sp.name}: N={g.n_nodes} E={g.n_edges} generated on {gen_dev} in {time.time() - t0:.1f}s")
    offsets, indices, order = g.offsets.to(dev), g.indices.to(dev), g.order.to(dev)
    g.offsets, g.indices, g.order, g.perm_seed = offsets, indices, order, g.perm_seed.to(dev)
    cache_order = "in-degree, ties by ID (BASELINE.json)"
    if args.presample_batches:
        # Sec. 3.2.2 "Cache Initialization": an epoch of pre-sampling on the GPU counts every vertex's hotness, the
        # GPU sorts the vertices by it, the hottest fill the GPU tier and the next the CPU tier
        Bp = min(sp.batch, g.n_nodes)
        per_epoch = -(-max(Bp, int(sp.train_frac * g.n_nodes)) // Bp)
        nb = per_epoch if args.presample_batches < 0 else args.presample_batches
        hp = helios.Helios(0)
        hp.csr_load(offsets, indices)
        hops_p = helios.alloc_hops(Bp, sp.fanouts, dev)
        cap_p = Bp + sum(hb.flat.numel() for hb in hops_p)
        uniq_p = torch.empty(cap_p, dtype=torch.int32, device=dev)
        sizes_p = torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory()
        nu_p = torch.zeros(1, dtype=torch.int64).pin_memory()
        counts = torch.zeros(g.n_nodes, dtype=torch.int32, device=dev)
        for b in range(nb):
            sd = W.seed_batch(sp, g, b, epoch=1).to(dev)         # another shuffle of the train split than the timed batches
            hp.sample(sd, sp.fanouts, W.batch_rng_seed(args.seed + 1, b), hops_p, sizes_p)
            hp.sync()
            cat = torch.cat([sd] + [hops_p[k].flat[:int(sizes_p[2 * k + 1])] for k in range(len(sp.fanouts))])
            hp.dedup(cat, uniq_p, None, nu_p)
            hp.hotness_add(uniq_p, uniq_p.numel(), nu_p, counts)
        order = torch.empty(g.n_nodes, dtype=torch.int32, device=dev)
        hp.hotness_order(counts, order)
        hp.sync()
        hp.close()
        g.order = order
        cache_order = f"pre-sampling hotness over {nb} batches (helios_hotness_add / helios_hotness_order)"
        log(f"cache order: {cache_order}; {int((counts > 0).sum())} nodes seen")
        del counts, uniq_p, hops_p
    t1 = time.time()
    pinned_bufs = []

    def pinned_exact(shape, dtype):          # torch's pinned allocator rounds 28 GB up to 32 GB and keeps it; this one does not
        pinned_bufs.append(helios.pinned_empty(shape, dtype))
        return pinned_bufs[-1].tensor

    tiers = W.make_tiers(sp, g, dev, progress=log if big else None, pinned_empty=pinned_exact)
    log(f"tiers: hbm {tiers.n_hbm} host {tiers.n_host} stand-in {tiers.n_rest} rows x {sp.row_bytes} B "
        f"filled in {time.time() - t1:.1f}s")

    h = helios.Helios(0)                     # the default stream: set-up and the parity check only
    copy_gbs = measure_plain_copy(torch, h)
    log(f"plain device copy (1 GiB, read+write): {copy_gbs:.0f} GB/s")
    h.csr_load(offsets, indices)
    h.cache_build(order, tiers.n_hbm, tiers.n_host, sp.row_bytes, tiers.hbm, tiers.host, tiers.standin)
    h.sync()

    B = min(sp.batch, g.n_nodes)
    n_batches = K + Wm
    seeds = [W.seed_batch(sp, g, b).to(dev) for b in range(n_batches)]
    rng_seeds = [W.batch_rng_seed(args.seed, b) for b in range(n_batches)]
    rb = sp.row_bytes
    n_hops = len(sp.fanouts)

    class Buffers:
        """Caller-owned outputs of one mini-batch, and the recordings that write to them."""

        def __init__(self, cap):
            self.hops = helios.alloc_hops(B, sp.fanouts, dev)
            self.unique = torch.empty(cap, dtype=torch.int32, device=dev)
            self.inverse = torch.empty(cap, dtype=torch.int32, device=dev)
            self.out = torch.empty((cap, rb), dtype=torch.uint8, device=dev)
            self.mp = torch.empty(cap, dtype=torch.int32, device=dev)
            self.mi, self.ms = torch.empty_like(self.mp), torch.empty_like(self.mp)
            self.sizes = torch.zeros(2 * n_hops, dtype=torch.int64).pin_memory()
            self.n_unique = torch.zeros(1, dtype=torch.int64).pin_memory()
            self.stats = torch.zeros(4, dtype=torch.int64).pin_memory()
            # zero-copy numpy views of the pinned result words: reading them costs the host almost nothing
            self.stats_np, self.sizes_np = self.stats.numpy(), self.sizes.numpy()
            self.plans = {}

        def args(self):
            return (self.hops, self.sizes, self.unique, self.inverse, self.n_unique, self.out, self.mp, self.mi, self.ms,
                    self.stats)

    class Lane:
        """One library context on its own stream.  It has two buffer sets: one mini-batch of the lane runs
        while the next is already queued behind it on the stream."""

        def __init__(self, ctx, stream):
            self.h, self.stream = ctx, stream
            cap = width = B                      # seeds + the largest possible sample lists
            for f in sp.fanouts:
                width *= f
                cap += width
            self.h.reserve(cap)
            self.cap = cap
            self.sets = [Buffers(cap) for _ in range(max(1, args.per_lane))]
            self.queue = None

        def record(self) -> None:
            """One recording (HIP graph) of the whole-path call per buffer set, and one with the roles timed.  A
            directly launched batch comes first: the library sizes the grid of the HBM-tier copy from the hit counts
            of the context's last finished batch, and a recording keeps the grid it was made with."""
            self.h.prepare_batch(seeds[0], sp.fanouts, rng_seeds[0], *self.sets[0].args())
            self.h.sync()
            for bs in self.sets:
                bs.plans[0] = self.h.plan_create(B, sp.fanouts, *bs.args())
            self.h.set_timing(1)
            self.sets[0].plans[1] = self.h.plan_create(B, sp.fanouts, *self.sets[0].args())
            self.h.set_timing(0)

        def record_with_queue(self) -> None:
            """A miss queue of this lane's own and a recording in which the batch submits its misses to it."""
            nq = args.missq_queues
            self.queue = helios.MissQueue(self.h, nq, (self.cap + nq - 1) // nq, args.missq_threads)
            self.queue.attach()
            self.sets[0].plans["queue"] = self.h.plan_create(B, sp.fanouts, *self.sets[0].args())

        def drop_queue(self) -> None:
            self.sets[0].plans.pop("queue").destroy()
            self.queue.destroy()
            self.queue = None

    lanes = []
    for _ in range(max(1, args.depth)):
        st = torch.cuda.Stream(device=dev)
        ctx = helios.Helios(0, stream=st)
        ctx.csr_load(offsets, indices)
        ctx.cache_build(order, tiers.n_hbm, tiers.n_host, rb, tiers.hbm, tiers.host, tiers.standin)
        ctx.sync()
        lanes.append(Lane(ctx, st))
    torch.cuda.synchronize()
    for ln in lanes:
        ln.record()
    torch.cuda.synchronize()
    D, P = len(lanes), max(1, args.per_lane)

    def new_acc():
        return dict(hbm_rows=0, host_rows=0, miss=0, unique=0, raw=0)

    def tally(acc, bs):
        st = bs.stats_np
        acc["hbm_rows"] += int(st[1])
        acc["host_rows"] += int(st[2])
        acc["miss"] += int(st[3])
        acc["unique"] += int(st[0])
        acc["raw"] += int(bs.sizes_np[1::2].sum())

    def region_queued(first: int, count: int):
        """`count` steps on D lanes with P buffer sets each: a batch is queued behind the lane's running one and
        each batch is waited for by itself (helios_plan_wait).  Returns (seconds, sums)."""
        acc = new_acc()
        units = [(ln, w) for w in range(P) for ln in lanes]      # lane 0 set 0, lane 1 set 0, ..., lane 0 set 1, ...
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for k in range(count):
            ln, w = units[k % len(units)]
            bs = ln.sets[w]
            if k >= len(units):
                bs.plans[0].wait()
                tally(acc, bs)
            bs.plans[0].launch(seeds[first + k], rng_seeds[first + k])
        for k in range(max(0, count - len(units)), count):
            ln, w = units[k % len(units)]
            ln.sets[w].plans[0].wait()
            tally(acc, ln.sets[w])
        for ln in lanes:
            ln.h.sync()
        torch.cuda.synchronize()
        return time.perf_counter() - t_begin, acc

    def region_serial(first: int, count: int, depth: int, serve):
        """`count` steps, lane b % depth takes batch b on its first buffer set and is synchronised (helios_sync)
        before it is reused.  serve: None, "zero-copy" (helios_gather_miss) or "queue" (the asynchronous miss
        queue).  Returns (seconds, sums)."""
        acc = new_acc()
        use = lanes[:depth]

        def launch(ln, b):
            bs = ln.sets[0]
            if serve == "queue":
                bs.plans["queue"].launch(seeds[b], rng_seeds[b])
                ln.queue.complete(bs.out)
                return
            bs.plans[0].launch(seeds[b], rng_seeds[b])
            if serve == "zero-copy":
                ln.h.gather_miss(bs.mp, bs.ms, bs.mp.numel(), bs.stats[3:4], bs.out)

        def retire(ln):
            ln.h.sync()
            tally(acc, ln.sets[0])

        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for k in range(count):
            ln = use[k % depth]
            if k >= depth:
                retire(ln)
            launch(ln, first + k)
        for k in range(max(0, count - depth), count):
            retire(use[k % depth])
        torch.cuda.synchronize()
        return time.perf_counter() - t_begin, acc

    def repeated(fn, *a):
        """The K-step region several times over: (median seconds, sums of the median run, all seconds)."""
        runs = [fn(*a) for _ in range(max(1, args.repeats))]
        runs.sort(key=lambda r: r[0])
        mid = runs[len(runs) // 2]
        return mid[0], mid[1], [r[0] for r in runs]

    def region_roofline(count: int):
        """One mini-batch in flight, launched directly with the two tier copies as kernels of their own
        (HELIOS_PARAM_SPLIT_COPIES), each carrying HIP events that take the kernel's own begin and end: what a
        kernel trace of this region shows per launch.  A second pass takes the same kernels' in-kernel span
        (first workgroup start to last end, device clock)."""
        ln = lanes[0]
        bs = ln.sets[0]
        ln.h.set_param(helios.PARAM_SPLIT_COPIES, 1)
        res = {}
        for level, keys in ((2, ("hbm_event_ms", "host_event_ms")), (1, ("hbm_span_ms", "host_span_ms"))):
            ln.h.set_timing(level)
            acc = new_acc()
            sums = [0.0, 0.0]
            for k in range(Wm + count):
                b = k % n_batches
                ln.h.prepare_batch(seeds[b], sp.fanouts, rng_seeds[b], *bs.args())
                ln.h.sync()
                if k < Wm:
                    continue
                t = ln.h.gather_times()
                sums[0] += t[2] if level == 2 else t[0]
                sums[1] += t[3] if level == 2 else t[1]
                tally(acc, bs)
            res[keys[0]], res[keys[1]] = sums[0] / count, sums[1] / count
            res["hbm_rows"], res["host_rows"] = acc["hbm_rows"] / count, acc["host_rows"] / count
        ln.h.set_timing(0)
        ln.h.set_param(helios.PARAM_SPLIT_COPIES, 0)
        return res

    def region_roles(count: int):
        """One mini-batch in flight, the recorded (fused) batch with every role timed by the device clock: average
        span per role, and where the host-tier copies sit relative to the sampling passes."""
        ln = lanes[0]
        bs = ln.sets[0]
        spans, first_link_start, last_sample_end, batch_span = {}, 0.0, 0.0, 0.0
        for k in range(count):
            b = (Wm + k) % n_batches
            bs.plans[1].launch(seeds[b], rng_seeds[b])
            ln.h.sync()
            roles, per_us = ln.h.batch_ticks()
            live = [r for r in roles if r[4] > r[3]]
            if not live:
                continue
            t0_ = min(r[3] for r in live)
            for kind, stage, wgs, a, z in live:
                spans.setdefault(f"{ROLE_NAMES.get(kind, kind)}_{stage}", []).append((z - a) / per_us)
            links = [r for r in live if r[0] == helios.ROLE_COPY_HOST]
            samples = [r for r in live if r[0] == helios.ROLE_SAMPLE]
            if links and samples:
                first_link_start += (min(r[3] for r in links) - t0_) / per_us
                last_sample_end += (max(r[4] for r in samples) - t0_) / per_us
            batch_span += (max(r[4] for r in live) - t0_) / per_us
        return {"avg_us_per_role": {k: sum(v) / len(v) for k, v in spans.items()},
                "first_host_tier_copy_starts_at_us": first_link_start / count,
                "last_sampling_pass_ends_at_us": last_sample_end / count,
                "batch_span_us": batch_span / count,
                "note": "device clock, one mini-batch in flight, recorded batch; times from the batch's first workgroup"}

    class GangOnStream:
        """A gang of `members` contexts on one stream, one buffer set per member: the batches of the members go
        through the same launches.  Every member runs one directly launched batch first (see Lane.record)."""

        def __init__(self, members: int, cap: int, host_blocks: int, serve_misses: bool = False, timed: bool = False):
            self.stream = torch.cuda.Stream(device=dev)
            self.ctxs, self.sets = [], []
            for _ in range(members):
                ctx = helios.Helios(0, stream=self.stream)
                ctx.csr_load(offsets, indices)
                ctx.cache_build(order, tiers.n_hbm, tiers.n_host, rb, tiers.hbm, tiers.host, tiers.standin)
                if host_blocks > 0:
                    ctx.set_param(helios.PARAM_HOST_GATHER_BLOCKS, host_blocks)
                if serve_misses:
                    ctx.set_param(helios.PARAM_SERVE_MISSES, 1)
                if timed:
                    ctx.set_timing(1)
                ctx.reserve(cap)
                bs = Buffers(cap)
                ctx.prepare_batch(seeds[0], sp.fanouts, rng_seeds[0], *bs.args())
                ctx.sync()
                self.ctxs.append(ctx)
                self.sets.append(bs)
            self.gang = helios.Gang(self.ctxs, B, sp.fanouts, [
                helios.BatchBuffers(hops=bs.hops, sizes=bs.sizes, unique=bs.unique, inverse=bs.inverse, n_unique=bs.n_unique,
                                    out=bs.out, miss_pos=bs.mp, miss_id=bs.mi, miss_slot=bs.ms, stats=bs.stats)
                for bs in self.sets])
            self.live = 0                      # batches of the gang's last launch that count

        def close(self) -> None:
            self.gang.destroy()
            for ctx in self.ctxs:
                ctx.close()

    gangs = []

    def region_gangs(first: int, count: int):
        """`count` steps by gangs: the batches go out M at a time, to the gangs in turn (each on its own stream); a gang
        is waited for (helios_gang_wait) before it gets its next batches.  If M does not divide count, the last launch is
        filled up with batches that are run but not counted.  Returns (seconds, sums)."""
        acc = new_acc()
        M = len(gangs[0].ctxs)
        rounds = (count + M - 1) // M
        for gd in gangs:
            gd.live = 0
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        for r in range(rounds):
            gd = gangs[r % len(gangs)]
            if gd.live:
                gd.gang.wait()
                for bs in gd.sets[:gd.live]:
                    tally(acc, bs)
            ks = [min(r * M + m, count - 1) for m in range(M)]
            gd.gang.launch([seeds[first + k] for k in ks], [rng_seeds[first + k] for k in ks])
            gd.live = min(M, count - r * M)
        for r in range(max(0, rounds - len(gangs)), rounds):
            gd = gangs[r % len(gangs)]
            if gd.live:
                gd.gang.wait()
                for bs in gd.sets[:gd.live]:
                    tally(acc, bs)
                gd.live = 0
        torch.cuda.synchronize()
        return time.perf_counter() - t_begin, acc

    def region_gang_roles(count: int, members: int):
        """One gang in flight, its roles timed by the device clock (timing level 1 is part of the recording): per role
        the average span in one member and the span over all members (first start to last end), and the whole gang."""
        gd = GangOnStream(members, lanes[0].cap, args.gang_host_blocks, timed=True)
        per_member, over_gang, whole = {}, {}, 0.0
        for k in range(count):
            ks = [(Wm + k * members + m) % n_batches for m in range(members)]
            gd.gang.launch([seeds[b] for b in ks], [rng_seeds[b] for b in ks])
            gd.gang.wait()
            per_us, live = 1.0, []
            for ctx in gd.ctxs:
                roles, per_us = ctx.batch_ticks()
                live.append({f"{ROLE_NAMES.get(kind, kind)}_{stage}": (a, z) for kind, stage, wgs, a, z in roles if z > a})
            keys = sorted(set(k_ for lv in live for k_ in lv))
            t_first = min(a for lv in live for a, _ in lv.values())
            whole += (max(z for lv in live for _, z in lv.values()) - t_first) / per_us
            for key in keys:
                spans = [lv[key] for lv in live if key in lv]
                per_member.setdefault(key, []).append(sum(z - a for a, z in spans) / len(spans) / per_us)
                over_gang.setdefault(key, []).append((max(z for _, z in spans) - min(a for a, _ in spans)) / per_us)
        gd.close()
        return {"members": members, "avg_us_per_role_in_one_member": {k_: sum(v) / len(v) for k_, v in per_member.items()},
                "avg_us_per_role_over_the_gang": {k_: sum(v) / len(v) for k_, v in over_gang.items()},
                "gang_span_us": whole / count,
                "note": "device clock, one gang in flight (its members' mini-batches in the same launches)"}

    result = {"dtype": "int32 ids / byte rows (" + ("fp32" if sp.dtype == torch.float32 else "fp16") + " features)",
              "config": {"workload": f"BASELINE.json configs[{cfg}] {sp.name}", "n_nodes": g.n_nodes, "n_edges": g.n_edges,
                         "batch": B, "fanouts": sp.fanouts, "row_bytes": rb,
                         "tier_rows": [tiers.n_hbm, tiers.n_host, tiers.n_rest], "seed": args.seed,
                         "cache_order": cache_order,
                         "step": "helios_plan_launch (recorded helios_prepare_batch: sample, dedup, lookup, HBM+host gather, "
                                 "miss list) + one helios_plan_wait per batch, %d contexts on %d streams, %d mini-batches "
                                 "queued on each; median of %d runs of the K steps" % (D, D, P, args.repeats)}}

    # ---------------- the roofline region: the two row copies as kernels of their own
    roof = region_roofline(min(K, 100))
    hbm_gbs = 2.0 * roof["hbm_rows"] * rb / (roof["hbm_event_ms"] * 1e-3) / 1e9 if roof["hbm_event_ms"] > 0 else 0.0
    host_gbs = 1.0 * roof["host_rows"] * rb / (roof["host_event_ms"] * 1e-3) / 1e9 if roof["host_event_ms"] > 0 else 0.0
    result["roofline"] = {
        "kernel": "gather_rows_kernel<.., 0> (HBM-tier row copy)", "bound": "hbm", "achieved": hbm_gbs, "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": counted_traffic(rb, roof["hbm_rows"]),
        "avg_kernel_us": roof["hbm_event_ms"] * 1e3, "in_kernel_span_us": roof["hbm_span_ms"] * 1e3,
        "rows_per_launch": roof["hbm_rows"], "bytes_per_row": 2 * rb,
        "timer": "HIP events carried by the kernel launch (the kernel's own begin and end, as rocprofv3 --kernel-trace "
                 "reports them); in_kernel_span_us: first workgroup start to last end by the device clock",
        "region": "%d mini-batches, one in flight, launched directly with HELIOS_PARAM_SPLIT_COPIES (the tier copies as "
                  "kernels of their own, as `bench.py --only roofline` runs them under the profiler)" % min(K, 100),
        "plain_copy_GBs_on_this_box": copy_gbs}
    result["roofline_host_link"] = {
        "kernel": "gather_rows_kernel<.., 1> (host-tier row copy)", "bound": "host_link", "achieved": host_gbs, "peak": link_gbs,
        "unit": "GB/s", "frac": host_gbs / link_gbs if link_gbs > 0 else None,
        "peak_source": "given on the command line" if args.link_gbs else "pinned H2D copy measured in this run",
        "avg_kernel_us": roof["host_event_ms"] * 1e3, "in_kernel_span_us": roof["host_span_ms"] * 1e3,
        "rows_per_launch": roof["host_rows"], "bytes_per_row": rb}
    if only == "roofline":
        for ln in lanes:
            for bs in ln.sets:
                for pl in bs.plans.values():
                    pl.destroy()
            ln.h.close()
        h.close()
        return result

    # ---------------- the timed region: W warm-up steps, then K whole steps (S1-S5)
    # by lanes: D contexts on D streams, P mini-batches queued on each
    region_queued(0, Wm)
    elapsed, acc, all_runs = repeated(region_queued, Wm, K)
    lanes_res = {"value": K / elapsed, "ms_per_step": elapsed / K * 1e3, "runs_ms_per_step": [s / K * 1e3 for s in all_runs],
                 "batches_in_flight": D * P, "host_link_use": 1.0 * acc["host_rows"] * rb / elapsed / 1e9 / link_gbs if link_gbs > 0 else None,
                 "note": "the K steps by helios_plan_launch + helios_plan_wait per batch: %d contexts on %d streams, %d "
                         "mini-batches queued on each" % (D, D, P)}
    # by gangs (the headline): the mini-batches of M contexts share every launch, G such gangs on a stream each
    n_members = min(args.gang_members, helios.MAX_GANG) if B <= 2048 else 0
    if n_members > 0:
        for _ in range(max(1, args.gangs)):
            gangs.append(GangOnStream(n_members, lanes[0].cap, args.gang_host_blocks))
        torch.cuda.synchronize()
        region_gangs(0, Wm)
        elapsed, acc, all_runs = repeated(region_gangs, Wm, K)
        for gd in gangs:
            gd.close()
        n_gangs = len(gangs)
        gangs.clear()
        result["config"]["step"] = (
            "one mini-batch of a recorded gang (helios_gang_launch: sample, dedup, lookup, HBM+host gather, miss list of %d "
            "mini-batches in the same launches; helios_gang_wait), %d gangs of %d contexts, each gang on its own stream with "
            "one launch sequence queued; median of %d runs of the K steps" % (n_members, n_gangs, n_members, args.repeats))
        result["lanes"] = lanes_res
        result["gang_roles"] = optional("gang_roles", lambda: region_gang_roles(min(K, 25), n_members))
        hbm_role_us = max([v for k_, v in result["gang_roles"].get("avg_us_per_role_in_one_member", {}).items()
                           if k_.startswith("copy_hbm")] or [0.0])
        if hbm_role_us > 0:
            in_gang = 2.0 * (acc["hbm_rows"] / K) * rb / (hbm_role_us * 1e-6) / 1e9
            result["roofline"]["inside_a_gang"] = {
                "achieved": in_gang, "frac": in_gang / HBM_PEAK_GBS, "avg_role_us": hbm_role_us,
                "note": "the HBM-tier copy as a role of a gang's last launch (the timed region's form), beside the host-tier "
                        "copies: rows per batch x bytes per row / span of one member's role by the device clock"}
        result.update(value=K / elapsed, ms_per_step=elapsed / K * 1e3, runs_ms_per_step=[s / K * 1e3 for s in all_runs],
                      batches_in_flight=n_members * n_gangs)
    else:
        result.update(value=lanes_res["value"], ms_per_step=lanes_res["ms_per_step"], runs_ms_per_step=lanes_res["runs_ms_per_step"],
                      batches_in_flight=D * P)
    link_whole_run = 1.0 * acc["host_rows"] * rb / elapsed / 1e9
    result["roofline_host_link"]["in_the_timed_region"] = {
        "link_GBs": link_whole_run, "frac": link_whole_run / link_gbs if link_gbs > 0 else None,
        "note": "host-tier bytes of the K steps / wall time of the timed region (value)"}
    result["per_batch"] = {"raw_sampled_ids": acc["raw"] / K, "unique_ids": acc["unique"] / K,
                           "hit_ratio_hbm": acc["hbm_rows"] / max(acc["unique"], 1),
                           "hit_ratio_host": acc["host_rows"] / max(acc["unique"], 1),
                           "miss_ratio": acc["miss"] / max(acc["unique"], 1)}
    region_serial(0, Wm, 1, None)
    one_elapsed, _, _ = repeated(region_serial, Wm, K, 1, None)
    result["one_batch_in_flight"] = {"value": K / one_elapsed, "ms_per_step": one_elapsed / K * 1e3,
                                     "note": "the same K steps with helios_sync after every batch"}
    result["roles"] = region_roles(min(K, 50))
    if not full:
        for ln in lanes:
            for bs in ln.sets:
                for pl in bs.plans.values():
                    pl.destroy()
            ln.h.close()
        h.close()
        for pb in pinned_bufs:
            pb.free()
        return result

    def per_lane_region():
        lane_elapsed, _, _ = repeated(region_serial, Wm, K, D, None)
        return {"value": K / lane_elapsed, "ms_per_step": lane_elapsed / K * 1e3,
                "note": "%d lanes, helios_sync on a lane before it gets its next batch" % D}

    def miss_service_region():
        s6_elapsed, _, _ = repeated(region_serial, Wm, K, D, "zero-copy")
        return {"value": K / s6_elapsed, "ms_per_step": s6_elapsed / K * 1e3,
                "note": "S6 by helios_gather_miss (zero-copy reads of the stand-in) after every batch"}

    def miss_service_by_gangs():
        for _ in range(max(1, args.gangs)):
            gangs.append(GangOnStream(n_members, lanes[0].cap, args.gang_host_blocks, serve_misses=True))
        torch.cuda.synchronize()
        region_gangs(0, Wm)
        gs_elapsed, _, _ = repeated(region_gangs, Wm, K)
        for gd in gangs:
            gd.close()
        gangs.clear()
        return {"value": K / gs_elapsed, "ms_per_step": gs_elapsed / K * 1e3,
                "note": "the timed region with HELIOS_PARAM_SERVE_MISSES: every batch copies the rows of its own miss list from "
                        "the stand-in as a role of its last launch (S1-S6 in the launches of S1-S5)"}

    def miss_queue_region():
        for ln in lanes:
            ln.record_with_queue()
        torch.cuda.synchronize()
        region_serial(0, Wm, D, "queue")
        q_elapsed, _, _ = repeated(region_serial, Wm, K, D, "queue")
        for ln in lanes:
            ln.drop_queue()
        return {"value": K / q_elapsed, "ms_per_step": q_elapsed / K * 1e3, "queues_per_lane": args.missq_queues,
                "service_threads_per_lane": args.missq_threads,
                "note": "S6 in the shape of the paper's IO stack: submission kernel, host threads serving the stand-in "
                        "into a pinned staging buffer, completion kernel"}

    result["one_batch_per_lane"] = optional("one_batch_per_lane", per_lane_region)
    result["with_miss_service"] = optional("with_miss_service", miss_service_region)
    if n_members > 0 and tiers.n_rest > 0:
        result["with_miss_service"]["by_gangs"] = optional("with_miss_service.by_gangs", miss_service_by_gangs)
    if args.missq_queues > 0 and tiers.n_rest > 0:
        result["with_async_miss_queue"] = optional("with_async_miss_queue", miss_queue_region)
    if args.large_list_gb > 0:
        result["roofline"]["large_list"] = optional("large_list", lambda: large_list(torch, helios, dev, rb, args.large_list_gb, args.seed))

    # ---------------- CPU oracle on the same batches (reported baseline) + parity of one batch
    if not args.no_cpu:
        from oracle import helios_oracle as oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from pathlib_helios import assert_same, gpu_path, oracle_path, to_bytes
        off_h, idx_h, ord_h = offsets.cpu().numpy(), indices.cpu().numpy(), order.cpu().numpy()
        rank_h = oracle.rank_build(ord_h)
        tabs = [to_bytes(tiers.hbm[:tiers.n_hbm]), to_bytes(tiers.host[:tiers.n_host]),
                to_bytes(tiers.standin[:tiers.n_rest])]
        log("CPU oracle leg: host copies ready")
        b0 = Wm
        want = oracle_path(oracle, off_h, idx_h, seeds[b0].cpu().numpy(), sp.fanouts, rng_seeds[b0], rank_h,
                           tiers.n_hbm, tiers.n_host, *tabs, rb)
        got = gpu_path(h, helios, seeds[b0], sp.fanouts, rng_seeds[b0], fused=True)
        assert_same(got, want)
        result["parity"] = "bit-exact vs CPU oracle on batch %d (all outputs)" % b0
        seeds_h = [sd.cpu().numpy() for sd in seeds]

        def oracle_leg(seconds):
            done, t_cpu, steps = 0, time.perf_counter(), [0.0, 0.0, 0.0]
            while (time.perf_counter() - t_cpu) < seconds:
                b = Wm + done % K
                ta = time.perf_counter()
                hops_o = oracle.sample(off_h, idx_h, seeds_h[b], sp.fanouts, rng_seeds[b])
                tb = time.perf_counter()
                cat = np.concatenate([seeds_h[b]] + [fl for _, _, fl in hops_o])
                uq, _ = oracle.dedup(g.n_nodes, cat)
                tc = time.perf_counter()
                o = np.empty((uq.size, rb), np.uint8)
                oracle.gather(uq, rank_h, tiers.n_hbm, tiers.n_host, tabs[0], tabs[1], o)
                td = time.perf_counter()
                steps = [steps[0] + tb - ta, steps[1] + tc - tb, steps[2] + td - tc]
                done += 1
            return done, time.perf_counter() - t_cpu, [s / max(done, 1) * 1e3 for s in steps]

        all_cores = oracle.num_threads()
        done, cpu_elapsed, step_ms = oracle_leg(args.cpu_seconds)
        oracle.set_num_threads(1)
        done1, cpu_elapsed1, _ = oracle_leg(args.cpu_seconds / 3)
        oracle.set_num_threads(all_cores)
        result["cpu_baseline"] = {"value": done / cpu_elapsed, "unit": "mini-batches/s", "cores": all_cores,
                                  "kind": "oracle",
                                  "sample": f"{done} batches (passes over the {K} timed batches; sample, dedup, lookup, "
                                            f"gather of both cached tiers, miss list), {cpu_elapsed:.1f} s",
                                  "ms_per_step_by_part": {"sample": step_ms[0], "dedup": step_ms[1],
                                                          "lookup_gather_miss_list": step_ms[2]},
                                  "one_thread": {"value": done1 / cpu_elapsed1, "cores": 1,
                                                 "sample": f"{done1} batches, {cpu_elapsed1:.1f} s"}}
        del tabs, off_h, idx_h
    for ln in lanes:
        for bs in ln.sets:
            for pl in bs.plans.values():
                pl.destroy()
        ln.h.close()
    h.close()
    for pb in pinned_bufs:
        pb.free()
    return result


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="workload index in BASELINE.json configs (0-based)")
    ap.add_argument("--also", type=int, default=2,
                    help="a second workload whose headline figures go under \"also\" in the same line (-1: none)")
    ap.add_argument("--hbm-frac", type=float, default=None, help="config 4 only: HBM-tier fraction of the sweep")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--repeats", type=int, default=5, help="runs of the K-step timed region; the median is reported")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time given to the CPU-oracle leg")
    ap.add_argument("--depth", type=int, default=3,
                    help="lanes: library contexts, each on its own stream, that take the mini-batches in turn")
    ap.add_argument("--per-lane", type=int, default=2,
                    help="mini-batches queued per lane in the timed region (buffer sets per context): one runs, "
                         "the next waits behind it on the lane's stream")
    ap.add_argument("--gang-members", type=int, default=4,
                    help="members of a gang in the timed region (contexts whose mini-batches share every launch); 0: the timed "
                         "region is the one by lanes (--depth, --per-lane)")
    ap.add_argument("--gangs", type=int, default=3, help="gangs in flight in the timed region, each on its own stream")
    ap.add_argument("--gang-host-blocks", type=int, default=0,
                    help="workgroups of a gang member's host-tier copy (0: the library's default, a member's share of what fills the link)")
    ap.add_argument("--missq-queues", type=int, default=128,
                    help="queues of the asynchronous miss queue region (0 skips the region)")
    ap.add_argument("--missq-threads", type=int, default=4, help="service threads per miss queue (one queue per lane)")
    ap.add_argument("--large-list-gb", type=float, default=20.0,
                    help="table size of the bandwidth-bound run of the HBM-tier copy (1 M random rows; 0 skips it)")
    ap.add_argument("--presample-batches", type=int, default=0,
                    help="0: tiers in the in-degree order BASELINE.json names; N > 0: in the order of hotness counted over "
                         "N pre-sampling batches (the paper's policy); -1: over one epoch of the train split")
    ap.add_argument("--only", choices=["roofline", "large-list"], default=None,
                    help="roofline: set-up and the roofline region only (the command the kernel traces under profiles/ use); "
                         "large-list: only the bandwidth-bound run of the HBM-tier copy with the workload's row size (no "
                         "graph, no pinned tiers: the command the counter runs under profiles/ use)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--link-gbs", type=float, default=None,
                    help="skip the host-link probe and use this rate (for runs under a counter profiler)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU; the path shards by giving each GPU its own "
              "mini-batches, which needs no code here. Use --gpus 1.", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    link_gbs = args.link_gbs if args.link_gbs else measure_host_link(torch)
    log(f"host link (pinned H2D copy): {link_gbs:.1f} GB/s" + (" (given)" if args.link_gbs else ""))
    K, Wm = args.steps, args.warmup
    if args.only == "large-list":
        from paper_2310_00837_amd import helios, workload as W
        h = helios.Helios(0)
        copy_gbs = measure_plain_copy(torch, h)          # the yardstick kernel runs in the same process
        h.close()
        res = large_list(torch, helios, torch.device("cuda", 0), W.spec(args.config).row_bytes, args.large_list_gb, args.seed)
        res["plain_copy_GBs_on_this_box"] = copy_gbs
        print(json.dumps(res))
        return 0

    main_res = run_workload(args, args.config, args.hbm_frac, K, Wm, link_gbs, full=True)
    line = {"metric": "sampled mini-batches/sec; feature gather GB/s vs HBM and host-link peak",
            "value": main_res.get("value"), "unit": "mini-batches/s", "n_gpus": 1, "steps": K, "warmup": Wm,
            "ms_per_step": main_res.get("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": main_res["dtype"], "data": "synthetic"}
    line.update(main_res)
    if args.also >= 0 and args.also != args.config and args.only is None:
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        line["also"] = optional("also", lambda: run_workload(args, args.also, None, K, Wm, link_gbs, full=False))
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
