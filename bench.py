"""Benchmark of the Helios mini-batch preparation path on one MI355X.

A step is one pass of the whole path (k-hop sampling, de-duplication, cache lookup, gather of
both cached tiers, miss list: helios_prepare_batch + helios_sync) over one batch of seeds of a
synthetic workload whose graph, feature tables and seeds are resident before the timed region
(graph, cache map and HBM tier in HBM; host tier and storage stand-in in pinned host memory,
where the method keeps them).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..4] [--hbm-frac P]
"""
import argparse
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


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


def probe_launch_delay(torch, helios, dev, args) -> int:
    """What a kernel launch costs while the host link is saturated: stream B runs a chain of `chain` one-workgroup
    copies (64 B each) with and without a long row copy from pinned host memory running on stream A (512 B rows,
    --host-blocks workgroups, library default if 0).  The difference is what every launch of a mini-batch's
    front pays while another mini-batch's host-tier copy is running."""
    rb, table_rows, n_rows, chain = 512, 600_000, 1 << 19, 200
    table = helios.pinned_empty((table_rows, rb), torch.uint8)
    table.tensor.fill_(1)
    out = torch.empty((n_rows, rb), dtype=torch.uint8, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    slot = torch.randint(0, table_rows, (n_rows,), device=dev, dtype=torch.int32, generator=gen)
    pos = torch.arange(n_rows, device=dev, dtype=torch.int32)
    small_src = torch.zeros(64, dtype=torch.uint8, device=dev)
    small_dst = torch.zeros(64, dtype=torch.uint8, device=dev)
    sa, sb = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)
    a, b = helios.Helios(0, stream=sa), helios.Helios(0, stream=sb)
    n1 = torch.tensor([0, 1], dtype=torch.int64, device=dev)
    order = torch.tensor([0], dtype=torch.int32, device=dev)
    for ctx in (a, b):                       # a one-node graph whose only row lives in the stand-in: the long copy is S6
        ctx.csr_load(n1, order)
    a.cache_build(order, 0, 0, rb, None, None, table.tensor)
    if args.host_blocks:
        a.set_param(helios.PARAM_HOST_GATHER_BLOCKS, args.host_blocks)
    a.sync()
    res = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(sa)
    a._check(helios._lib.helios_gather_miss(a._h, pos.data_ptr(), slot.data_ptr(), n_rows, None, out.data_ptr()))
    e1.record(sa)
    e1.synchronize()
    res["link_copy_alone_GBs"] = n_rows * rb / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # the chain as one recorded graph, so that the host's launch rate does not hide what the GPU does
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=sb):
        for _ in range(chain):
            b.calibration_copy(small_src, small_dst)
    torch.cuda.synchronize()
    for with_link in (0, 1):
        best = 1e30
        for _ in range(5):
            torch.cuda.synchronize()
            if with_link:
                a._check(helios._lib.helios_gather_miss(a._h, pos.data_ptr(), slot.data_ptr(), n_rows, None, out.data_ptr()))
            t0 = time.perf_counter()
            with torch.cuda.stream(sb):
                graph.replay()
            sb.synchronize()
            best = min(best, (time.perf_counter() - t0) / chain * 1e6)
            torch.cuda.synchronize()
        res["us_per_launch_link_busy" if with_link else "us_per_launch_link_idle"] = best
    res["chain"] = chain
    res["what"] = ("a recorded chain of one-workgroup kernels on one stream; the other stream copies 2^19 rows of 512 B "
                   "from pinned host memory")
    a.close()
    b.close()
    table.free()
    print(json.dumps(res))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload index in BASELINE.json configs (0-based)")
    ap.add_argument("--hbm-frac", type=float, default=None, help="config 4 only: HBM-tier fraction of the sweep")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time given to the CPU-oracle leg")
    ap.add_argument("--depth", type=int, default=3,
                    help="mini-batches in flight during the timed region (each on its own context and stream)")
    ap.add_argument("--per-lane", type=int, default=2,
                    help="mini-batches queued per lane in the timed region (buffer sets per context): one runs, "
                         "the next waits behind it on the lane's stream")
    ap.add_argument("--threads", type=int, default=0, help="0: one host thread drives all lanes (default, fastest); 1: one host thread per lane")
    ap.add_argument("--graph", type=int, default=1, help="1: replay a recorded batch (HIP graph) per step; 0: launch directly")
    ap.add_argument("--hbm-blocks", type=int, default=0, help="workgroups of the HBM-tier copy (0 = library default)")
    ap.add_argument("--host-blocks", type=int, default=0, help="workgroups of the host-link copies (0 = library default)")
    ap.add_argument("--missq-queues", type=int, default=128,
                    help="queues of the asynchronous miss queue region (0 skips the region)")
    ap.add_argument("--missq-threads", type=int, default=4, help="service threads per miss queue (one queue per lane)")
    ap.add_argument("--large-list-gb", type=float, default=20.0,
                    help="table size of the bandwidth-bound run of the HBM-tier copy (1 M random rows; 0 skips it)")
    ap.add_argument("--serial-tiers", type=int, default=1,
                    help="1: the host-tier copy follows the HBM-tier copy on the lane's stream (library default); "
                         "0: the two run side by side on two streams")
    ap.add_argument("--probe-launch-delay", action="store_true",
                    help="instead of the benchmark: time a chain of small kernels on one stream while another "
                         "stream's row copy saturates the host link, and print that as one JSON line")
    ap.add_argument("--presample-batches", type=int, default=0,
                    help="0: tiers in the in-degree order BASELINE.json names; N > 0: in the order of hotness counted over "
                         "N pre-sampling batches (the paper's policy); -1: over one epoch of the train split")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--link-gbs", type=float, default=None,
                    help="skip the host-link probe and use this rate (for runs under a counter profiler)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU; the path shards by giving each GPU its own "
              "mini-batches, which needs no code here. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2310_00837_amd import helios, workload as W
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    if args.probe_launch_delay:
        return probe_launch_delay(torch, helios, dev, args)
    sp = W.spec(args.config, args.hbm_frac)
    K, Wm = args.steps, args.warmup

    # ---------------- inputs (untimed)
    t0 = time.time()
    gen_dev = dev if sp.n_nodes > 5_000_000 else "cpu"
    g = W.make_graph(sp, args.seed, gen_dev, progress=log if sp.n_nodes > 5_000_000 else None)
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

    tiers = W.make_tiers(sp, g, dev, progress=log if sp.n_nodes > 5_000_000 else None, pinned_empty=pinned_exact)
    log(f"tiers: hbm {tiers.n_hbm} host {tiers.n_host} stand-in {tiers.n_rest} rows x {sp.row_bytes} B "
        f"filled in {time.time() - t1:.1f}s")
    link_gbs = args.link_gbs if args.link_gbs else measure_host_link(torch)
    log(f"host link (pinned H2D copy): {link_gbs:.1f} GB/s" + (" (given)" if args.link_gbs else ""))

    h = helios.Helios(0)
    # yardstick: a plain 1 GiB device copy with the row copy's accesses (known traffic: 1 GiB read + 1 GiB written)
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_src.fill_(3)
    copy_gbs = 0.0
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        h.calibration_copy(cal_src, cal_dst)
        e1.record()
        e1.synchronize()
        copy_gbs = max(copy_gbs, 2.0 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del cal_src, cal_dst
    log(f"plain device copy (1 GiB, read+write): {copy_gbs:.0f} GB/s")
    h.csr_load(offsets, indices)
    h.cache_build(order, tiers.n_hbm, tiers.n_host, sp.row_bytes, tiers.hbm, tiers.host, tiers.standin)
    h.sync()

    B = min(sp.batch, g.n_nodes)
    n_batches = K + Wm
    seeds = [W.seed_batch(sp, g, b).to(dev) for b in range(n_batches)]
    rng_seeds = [W.batch_rng_seed(args.seed, b) for b in range(n_batches)]

    class Buffers:
        """Caller-owned outputs of one mini-batch, and the recordings that write to them."""

        def __init__(self, cap):
            self.hops = helios.alloc_hops(B, sp.fanouts, dev)
            self.unique = torch.empty(cap, dtype=torch.int32, device=dev)
            self.inverse = torch.empty(cap, dtype=torch.int32, device=dev)
            self.out = torch.empty((cap, sp.row_bytes), dtype=torch.uint8, device=dev)
            self.mp = torch.empty(cap, dtype=torch.int32, device=dev)
            self.mi, self.ms = torch.empty_like(self.mp), torch.empty_like(self.mp)
            self.sizes = torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory()
            self.n_unique = torch.zeros(1, dtype=torch.int64).pin_memory()
            self.stats = torch.zeros(4, dtype=torch.int64).pin_memory()
            # zero-copy numpy views of the pinned result words: reading them costs the host almost nothing
            self.stats_np, self.sizes_np = self.stats.numpy(), self.sizes.numpy()
            self.plans = {}

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
            self.sets = [Buffers(cap) for _ in range(max(1, args.per_lane))]
            first = self.sets[0]                 # the set the one-per-lane regions use
            for name in ("hops", "unique", "inverse", "out", "mp", "mi", "ms", "sizes", "n_unique", "stats", "stats_np",
                         "sizes_np", "plans"):
                setattr(self, name, getattr(first, name))
            self.cap = cap
            self.queue = None

        def record_with_queue(self) -> None:
            """A miss queue of this lane's own and a recording in which the batch submits its misses to it."""
            nq = args.missq_queues
            self.queue = helios.MissQueue(self.h, nq, (self.cap + nq - 1) // nq, args.missq_threads)
            self.queue.attach()
            self.h.set_timing(0)
            self.plans["queue"] = self.h.plan_create(B, sp.fanouts, self.hops, self.sizes, self.unique, self.inverse,
                                                     self.n_unique, self.out, self.mp, self.mi, self.ms, self.stats)

        def record(self) -> None:
            """One recording (HIP graph) of the whole-path call per timing level (and per buffer set for level 0)."""
            for level in (0, 1):
                self.h.set_timing(level)
                for bs in (self.sets if level == 0 else self.sets[:1]):
                    bs.plans[level] = self.h.plan_create(B, sp.fanouts, bs.hops, bs.sizes, bs.unique, bs.inverse,
                                                         bs.n_unique, bs.out, bs.mp, bs.mi, bs.ms, bs.stats)
            self.h.set_timing(0)

        def launch_set(self, which: int, b: int) -> None:
            """Batch b into buffer set `which` (timing off)."""
            bs = self.sets[which]
            if args.graph:
                bs.plans[0].launch(seeds[b], rng_seeds[b])
            else:
                self.h.prepare_batch(seeds[b], sp.fanouts, rng_seeds[b], bs.hops, bs.sizes, bs.unique, bs.inverse,
                                     bs.n_unique, bs.out, bs.mp, bs.mi, bs.ms, bs.stats)

        def launch(self, b: int, serve_misses, timing: int = 0) -> None:
            if serve_misses == "queue":          # the batch submits its misses itself; the completion kernel follows
                if args.graph:
                    self.plans["queue"].launch(seeds[b], rng_seeds[b])
                else:
                    self.h.prepare_batch(seeds[b], sp.fanouts, rng_seeds[b], self.hops, self.sizes, self.unique,
                                         self.inverse, self.n_unique, self.out, self.mp, self.mi, self.ms, self.stats)
                self.queue.complete(self.out)
                return
            plan = self.plans.get(timing) if args.graph else None
            if plan is not None:
                plan.launch(seeds[b], rng_seeds[b])
            else:
                self.h.prepare_batch(seeds[b], sp.fanouts, rng_seeds[b], self.hops, self.sizes, self.unique,
                                     self.inverse, self.n_unique, self.out, self.mp, self.mi, self.ms, self.stats)
            if serve_misses:
                self.h.gather_miss(self.mp, self.ms, self.mp.numel(), self.stats[3:4], self.out)

    # every lane gets a stream of its own (a batch cannot be recorded on the NULL stream); `h` keeps the
    # default stream and is used for set-up and the parity check only
    lanes = []
    for _ in range(max(1, args.depth)):
        st = torch.cuda.Stream(device=dev)
        ctx = helios.Helios(0, stream=st)
        ctx.csr_load(offsets, indices)
        ctx.cache_build(order, tiers.n_hbm, tiers.n_host, sp.row_bytes, tiers.hbm, tiers.host, tiers.standin)
        ctx.sync()
        if args.host_blocks:
            ctx.set_param(helios.PARAM_HOST_GATHER_BLOCKS, args.host_blocks)
        if args.hbm_blocks:
            ctx.set_param(helios.PARAM_HBM_GATHER_BLOCKS, args.hbm_blocks)
        if not args.serial_tiers:
            ctx.set_param(helios.PARAM_SERIAL_TIERS, 0)
        lanes.append(Lane(ctx, st))
    torch.cuda.synchronize()
    if args.graph:
        for ln in lanes:
            ln.record()
        torch.cuda.synchronize()

    def run_region(first: int, count: int, depth: int, timing: int, serve_misses, per_lane: int = 1):
        """`count` whole steps on `depth` lanes.  per_lane == 1: lane b % depth takes batch b and is waited for
        (helios_sync) before it is reused.  per_lane > 1 (recorded batches, no timing, no miss service): every
        lane has per_lane buffer sets, a batch is queued behind the lane's running one, and each batch is waited
        for by itself (helios_plan_wait).  Returns (seconds, sums)."""
        acc = dict(hbm_ms=0.0, host_ms=0.0, hbm_ev_ms=0.0, host_ev_ms=0.0, hbm_rows=0, host_rows=0, miss=0, unique=0,
                   raw=0)
        use = lanes[:depth]
        for ln in use:
            ln.h.set_timing(timing)

        def tally(bs):
            st = bs.stats_np
            acc["hbm_rows"] += int(st[1])
            acc["host_rows"] += int(st[2])
            acc["miss"] += int(st[3])
            acc["unique"] += int(st[0])
            acc["raw"] += int(bs.sizes_np[1::2].sum())

        def retire(ln):
            ln.h.sync()
            if timing:
                a_ms, b_ms, a_ev, b_ev = ln.h.gather_times()
                acc["hbm_ms"] += a_ms
                acc["host_ms"] += b_ms
                acc["hbm_ev_ms"] += a_ev
                acc["host_ev_ms"] += b_ev
            tally(ln)

        def worker(w: int) -> None:          # lane w takes batches w, w + depth, ... one after the other
            ln = use[w]
            for k in range(w, count, depth):
                ln.launch(first + k, serve_misses, timing)
                retire(ln)

        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        if per_lane > 1 and args.graph and not timing and not serve_misses:
            units = [(ln, w) for w in range(per_lane) for ln in use]      # lane 0 set 0, lane 1 set 0, ..., lane 0 set 1, ...
            for k in range(count):
                ln, w = units[k % len(units)]
                if k >= len(units):
                    ln.sets[w].plans[0].wait()
                    tally(ln.sets[w])
                ln.launch_set(w, first + k)
            for k in range(max(0, count - len(units)), count):
                ln, w = units[k % len(units)]
                ln.sets[w].plans[0].wait()
                tally(ln.sets[w])
            for ln in use:
                ln.h.sync()
        elif depth == 1 or not args.threads:
            for k in range(count):
                ln = use[k % depth]
                if k >= depth:
                    retire(ln)
                ln.launch(first + k, serve_misses, timing)
            for k in range(max(0, count - depth), count):
                retire(use[k % depth])
        else:                                # one host thread per lane (the library calls release the GIL)
            ts = [threading.Thread(target=worker, args=(w,)) for w in range(depth)]
            for t in ts:
                t.start()
            for t in ts:
                t.join()
        torch.cuda.synchronize()
        seconds = time.perf_counter() - t_begin
        for ln in use:
            ln.h.set_timing(0)
        return seconds, acc

    # ---------------- timed region: W warm-up steps, then K whole steps (S1-S5) with `depth` mini-batches in
    # flight; the row-copy kernels are timed with the device clock inside the same region
    D = len(lanes)
    P = max(1, args.per_lane) if args.graph else 1
    run_region(0, Wm, D, 0, False, P)
    elapsed, acc = run_region(Wm, K, D, 0, False, P)
    # the same K steps: one batch per lane with the copies timed by the device clock; one batch in flight; with
    # the miss list served (S6); with HIP events around the copies
    run_region(0, Wm, D, 1, False)
    ov_elapsed, ov_acc = run_region(Wm, K, D, 1, False)
    run_region(0, Wm, 1, 1, False)
    one_elapsed, one_acc = run_region(Wm, K, 1, 1, False)
    elapsed_s6, _ = run_region(Wm, K, D, 0, True)
    _, ev_acc = run_region(Wm, min(K, 50), 1, 2, False)
    # S6 through the asynchronous miss queue: submission kernel after the lookup, host service threads,
    # completion kernel after the cached tiers (each lane has a queue of its own)
    elapsed_q = None
    if args.missq_queues > 0 and tiers.n_rest > 0:
        for ln in lanes:
            ln.record_with_queue()
        torch.cuda.synchronize()
        run_region(0, Wm, D, 0, "queue")
        elapsed_q, _ = run_region(Wm, K, D, 0, "queue")
        for ln in lanes:
            ln.plans.pop("queue").destroy()
            ln.queue.destroy()
            ln.queue = None

    rb = sp.row_bytes

    def large_list():
        """The HBM-tier copy where it is bound by bandwidth: helios_gather of 1 M random IDs (fewer for rows
        above 1 KB) that all hit an HBM tier of --large-list-gb, far larger than the last-level cache."""
        n_tab = int(args.large_list_gb * 1e9) // rb
        n_ids = 1_000_000 if rb <= 1024 else 500_000
        if n_tab < 2 * n_ids:
            return None
        table = torch.empty((n_tab, rb), dtype=torch.uint8, device=dev)
        table.fill_(5)
        order_l = torch.arange(n_tab, device=dev, dtype=torch.int32)       # the IDs are random, so are the rows
        gen = torch.Generator(device=dev)
        gen.manual_seed(args.seed)
        ids = torch.randint(0, n_tab, (n_ids,), device=dev, dtype=torch.int32, generator=gen)
        out = torch.empty((n_ids, rb), dtype=torch.uint8, device=dev)
        mp = torch.empty(16, dtype=torch.int32, device=dev)
        stats = torch.zeros(4, dtype=torch.int64).pin_memory()
        ctx = helios.Helios(0, stream=torch.cuda.Stream(device=dev))
        ctx.csr_load(torch.zeros(n_tab + 1, dtype=torch.int64, device=dev), torch.zeros(1, dtype=torch.int32, device=dev))
        ctx.cache_build(order_l, n_tab, 0, rb, table, None, None)
        ctx.set_timing(1)
        best = 0.0
        for _ in range(5):
            ctx.gather(ids, out, mp, mp.clone(), mp.clone(), stats)
            ctx.sync()
            ms = ctx.gather_times()[0]
            best = max(best, 2.0 * n_ids * rb / (ms * 1e-3) / 1e9) if ms > 0 else best
        ctx.close()
        return {"rows": n_ids, "table_GB": n_tab * rb / 1e9, "achieved": best, "frac": best / HBM_PEAK_GBS,
                "note": "same kernel, best of 5, device clock; a list long enough to be bound by bandwidth"}

    big = large_list() if args.large_list_gb > 0 else None

    def rates(a):
        hbm = 2.0 * a["hbm_rows"] * rb / (a["hbm_ms"] * 1e-3) / 1e9 if a["hbm_ms"] > 0 else 0.0     # read + write
        host = 1.0 * a["host_rows"] * rb / (a["host_ms"] * 1e-3) / 1e9 if a["host_ms"] > 0 else 0.0  # bytes over the link
        return hbm, host

    hbm_gbs, host_gbs = rates(one_acc)              # kernel quality: nothing else runs beside the copies
    ov_hbm_gbs, ov_host_gbs = rates(ov_acc)         # the same kernels with one batch on each lane
    dominant_host = one_acc["host_ms"] > one_acc["hbm_ms"]
    link_whole_run = 1.0 * acc["host_rows"] * rb / elapsed / 1e9

    # HBM bytes per launch of the HBM-tier copy from the committed counter runs (two rocprofv3 --pmc runs,
    # scaled by the calibration copy); only for the workload they were taken on
    traffic = None
    names = {1: "hbm_traffic_cfg1_medium.txt"}
    tpath = os.path.join(ROOT, "profiles", names.get(args.config, "none"))
    if os.path.exists(tpath) and args.hbm_frac is None:
        for line in open(tpath):
            if line.startswith("TRAFFIC_JSON:"):
                try:
                    traffic = json.loads(line[len("TRAFFIC_JSON:"):])
                except Exception:
                    traffic = None

    result = {
        "metric": "sampled mini-batches/sec; feature gather GB/s vs HBM and host-link peak",
        "value": K / elapsed,
        "unit": "mini-batches/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32 ids / byte rows (" + ("fp32" if sp.dtype == torch.float32 else "fp16") + " features)",
        "data": "synthetic",
        "config": {"workload": f"BASELINE.json configs[{args.config}] {sp.name}", "n_nodes": g.n_nodes,
                   "n_edges": g.n_edges, "batch": B, "fanouts": sp.fanouts, "row_bytes": rb,
                   "tier_rows": [tiers.n_hbm, tiers.n_host, tiers.n_rest], "seed": args.seed, "cache_order": cache_order,
                   "step": ("helios_plan_launch (recorded helios_prepare_batch" if args.graph else "helios_prepare_batch (") +
                           ": sample, dedup, lookup, HBM+host gather, miss list) + one wait per batch (helios_plan_wait / helios_sync), "
                           "%d contexts on %d streams, %d mini-batches queued on each" % (D, D, P)},
        "roofline": {"kernel": "gather_rows_kernel (HBM tier)", "bound": "hbm", "achieved": hbm_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "avg_kernel_us": one_acc["hbm_ms"] / K * 1e3,
                     "avg_event_us": ev_acc["hbm_ev_ms"] / min(K, 50) * 1e3,
                     "region": "the K timed steps run with one mini-batch in flight (as a kernel trace sees them)",
                     "timer": "device clock, earliest workgroup start to latest end; avg_event_us: HIP events on the kernel's stream",
                     "rows_per_launch": one_acc["hbm_rows"] / K, "bytes_per_row": 2 * rb,
                     "plain_copy_GBs_on_this_box": copy_gbs,
                     "large_list": big,
                     "while_overlapped": {"achieved": ov_hbm_gbs, "frac": ov_hbm_gbs / HBM_PEAK_GBS,
                                          "avg_kernel_us": ov_acc["hbm_ms"] / K * 1e3,
                                          "note": "same kernel with one mini-batch on each of the %d lanes, beside other batches' host-link copies" % D}},
        "roofline_host_link": {"kernel": "gather_rows_kernel (host tier)", "bound": "host_link",
                               "achieved": host_gbs, "peak": link_gbs, "unit": "GB/s",
                               "frac": host_gbs / link_gbs if link_gbs > 0 else None,
                               "peak_source": "given on the command line" if args.link_gbs else "pinned H2D copy measured in this run",
                               "avg_kernel_us": one_acc["host_ms"] / K * 1e3,
                               "avg_event_us": ev_acc["host_ev_ms"] / min(K, 50) * 1e3,
                               "rows_per_launch": one_acc["host_rows"] / K, "bytes_per_row": rb,
                               "while_overlapped": {"link_GBs_over_the_whole_region": link_whole_run,
                                                    "frac": link_whole_run / link_gbs if link_gbs > 0 else None,
                                                    "per_kernel_GBs": ov_host_gbs,
                                                    "note": "host-tier bytes of all K steps / wall time of the timed region (value)"}},
        "dominant_kernel": "host-tier gather" if dominant_host else "HBM-tier gather",
        "with_miss_service": {"value": K / elapsed_s6, "ms_per_step": elapsed_s6 / K * 1e3},
        "with_async_miss_queue": None if elapsed_q is None else {
            "value": K / elapsed_q, "ms_per_step": elapsed_q / K * 1e3, "queues_per_lane": args.missq_queues,
            "service_threads_per_lane": args.missq_threads,
            "note": "S6 in the shape of the paper's IO stack: submission kernel, host threads serving the stand-in "
                    "into a pinned staging buffer, completion kernel"},
        "batches_in_flight": D * P,
        "one_batch_per_lane": {"value": K / ov_elapsed, "ms_per_step": ov_elapsed / K * 1e3,
                               "note": "%d lanes, helios_sync on a lane before it gets its next batch" % D},
        "one_batch_in_flight": {"value": K / one_elapsed, "ms_per_step": one_elapsed / K * 1e3,
                                "note": "the same K steps with helios_sync after every batch"},
        "per_batch": {"raw_sampled_ids": acc["raw"] / K, "unique_ids": acc["unique"] / K,
                      "hit_ratio_hbm": acc["hbm_rows"] / max(acc["unique"], 1),
                      "hit_ratio_host": acc["host_rows"] / max(acc["unique"], 1),
                      "miss_ratio": acc["miss"] / max(acc["unique"], 1)},
    }

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
            done, t_cpu = 0, time.perf_counter()
            while (time.perf_counter() - t_cpu) < seconds:
                b = Wm + done % K
                hops_o = oracle.sample(off_h, idx_h, seeds_h[b], sp.fanouts, rng_seeds[b])
                cat = np.concatenate([seeds_h[b]] + [fl for _, _, fl in hops_o])
                uq, _ = oracle.dedup(g.n_nodes, cat)
                o = np.empty((uq.size, rb), np.uint8)
                oracle.gather(uq, rank_h, tiers.n_hbm, tiers.n_host, tabs[0], tabs[1], o)
                done += 1
            return done, time.perf_counter() - t_cpu

        all_cores = oracle.num_threads()
        done, cpu_elapsed = oracle_leg(args.cpu_seconds)
        oracle.set_num_threads(1)
        done1, cpu_elapsed1 = oracle_leg(args.cpu_seconds / 3)
        oracle.set_num_threads(all_cores)
        result["cpu_baseline"] = {"value": done / cpu_elapsed, "unit": "mini-batches/s", "cores": all_cores,
                                  "kind": "oracle",
                                  "sample": f"{done} batches (passes over the {K} timed batches; sample, dedup, lookup, "
                                            f"gather of both cached tiers, miss list), {cpu_elapsed:.1f} s",
                                  "one_thread": {"value": done1 / cpu_elapsed1, "cores": 1,
                                                 "sample": f"{done1} batches, {cpu_elapsed1:.1f} s"}}
    for ln in lanes:
        for pl in ln.plans.values():
            pl.destroy()
        ln.h.close()
    h.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
