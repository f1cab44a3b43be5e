"""GPU parity at the full sizes of workloads 2, 3 and 4 (10^8 nodes, 10^9 edges, 57-102 GB of
features): first through helios_prepare_batch on one context, then in the launch configuration
bench.py times (three contexts on three streams, a recorded batch each, three mini-batches in
flight).  The inputs are generated on
the GPU; the CPU oracle runs the whole path on host copies of the same arrays and every output is
compared bit for bit.  In addition every gathered row is checked against the procedural feature
generator (out[j] == feat(unique[j]) for all j), a property that needs no table on the host."""
import time

import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import assert_same, gangs_in_flight, gpu_path, lanes_in_flight, oracle_path, to_bytes

pytestmark = pytest.mark.gpu
SEED = 1234


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


@pytest.fixture(scope="module")
def helios():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2310_00837_amd import helios as hl
    return hl


def _check_batches(h, helios, oracle, sp, g, host_csr, rank_h, n_hbm, n_host, tabs_dev, tabs_host, batches):
    off_h, idx_h = host_csr
    h.cache_build(g.order, n_hbm, n_host, sp.row_bytes, *tabs_dev)
    h.sync()
    wants = {}
    for b in batches:
        seeds = W.seed_batch(sp, g, b)
        rs = W.batch_rng_seed(SEED, b)
        got = gpu_path(h, helios, seeds, sp.fanouts, rs, fused=True)
        want = oracle_path(oracle, off_h, idx_h, seeds.cpu().numpy(), sp.fanouts, rs, rank_h, n_hbm, n_host,
                           *tabs_host, sp.row_bytes)
        assert_same(got, want)
        wants[b] = want
        uniq = torch.from_numpy(got["unique"]).cuda()
        for s in range(0, uniq.numel(), 1 << 16):                   # every row equals the generator's row
            rows = W.feature_rows(SEED, uniq[s:s + (1 << 16)], sp.dim, sp.dtype)
            mine = torch.from_numpy(got["out"][s:s + (1 << 16)]).cuda()
            assert torch.equal(rows.view(torch.uint8).reshape(rows.shape[0], -1), mine)
        st = want["stats"].tolist()
        say(f"  {sp.name} batch {b}: raw {sum(len(x[2]) for x in want['hops'])} unique {st[0]} "
            f"hbm {st[1]} host {st[2]} miss {st[3]}: bit-exact")
    # the same batches as bench.py launches them: every batch once on each of the three lanes
    order_of_jobs = [b for r in range(3) for b in (batches[r % len(batches):] + batches[:r % len(batches)])]
    while len(order_of_jobs) % 3:
        order_of_jobs.append(batches[0])
    jobs = [(W.seed_batch(sp, g, b).cuda(), W.batch_rng_seed(SEED, b)) for b in order_of_jobs]
    got = lanes_in_flight(helios, g.offsets, g.indices, g.order, n_hbm, n_host, sp.row_bytes, tabs_dev, sp.batch,
                          sp.fanouts, jobs)
    for b, res in zip(order_of_jobs, got):
        want = dict(wants[b])
        del want["out_before_miss"]
        assert_same(res, want)
    got = lanes_in_flight(helios, g.offsets, g.indices, g.order, n_hbm, n_host, sp.row_bytes, tabs_dev, sp.batch,
                          sp.fanouts, jobs + jobs, per_lane=2)
    for b, res in zip(order_of_jobs + order_of_jobs, got):
        want = dict(wants[b])
        del want["out"]
        assert_same(res, want)
    say(f"  {sp.name}: {len(jobs)} recorded batches, one per lane, and {2 * len(jobs)}, two per lane: bit-exact")
    # and as bench.py's timed region launches them: gangs of four contexts, three gangs in flight
    gang_jobs, gang_order = list(jobs), list(order_of_jobs)
    while len(gang_jobs) % 4:
        gang_jobs.append(jobs[0])
        gang_order.append(order_of_jobs[0])
    got = gangs_in_flight(helios, g.offsets, g.indices, g.order, n_hbm, n_host, sp.row_bytes, tabs_dev, sp.batch,
                          sp.fanouts, gang_jobs + gang_jobs, members=4, n_gangs=3)
    for b, res in zip(gang_order + gang_order, got):
        want = dict(wants[b])
        del want["out"]
        assert_same(res, want)
    say(f"  {sp.name}: {2 * len(gang_jobs)} batches in gangs of four, three gangs in flight: bit-exact")
    if tabs_dev[2] is not None:
        # ... and with every batch serving its own misses from the stand-in (S6 as a role of the last launch)
        got = gangs_in_flight(helios, g.offsets, g.indices, g.order, n_hbm, n_host, sp.row_bytes, tabs_dev, sp.batch,
                              sp.fanouts, gang_jobs, members=4, n_gangs=2, served=True)
        for b, res in zip(gang_order, got):
            want = dict(wants[b])
            del want["out_before_miss"]
            assert_same(res, want)
        say(f"  {sp.name}: {len(gang_jobs)} batches in gangs that serve their own misses: bit-exact")


def test_workloads_2_and_4_full_size(helios, oracle):
    """The PA-shaped graph (111 M nodes, 1.6 B edges, fp32 dim 128).  The feature table is laid
    out once in rank order, in HBM and in pinned host memory; workload 2 and the four tier splits
    of workload 4 are views of those two copies."""
    sp2 = W.spec(2)
    dev = torch.device("cuda", 0)
    t0 = time.time()
    g = W.make_graph(sp2, SEED, dev, progress=None)
    say(f"graph N={g.n_nodes} E={g.n_edges} in {time.time() - t0:.1f}s")
    full_dev = torch.empty((g.n_nodes, sp2.dim), dtype=sp2.dtype, device=dev)
    W.fill_rows(full_dev, SEED, g.order)
    full_host_buf = helios.pinned_empty((g.n_nodes, sp2.dim), sp2.dtype)
    full_host = full_host_buf.tensor
    full_host.copy_(full_dev)
    say(f"feature table in rank order on both sides at {time.time() - t0:.1f}s")
    off_h, idx_h = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    rank_h = oracle.rank_build(g.order.cpu().numpy())
    host_bytes = full_host.view(torch.uint8).reshape(g.n_nodes, -1).numpy()
    say(f"host copies ready at {time.time() - t0:.1f}s")
    h = helios.Helios(0)
    h.csr_load(g.offsets, g.indices)
    cases = [(sp2, [0, 1])] + [(W.spec(4, p), [0]) for p in (0.0, 0.25, 0.5, 1.0)]
    for sp, batches in cases:
        n_hbm, n_host, n_rest = sp.tier_rows(g.n_nodes)
        say(f"{sp.name}: tiers {n_hbm}/{n_host}/{n_rest}")
        tabs_dev = (full_dev[:n_hbm] if n_hbm else None, full_host[n_hbm:n_hbm + n_host] if n_host else None,
                    full_host[n_hbm + n_host:] if n_rest else None)
        tabs_host = (host_bytes[:n_hbm], host_bytes[n_hbm:n_hbm + n_host], host_bytes[n_hbm + n_host:])
        _check_batches(h, helios, oracle, sp, g, (off_h, idx_h), rank_h, n_hbm, n_host, tabs_dev, tabs_host, batches)
    # The hotness order at this size (Sec. 3.2.2 "Cache Initialization" sorts every vertex of the graph): with the
    # in-degrees as counters the result is the workload's own cache order, which the generator computes with
    # torch's stable sort; and the properties that define the order hold (a permutation, counters descending,
    # equal counters by ascending ID).
    counts = torch.zeros(g.n_nodes, dtype=torch.int64, device=dev)
    for s0 in range(0, g.indices.numel(), 1 << 28):
        counts += torch.bincount(g.indices[s0:s0 + (1 << 28)].to(torch.int64), minlength=g.n_nodes)
    counts = counts.to(torch.int32)
    order = torch.empty(g.n_nodes, dtype=torch.int32, device=dev)
    h.hotness_order(counts, order)
    h.sync()
    assert torch.equal(order, g.order.to(dev))
    by_order = counts[order.long()]
    assert bool((by_order[:-1] >= by_order[1:]).all())
    ties = by_order[:-1] == by_order[1:]
    assert bool((order[:-1][ties] < order[1:][ties]).all())
    assert bool((torch.bincount(order.long(), minlength=g.n_nodes) == 1).all())
    say(f"hotness order of {g.n_nodes} nodes ({int(ties.sum())} ties between neighbours): equal to the stable sort")
    del counts, order, by_order, ties
    h.close()
    del full_dev, full_host, host_bytes, tabs_dev, tabs_host
    full_host_buf.free()
    torch.cuda.empty_cache()
    say(f"done at {time.time() - t0:.1f}s")


def test_workload_3_full_size(helios, oracle):
    """Wide rows: 50 M nodes, 1 B edges, fp16 dim 1024 (2 KB rows), 3 hops."""
    sp = W.spec(3)
    dev = torch.device("cuda", 0)
    t0 = time.time()
    g = W.make_graph(sp, SEED, dev, progress=None)
    say(f"graph N={g.n_nodes} E={g.n_edges} in {time.time() - t0:.1f}s")
    bufs = []

    def pinned(shape, dtype):
        bufs.append(helios.pinned_empty(shape, dtype))
        return bufs[-1].tensor

    tiers = W.make_tiers(sp, g, dev, progress=None, pinned_empty=pinned)
    say(f"tiers {tiers.n_hbm}/{tiers.n_host}/{tiers.n_rest} filled at {time.time() - t0:.1f}s")
    # the oracle's copy of the HBM tier: 64 GB of ordinary host memory (pinned memory is limited on the box)
    hbm_host = torch.empty(tiers.hbm.shape, dtype=sp.dtype)
    step = 4_000_000
    for r0 in range(0, tiers.n_hbm, step):
        hbm_host[r0:r0 + step].copy_(tiers.hbm[r0:r0 + step])
        say(f"  HBM tier -> host {min(r0 + step, tiers.n_hbm)}/{tiers.n_hbm}")
    off_h, idx_h = g.offsets.cpu().numpy(), g.indices.cpu().numpy()
    rank_h = oracle.rank_build(g.order.cpu().numpy())
    say(f"host copies ready at {time.time() - t0:.1f}s")

    def as_bytes(t, n):
        return t.view(torch.uint8).reshape(t.shape[0], -1).numpy()[:n]

    tabs_host = (as_bytes(hbm_host, tiers.n_hbm), as_bytes(tiers.host, tiers.n_host), as_bytes(tiers.standin, tiers.n_rest))
    h = helios.Helios(0)
    h.csr_load(g.offsets, g.indices)
    _check_batches(h, helios, oracle, sp, g, (off_h, idx_h), rank_h, tiers.n_hbm, tiers.n_host,
                   (tiers.hbm, tiers.host, tiers.standin), tabs_host, [0, 1])
    h.close()
    del tabs_host, hbm_host, tiers
    for b in bufs:
        b.free()
    torch.cuda.empty_cache()
    say(f"done at {time.time() - t0:.1f}s")
