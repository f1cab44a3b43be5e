"""A recorded batch (HIP graph) must give what the directly launched path gives: every replay is
checked against the CPU oracle, with directly launched batches and synchronisations in between."""
import numpy as np
import pytest
import torch

from paper_2310_00837_amd import workload as W
from pathlib_helios import GpuCache, SENTINEL, assert_same, gpu_path, lanes_in_flight, oracle_path, to_bytes

pytestmark = pytest.mark.gpu
SEED = 1234


@pytest.fixture(scope="module")
def helios():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2310_00837_amd import helios as hl
    return hl


@pytest.mark.parametrize("cfg", [0, 1])
def test_recorded_batch_replays(helios, oracle, cfg):
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
    B = sp.batch
    hops = helios.alloc_hops(B, sp.fanouts, dev)
    cap = B + sum(hb.flat.numel() for hb in hops)
    h.reserve(cap)
    unique = torch.empty(cap, dtype=torch.int32, device=dev)
    inverse = torch.empty(cap, dtype=torch.int32, device=dev)
    out = torch.full((cap, sp.row_bytes), SENTINEL, dtype=torch.uint8, device=dev)
    mp = torch.empty(cap, dtype=torch.int32, device=dev)
    mi, ms = torch.empty_like(mp), torch.empty_like(mp)
    sizes = torch.zeros(2 * len(sp.fanouts), dtype=torch.int64).pin_memory()
    nu = torch.zeros(1, dtype=torch.int64).pin_memory()
    stats = torch.zeros(4, dtype=torch.int64).pin_memory()
    torch.cuda.synchronize()
    h.set_timing(1)                                      # the timing level is part of the recording
    plan = h.plan_create(B, sp.fanouts, hops, sizes, unique, inverse, nu, out, mp, mi, ms, stats)

    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    off, idx = g.offsets.numpy(), g.indices.numpy()
    rows = [torch.empty(hb.frontier.numel(), dtype=torch.int32, device=dev) for hb in hops]
    cols = [torch.empty(hb.flat.numel(), dtype=torch.int32, device=dev) for hb in hops]
    for b in range(6):
        seeds = W.seed_batch(sp, g, b).cuda()          # a fresh seed buffer every time
        rs = W.batch_rng_seed(SEED, b)
        out.fill_(SENTINEL)
        torch.cuda.synchronize()
        plan.launch(seeds, rs)
        h.make_blocks(hops, rows, cols)
        h.sync()
        hbm_ms, host_ms, _, _ = h.gather_times()
        assert hbm_ms > 0 and host_ms > 0
        want = oracle_path(oracle, off, idx, seeds.cpu().numpy(), sp.fanouts, rs, rank, n_hbm, n_host, *tabs, sp.row_bytes)
        U, nm = int(nu[0]), int(stats[3])
        got = dict(hops=[(hops[k].frontier[:int(sizes[2 * k])].cpu().numpy(), hops[k].indptr[:int(sizes[2 * k]) + 1].cpu().numpy(),
                          hops[k].flat[:int(sizes[2 * k + 1])].cpu().numpy()) for k in range(len(sp.fanouts))],
                   unique=unique[:U].cpu().numpy(), inverse=inverse[:want["inverse"].size].cpu().numpy(),
                   stats=stats.numpy().copy(), miss_pos=mp[:nm].cpu().numpy(), miss_id=mi[:nm].cpu().numpy(),
                   miss_slot=ms[:nm].cpu().numpy(), out_before_miss=out[:U].cpu().numpy())
        assert_same(got, want)
        nfl0 = int(sizes[1])
        assert np.array_equal(cols[0][:nfl0].cpu().numpy(), want["inverse"][B:B + nfl0])
        if b % 2 == 1:                                   # directly launched work between the replays
            eager = gpu_path(h, helios, seeds, sp.fanouts, rs + 1, fused=True)
            assert_same(eager, oracle_path(oracle, off, idx, seeds.cpu().numpy(), sp.fanouts, rs + 1, rank, n_hbm,
                                           n_host, *tabs, sp.row_bytes))
    # several replays queued without a sync in between: the last one wins the shared buffers
    for b in range(6, 10):
        plan.launch(W.seed_batch(sp, g, b).cuda(), W.batch_rng_seed(SEED, b))
    h.sync()
    want = oracle_path(oracle, off, idx, W.seed_batch(sp, g, 9).numpy(), sp.fanouts, W.batch_rng_seed(SEED, 9), rank,
                       n_hbm, n_host, *tabs, sp.row_bytes)
    assert np.array_equal(unique[:int(nu[0])].cpu().numpy(), want["unique"]) and stats.tolist() == want["stats"].tolist()
    # a context with a live plan is not destroyed
    assert helios._lib.helios_destroy(h._h) == helios.ESTATE
    # growing the scratch invalidates the plan
    h.reserve(4 * cap)
    with pytest.raises(helios.HeliosError) as e:
        plan.launch(W.seed_batch(sp, g, 0).cuda(), 1)
    assert e.value.code == helios.ESTATE
    plan.destroy()
    h.close()


def test_two_batches_queued_per_context(helios, oracle):
    """The benchmark's timed configuration: three contexts on three streams, two buffer sets and two
    recordings per context, a batch queued behind the running one, each waited for by helios_plan_wait."""
    sp = W.spec(1)
    g = W.make_graph(sp, SEED, "cpu")
    feats = W.feature_rows(SEED, torch.arange(g.n_nodes), sp.dim, sp.dtype)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    first = helios.Helios(0)
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    first.csr_load(off_d, idx_d)
    cache = GpuCache(first, feats, g.order, n_hbm, n_host)
    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]
    n_jobs = 48
    jobs = [(W.seed_batch(sp, g, b).cuda(), W.batch_rng_seed(SEED, b)) for b in range(n_jobs)]
    got = lanes_in_flight(helios, off_d, idx_d, cache.order, n_hbm, n_host, sp.row_bytes,
                          (cache.hbm, cache.host, cache.standin), sp.batch, sp.fanouts, jobs, per_lane=2)
    for b, res in enumerate(got):
        want = oracle_path(oracle, g.offsets.numpy(), g.indices.numpy(), jobs[b][0].cpu().numpy(), sp.fanouts, jobs[b][1],
                           rank, n_hbm, n_host, *tabs, sp.row_bytes)
        del want["out"]
        assert_same(res, want)
    first.close()


@pytest.mark.parametrize("params", [dict(split=1), dict(split=0, hbm_blocks=7, host_blocks=3), dict(split=1, hbm_blocks=8192, host_blocks=1), dict(split=0, hbm_blocks=1, host_blocks=300)])
def test_launch_parameters_do_not_change_results(helios, oracle, params):
    """The tuning parameters (tier copies as kernels of their own or as roles of the batch's other launches, grid
    sizes of the row copies) only change launch shapes: directly launched and recorded batches still match the oracle."""
    sp = W.spec(0)
    g = W.make_graph(sp, SEED, "cpu")
    feats = W.feature_rows(SEED, torch.arange(g.n_nodes), sp.dim, sp.dtype)
    n_hbm, n_host, _ = sp.tier_rows(g.n_nodes)
    first = helios.Helios(0)
    off_d, idx_d = g.offsets.cuda(), g.indices.cuda()
    first.csr_load(off_d, idx_d)
    cache = GpuCache(first, feats, g.order, n_hbm, n_host)
    order = g.order.numpy()
    rank = oracle.rank_build(order)
    by_rank = to_bytes(feats)[order]
    tabs = [np.ascontiguousarray(by_rank[:n_hbm]), np.ascontiguousarray(by_rank[n_hbm:n_hbm + n_host]),
            np.ascontiguousarray(by_rank[n_hbm + n_host:])]

    def tune(ctx):
        ctx.set_param(helios.PARAM_SPLIT_COPIES, params["split"])
        ctx.set_param(helios.PARAM_HBM_GATHER_BLOCKS, params.get("hbm_blocks", 0))
        ctx.set_param(helios.PARAM_HOST_GATHER_BLOCKS, params.get("host_blocks", 0))

    jobs = [(W.seed_batch(sp, g, b).cuda(), W.batch_rng_seed(SEED, b)) for b in range(6)]
    wants = [oracle_path(oracle, g.offsets.numpy(), g.indices.numpy(), sd.cpu().numpy(), sp.fanouts, rs, rank, n_hbm, n_host,
                         *tabs, sp.row_bytes) for sd, rs in jobs]
    for recorded in (False, True):
        got = lanes_in_flight(helios, off_d, idx_d, cache.order, n_hbm, n_host, sp.row_bytes,
                              (cache.hbm, cache.host, cache.standin), sp.batch, sp.fanouts, jobs, n_lanes=2,
                              recorded=recorded, tune=tune)
        for res, want in zip(got, wants):
            want = dict(want)
            del want["out_before_miss"]
            assert_same(res, want)
    first.close()


def test_plan_needs_a_real_stream(helios):
    h = helios.Helios(0)                                  # torch's default stream is the NULL stream
    off = torch.tensor([0, 1, 2], dtype=torch.int64, device="cuda")
    idx = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
    h.csr_load(off, idx)
    h.cache_build(torch.tensor([0, 1], dtype=torch.int32, device="cuda"), 2, 0, 16,
                  torch.zeros(32, dtype=torch.uint8, device="cuda"), None, None)
    h.sync()
    hops = helios.alloc_hops(1, [1], h.device)
    t = torch.zeros(8, dtype=torch.int32, device="cuda")
    p8 = torch.zeros(4, dtype=torch.int64).pin_memory()
    if torch.cuda.current_stream().cuda_stream == 0:
        with pytest.raises(helios.HeliosError) as e:
            h.plan_create(1, [1], hops, p8, t[:2], None, p8[:1].clone().pin_memory(), torch.zeros(2, 16, dtype=torch.uint8, device="cuda"),
                          t[2:4], t[4:6], t[6:8], p8.clone().pin_memory())
        assert e.value.code == helios.EINVAL
    h.close()
