// Host runtime and C ABI of the Helios library: context, scratch memory,
// launch order of the kernels, device-side error word.  See include/helios.h
// for the contract of every entry point.
#include "context.hpp"
#include "missq.hpp"
#include "noalloc.hpp"

using namespace helios;

namespace {

uint32_t pow2_at_least(int64_t n) {
    uint32_t p = 1024;
    while (static_cast<int64_t>(p) < n && p < (1u << 31)) p <<= 1;
    return p;
}

void free_scratch(helios_ctx* c) {
    (void)hipFree(c->dd.table);
    (void)hipFree(c->dd.slot_of);
    (void)hipFree(c->dd.index_of_first);
    for (int t = 0; t < 2; ++t) {
        (void)hipFree(c->list_pos[t]);
        (void)hipFree(c->list_slot[t]);
        c->list_pos[t] = c->list_slot[t] = nullptr;
    }
    (void)hipFree(c->cat);
    (void)hipFree(c->scan_status);
    (void)hipFree(c->hop_table[0]);
    (void)hipFree(c->hop_table[1]);
    (void)hipFree(c->hop_slot_of);
    c->hop_table[0] = c->hop_table[1] = nullptr;
    c->hop_slot_of = nullptr;
    c->dd = DedupScratch{nullptr, 0, nullptr, nullptr};
    c->cat = nullptr;
    c->scan_status = nullptr;
    c->cap_ids = 0;
    c->scan_stride = 0;
}

// Scratch for calls with up to n IDs.  Growing waits for the stream first: the
// old buffers may still be in use.
int ensure_capacity(helios_ctx* c, int64_t n) {
    if (n <= c->cap_ids) return HELIOS_OK;
    if (c->recording) return fail(c, HELIOS_ESTATE, "scratch must be reserved before a batch is recorded");
    c->scratch_generation += 1;
    if (n >= (1ll << 31) - 1024) return fail(c, HELIOS_EINVAL, "a call handles fewer than 2^31 IDs (got %lld)", (long long)n);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    free_scratch(c);
    const int64_t cap = (n + 4095) / 4096 * 4096;
    const uint32_t slots = pow2_at_least(2 * cap);
    const uint32_t stride = static_cast<uint32_t>(cap / kTileItems + 2);
    HIP_TRY(c, hipMalloc(&c->dd.table, sizeof(unsigned long long) * slots));
    HIP_TRY(c, hipMalloc(&c->dd.slot_of, sizeof(int32_t) * cap));
    HIP_TRY(c, hipMalloc(&c->dd.index_of_first, sizeof(int32_t) * cap));
    HIP_TRY(c, hipMalloc(&c->hop_table[0], sizeof(unsigned long long) * slots));
    HIP_TRY(c, hipMalloc(&c->hop_table[1], sizeof(unsigned long long) * slots));
    HIP_TRY(c, hipMalloc(&c->hop_slot_of, sizeof(int32_t) * cap));
    for (int t = 0; t < 2; ++t) {
        HIP_TRY(c, hipMalloc(&c->list_pos[t], sizeof(int32_t) * cap));
        HIP_TRY(c, hipMalloc(&c->list_slot[t], sizeof(int32_t) * cap));
    }
    HIP_TRY(c, hipMalloc(&c->cat, sizeof(int32_t) * cap));
    HIP_TRY(c, hipMalloc(&c->scan_status, sizeof(unsigned long long) * 3 * stride));
    HIP_TRY(c, hipMemsetAsync(c->scan_status, 0, sizeof(unsigned long long) * 3 * stride, c->stream));
    c->dd.n_slots = slots;
    c->scan_stride = stride;
    c->epoch = 0;
    c->cap_ids = cap;
    return HELIOS_OK;
}

// scan state with a fresh epoch; stale status words of earlier launches read as unpublished
int next_scan(helios_ctx* c, ScanState* out) {
    if (!c->recording && c->epoch >= (1u << 30) - 64) {
        HIP_TRY(c, hipMemsetAsync(c->scan_status, 0, sizeof(unsigned long long) * 3 * c->scan_stride, c->stream));
        c->epoch = 0;
    }
    if (c->recording) {                       // the batch's base epoch is added on the device
        c->rec_scans += 1;
        *out = ScanState{c->scan_status, c->scan_ticket, c->scan_stride, c->rec_scans, c->vars};
        return HELIOS_OK;
    }
    c->epoch += 1;
    *out = ScanState{c->scan_status, c->scan_ticket, c->scan_stride, c->epoch, nullptr};
    return HELIOS_OK;
}

int64_t sat_mul(int64_t a, int64_t b) {
    if (a == 0 || b == 0) return 0;
    if (a > (1ll << 40) / b) return 1ll << 40;
    return a * b;
}

struct HopPlan {
    int64_t frontier_max[HELIOS_MAX_HOPS];   // bound on |frontier h| that the buffers can hold
    int64_t flat_max[HELIOS_MAX_HOPS];       // bound on |flat h| that the buffers can hold
    int64_t cat_max;                         // n_seeds + sum flat_max
    int64_t ids_max;                         // the largest list any kernel of the call sees
};

int plan_hops(helios_ctx* c, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops, const helios_hop_out* hops,
              HopPlan* p) {
    if (n_seeds < 0) return fail(c, HELIOS_EINVAL, "n_seeds < 0");
    if (n_hops < 1 || n_hops > HELIOS_MAX_HOPS) return fail(c, HELIOS_EINVAL, "n_hops must be 1..%d", HELIOS_MAX_HOPS);
    if (!fanouts || !hops) return fail(c, HELIOS_EINVAL, "fanouts / hops is NULL");
    int64_t nf = n_seeds;
    p->cat_max = n_seeds;
    p->ids_max = n_seeds;
    for (int h = 0; h < n_hops; ++h) {
        const helios_hop_out& o = hops[h];
        if (fanouts[h] < 0 || fanouts[h] > HELIOS_MAX_FANOUT)
            return fail(c, HELIOS_EINVAL, "fanouts[%d] = %d outside 0..%d", h, fanouts[h], HELIOS_MAX_FANOUT);
        if (o.frontier_cap < 0 || o.flat_cap < 0) return fail(c, HELIOS_EINVAL, "negative capacity at hop %d", h);
        if (!o.indptr || (o.frontier_cap > 0 && !o.frontier) || (o.flat_cap > 0 && !o.flat))
            return fail(c, HELIOS_EINVAL, "hop %d: NULL output buffer", h);
        if (h == 0 && o.frontier_cap < n_seeds)
            return fail(c, HELIOS_EINVAL, "hops[0].frontier_cap (%lld) < n_seeds (%lld)", (long long)o.frontier_cap, (long long)n_seeds);
        if (nf > o.frontier_cap) nf = o.frontier_cap;
        p->frontier_max[h] = nf;
        int64_t fl = sat_mul(nf, fanouts[h]);
        if (fl > o.flat_cap) fl = o.flat_cap;
        p->flat_max[h] = fl;
        p->cat_max += fl;
        if (fl > p->ids_max) p->ids_max = fl;
        nf = fl;
    }
    if (p->cat_max > p->ids_max) p->ids_max = p->cat_max;
    return HELIOS_OK;
}

// slots of the hash table a de-duplication of up to n_max IDs uses (no more than it needs: a smaller
// table is cheaper to clear and stays in cache)
uint32_t dedup_slots(const helios_ctx* c, int64_t n_max) {
    const uint32_t want = pow2_at_least(2 * n_max);
    return want < c->dd.n_slots ? want : c->dd.n_slots;
}

SegLens one_segment(Count n) {
    SegLens lens{};
    lens.n_seg = 1;
    lens.len[0] = n;
    return lens;
}

// Hop 0: count pass over the seeds (it also empties the tables that the first sampling pass fills),
// sampling pass.  Hop h > 0: the de-duplication of flat_{h-1} yields frontier_h together with its
// indptr, then the sampling pass.  A sampling pass inserts its samples into the table of the
// de-duplication between this hop and the next, and, with batch_dedup_max > 0 (the whole-path call),
// into the table of the batch's ID list [seeds | flat_0 | ...], which c->cat receives; so those
// de-duplications start at their compaction pass.
int sample_impl(helios_ctx* c, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                uint64_t rng_seed, const helios_hop_out* hops, int64_t* sizes, const HopPlan& p,
                int64_t batch_dedup_max) {
    const BatchVars* vars = c->recording ? c->vars : nullptr;
    const BatchFeed feed = c->recording ? BatchFeed{c->vars_ring, kVarsRing, c->batches_run, c->vars}
                                        : BatchFeed{nullptr, 0, nullptr, nullptr};
    const InsertInto batch_table = batch_dedup_max > 0 ? InsertInto{c->dd.table, dedup_slots(c, batch_dedup_max), c->dd.slot_of}
                                                       : InsertInto{nullptr, 0, nullptr};
    auto hop_table = [&](int h) {               // hops alternate between two tables
        return h + 1 < n_hops ? InsertInto{c->hop_table[h % 2], dedup_slots(c, p.flat_max[h]), c->hop_slot_of}
                              : InsertInto{nullptr, 0, nullptr};
    };
    auto clear_of = [](const InsertInto& t) { return ClearJob{t.table, t.table ? t.n_slots : 0u}; };
    Count prev_flat[HELIOS_MAX_HOPS];
    Count nf{nullptr, n_seeds};
    {
        ScanState scan;
        int rc = next_scan(c, &scan);
        if (rc) return rc;
        HIP_TRY(c, launch_frontier_count(c->stream, c->g, seeds, feed, hops[0].frontier, nf, n_seeds, fanouts[0],
                                         hops[0].indptr, hops[0].flat_cap, c->cnt + kCntFlat + 0, sizes,
                                         clear_of(hop_table(0)), clear_of(batch_table), scan, c->err));
    }
    for (int h = 0; h < n_hops; ++h) {
        const bool last = h + 1 == n_hops;
        const InsertInto mine = hop_table(h);
        HIP_TRY(c, launch_sample_hop(c->stream, c->g, hops[h].frontier, hops[h].indptr, nf, p.frontier_max[h], fanouts[h],
                                     h, rng_seed, vars, hops[h].flat, p.flat_max[h], clear_of(hop_table(h + 1)), mine,
                                     batch_table, c->cat, n_seeds, prev_flat, c->recording ? c->batches_run : nullptr, c->err));
        prev_flat[h] = Count{c->cnt + kCntFlat + h, p.flat_max[h]};
        if (!last) {
            NextHopCount next{c->g.offsets, c->g.n_nodes, fanouts[h + 1], hops[h + 1].indptr, hops[h + 1].flat_cap,
                              c->cnt + kCntFlat + h + 1, sizes ? sizes + 2 * (h + 1) : nullptr};
            ScanState scan;
            int rc = next_scan(c, &scan);
            if (rc) return rc;
            const DedupScratch s{mine.table, mine.n_slots, mine.slot_of, c->dd.index_of_first};
            HIP_TRY(c, launch_dedup_compact(c->stream, hops[h].flat, one_segment(prev_flat[h]), p.flat_max[h],
                                            c->cnt + kCntHopTotal, s, hops[h + 1].frontier, hops[h + 1].frontier_cap,
                                            c->cnt + kCntFrontier + h + 1, nullptr, &next, nullptr, scan, c->err));
            nf = Count{c->cnt + kCntFrontier + h + 1, p.frontier_max[h + 1]};
        }
    }
    c->blocks_ready = false;
    return HELIOS_OK;
}

TierLists tier_lists(helios_ctx* c) {
    return TierLists{{c->list_pos[0], c->list_pos[1]}, {c->list_slot[0], c->list_slot[1]}, c->cnt + kCntTier};
}

int copy_tiers(helios_ctx* c, Count n, void* out);

int gather_impl(helios_ctx* c, const int32_t* ids, Count n, void* out, int32_t* miss_pos, int32_t* miss_id,
                int32_t* miss_slot, int64_t miss_cap, helios_gather_stats* stats) {
    ScanState scan;
    int rc = next_scan(c, &scan);
    if (rc) return rc;
    HIP_TRY(c, launch_lookup_partition(c->stream, ids, n, n.host, c->rank, c->g.n_nodes, c->n_hbm, c->n_host,
                                       tier_lists(c), miss_pos, miss_id, miss_slot, miss_cap,
                                       reinterpret_cast<int64_t*>(stats), scan, c->err));
    return copy_tiers(c, n, out);
}

// The two row copies over the per-tier lists that a lookup has left behind; n bounds the lists.
int copy_tiers(helios_ctx* c, Count n, void* out) {
    const TierLists lists = tier_lists(c);
    c->timed_hbm = c->timed_host = false;
    const bool do_hbm = c->n_hbm > 0 && n.host > 0, do_host = c->n_host > 0 && n.host > 0;
    const bool fork = do_host && !c->serial_tiers;
    hipStream_t host_stream = fork ? c->aux : c->stream;
    if (fork) {                                 // the host-tier copy runs beside the HBM-tier copy
        HIP_TRY(c, hipEventRecord(c->ev_fork, c->stream));
        HIP_TRY(c, hipStreamWaitEvent(c->aux, c->ev_fork, 0));
    }
    if (do_hbm) {
        if (c->timing > 1) HIP_TRY(c, hipEventRecord(c->t_hbm[0], c->stream));
        HIP_TRY(c, launch_gather_rows(c->stream, c->hbm_table, lists.pos[0], lists.slot[0],
                                      Count{c->cnt + kCntTier + 0, n.host}, n.host, c->row_bytes, out, false,
                                      c->timing ? c->clock : nullptr, &c->clock_blocks[0], c->hbm_blocks));
        if (c->timing) {
            if (c->timing > 1) HIP_TRY(c, hipEventRecord(c->t_hbm[1], c->stream));
            HIP_TRY(c, launch_clock_publish(c->stream, c->clock, c->clock_blocks[0], c->clock_host));
            c->timed_hbm = true;
        }
    }
    if (do_host) {
        if (c->timing > 1) HIP_TRY(c, hipEventRecord(c->t_host[0], host_stream));
        HIP_TRY(c, launch_gather_rows(host_stream, c->host_table, lists.pos[1], lists.slot[1],
                                      Count{c->cnt + kCntTier + 1, n.host}, n.host, c->row_bytes, out, true,
                                      c->timing ? c->clock + 2 * kGatherMaxBlocks : nullptr, &c->clock_blocks[1], c->host_blocks));
        if (c->timing) {
            if (c->timing > 1) HIP_TRY(c, hipEventRecord(c->t_host[1], host_stream));
            HIP_TRY(c, launch_clock_publish(host_stream, c->clock + 2 * kGatherMaxBlocks, c->clock_blocks[1],
                                            c->clock_host + 2));
            c->timed_host = true;
        }
        if (fork) {
            HIP_TRY(c, hipEventRecord(c->ev_join, c->aux));
            HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_join, 0));
        }
    }
    return HELIOS_OK;
}

}  // namespace

extern "C" {

int helios_create(helios_ctx** out, int device, void* hip_stream) {
    if (!out) return HELIOS_EINVAL;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return HELIOS_EHIP;
    DeviceGuard guard(device);
    if (!guard.ok) return HELIOS_EHIP;
    helios_ctx* c = new helios_ctx();
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    bool ok = hipStreamCreateWithFlags(&c->aux, hipStreamNonBlocking) == hipSuccess &&
              hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) == hipSuccess &&
              hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) == hipSuccess &&
              hipEventCreate(&c->t_hbm[0]) == hipSuccess && hipEventCreate(&c->t_hbm[1]) == hipSuccess &&
              hipEventCreate(&c->t_host[0]) == hipSuccess && hipEventCreate(&c->t_host[1]) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->err), 64, hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess &&
              hipMalloc(&c->cnt, sizeof(int64_t) * kNumCounters) == hipSuccess &&
              hipMalloc(&c->vars, sizeof(BatchVars)) == hipSuccess &&
              hipMalloc(&c->scan_ticket, 64) == hipSuccess &&
              hipMalloc(&c->batches_run, 64) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->vars_ring), sizeof(BatchVars) * kVarsRing,
                            hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess &&
              hipMalloc(&c->clock, sizeof(uint64_t) * 4 * kGatherMaxBlocks) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->clock_host), sizeof(uint64_t) * 4,
                            hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess;
    ok = ok && c->err && c->cnt && c->vars && c->scan_ticket && c->batches_run && c->vars_ring && c->clock && c->clock_host;
    ok = ok && noalloc_init(device) == HELIOS_OK;      // address of this device's static scratch (helios_dedup_noalloc)
    if (ok) {
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, device) == hipSuccess && khz > 0) c->clock_khz = khz;
        c->err[0] = c->err[1] = 0;
        ok = hipMemsetAsync(c->cnt, 0, sizeof(int64_t) * kNumCounters, c->stream) == hipSuccess &&
             hipMemsetAsync(c->scan_ticket, 0, 64, c->stream) == hipSuccess &&
             hipMemsetAsync(c->batches_run, 0, 64, c->stream) == hipSuccess &&
             hipStreamSynchronize(c->stream) == hipSuccess;
    }
    if (!ok) {
        helios_destroy(c);
        return HELIOS_EHIP;
    }
    *out = c;
    return HELIOS_OK;
}

int helios_destroy(helios_ctx* c) {
    if (!c) return HELIOS_EINVAL;
    if (c->n_children > 0)
        return fail(c, HELIOS_ESTATE, "%d plan(s) / miss queue(s) of this context are still alive; destroy them first", c->n_children);
    DeviceGuard guard(c->device);
    (void)hipStreamSynchronize(c->stream);
    if (c->aux) (void)hipStreamSynchronize(c->aux);
    free_scratch(c);
    (void)hipFree(c->rank);
    (void)hipFree(c->cnt);
    (void)hipFree(c->vars);
    (void)hipFree(c->scan_ticket);
    (void)hipFree(c->batches_run);
    if (c->vars_ring) (void)hipHostFree(c->vars_ring);
    (void)hipFree(c->clock);
    if (c->clock_host) (void)hipHostFree(c->clock_host);
    if (c->err) (void)hipHostFree(c->err);
    for (hipEvent_t e : {c->ev_fork, c->ev_join, c->t_hbm[0], c->t_hbm[1], c->t_host[0], c->t_host[1]})
        if (e) (void)hipEventDestroy(e);
    if (c->aux) (void)hipStreamDestroy(c->aux);
    delete c;
    return HELIOS_OK;
}

const char* helios_last_error(const helios_ctx* c) { return c ? c->errmsg : "no context"; }

int helios_reserve(helios_ctx* c, int64_t max_ids) {
    if (!c || max_ids < 0) return fail(c, HELIOS_EINVAL, "helios_reserve: bad argument");
    DeviceGuard guard(c->device);
    return ensure_capacity(c, max_ids);
}

// the device-side error word: reports and clears what kernels have recorded since the last check
static int check_device_error(helios_ctx* c) {
    const int code = *reinterpret_cast<volatile int32_t*>(c->err);
    if (code != 0) {
        c->err[0] = 0;
        return fail(c, code, code == HELIOS_ECAPACITY ? "an output did not fit its capacity"
                             : code == HELIOS_EINTERNAL ? "a workgroup gave up waiting (chained scan, or a miss queue that stopped answering)"
                             : "a node ID outside [0, n_nodes), or an order that is not a permutation");
    }
    return HELIOS_OK;
}

int helios_sync(helios_ctx* c) {
    if (!c) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->vars_unsynced = 0;
    return check_device_error(c);
}

int helios_csr_load(helios_ctx* c, int64_t n_nodes, int64_t n_edges, const int64_t* offsets, const int32_t* indices) {
    if (!c) return HELIOS_EINVAL;
    if (n_nodes < 0 || n_edges < 0 || n_nodes > 0x7fffffffLL) return fail(c, HELIOS_EINVAL, "bad graph size");
    if (!offsets || (n_edges > 0 && !indices)) return fail(c, HELIOS_EINVAL, "offsets / indices is NULL");
    c->g = CsrView{offsets, indices, n_nodes};
    c->n_edges = n_edges;
    c->has_graph = true;
    c->has_cache = false;              // the cache map belongs to the graph it was built for
    return HELIOS_OK;
}

int helios_cache_build(helios_ctx* c, const int32_t* order, int64_t hbm_rows, int64_t host_rows, int32_t row_bytes,
                       const void* hbm_table, const void* host_table, const void* standin_table) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph) return fail(c, HELIOS_ESTATE, "helios_cache_build before helios_csr_load");
    if (!order && c->g.n_nodes > 0) return fail(c, HELIOS_EINVAL, "hotness_order is NULL");
    if (hbm_rows < 0 || host_rows < 0) return fail(c, HELIOS_EINVAL, "negative tier size");
    if (row_bytes <= 0 || row_bytes % 16 != 0) return fail(c, HELIOS_EINVAL, "row_bytes must be a positive multiple of 16");
    const int64_t n = c->g.n_nodes;
    if (hbm_rows > n) hbm_rows = n;
    if (host_rows > n - hbm_rows) host_rows = n - hbm_rows;
    if ((hbm_rows > 0 && !hbm_table) || (host_rows > 0 && !host_table))
        return fail(c, HELIOS_EINVAL, "a tier with rows has a NULL table");
    DeviceGuard guard(c->device);
    if (n > c->rank_cap) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        (void)hipFree(c->rank);
        c->rank = nullptr;
        c->rank_cap = 0;
        HIP_TRY(c, hipMalloc(&c->rank, sizeof(int32_t) * (n > 0 ? n : 1)));
        c->rank_cap = n;
    }
    if (n > 0) HIP_TRY(c, launch_rank_build(c->stream, order, n, c->rank, c->err));
    c->n_hbm = hbm_rows;
    c->n_host = host_rows;
    c->row_bytes = row_bytes;
    c->hbm_table = hbm_table;
    c->host_table = host_table;
    c->standin_table = standin_table;
    c->has_cache = true;
    c->cache_generation += 1;
    return HELIOS_OK;
}

int helios_cache_fill(helios_ctx* c, const void* src_table, const int32_t* order, int64_t first_rank, int64_t n_rows,
                      int32_t row_bytes, void* dst) {
    if (!c) return HELIOS_EINVAL;
    if (n_rows < 0 || first_rank < 0) return fail(c, HELIOS_EINVAL, "negative row range");
    if (row_bytes <= 0 || row_bytes % 16 != 0) return fail(c, HELIOS_EINVAL, "row_bytes must be a positive multiple of 16");
    if (n_rows == 0) return HELIOS_OK;
    if (!src_table || !order || !dst) return fail(c, HELIOS_EINVAL, "NULL pointer");
    DeviceGuard guard(c->device);
    HIP_TRY(c, launch_gather_rows(c->stream, src_table, nullptr, order + first_rank, Count{nullptr, n_rows}, n_rows,
                                  row_bytes, dst, false, nullptr, nullptr, 0));
    return HELIOS_OK;
}

int helios_sample(helios_ctx* c, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                  uint64_t rng_seed, const helios_hop_out* hops, int64_t* sizes) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph) return fail(c, HELIOS_ESTATE, "helios_sample before helios_csr_load");
    HopPlan p;
    int rc = plan_hops(c, n_seeds, fanouts, n_hops, hops, &p);
    if (rc) return rc;
    if (n_seeds > 0 && !seeds) return fail(c, HELIOS_EINVAL, "seeds is NULL");
    DeviceGuard guard(c->device);
    rc = ensure_capacity(c, p.ids_max);
    if (rc) return rc;
    return sample_impl(c, seeds, n_seeds, fanouts, n_hops, rng_seed, hops, sizes, p, 0);
}

int helios_dedup(helios_ctx* c, const int32_t* ids, int64_t n_ids, int32_t* unique, int64_t unique_cap,
                 int32_t* inverse, int64_t* n_unique) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph) return fail(c, HELIOS_ESTATE, "helios_dedup before helios_csr_load");
    if (n_ids < 0 || unique_cap < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if ((n_ids > 0 && !ids) || (unique_cap > 0 && !unique)) return fail(c, HELIOS_EINVAL, "NULL pointer");
    DeviceGuard guard(c->device);
    int rc = ensure_capacity(c, n_ids);
    if (rc) return rc;
    ScanState scan;
    rc = next_scan(c, &scan);
    if (rc) return rc;
    DedupScratch s = c->dd;
    s.n_slots = dedup_slots(c, n_ids);
    c->blocks_ready = false;
    c->last_slots = s.n_slots;
    const Count n{nullptr, n_ids};
    HIP_TRY(c, launch_dedup_insert(c->stream, ids, n, n_ids, c->g.n_nodes, s, false, c->err));
    HIP_TRY(c, launch_dedup_compact(c->stream, ids, one_segment(n), n_ids, c->cnt + kCntCat, s, unique, unique_cap,
                                    c->cnt + kCntUnique, n_unique, nullptr, nullptr, scan, c->err));
    if (inverse) HIP_TRY(c, launch_dedup_inverse(c->stream, c->cnt + kCntCat, n_ids, s, inverse));
    return HELIOS_OK;
}

int helios_gather(helios_ctx* c, const int32_t* ids, int64_t n_ids, void* out, int32_t* miss_pos, int32_t* miss_id,
                  int32_t* miss_slot, int64_t miss_cap, helios_gather_stats* stats) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_cache) return fail(c, HELIOS_ESTATE, "helios_gather before helios_cache_build");
    if (n_ids < 0 || miss_cap < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (n_ids > 0 && (!ids || !out)) return fail(c, HELIOS_EINVAL, "NULL pointer");
    if (miss_cap > 0 && (!miss_pos || !miss_id || !miss_slot)) return fail(c, HELIOS_EINVAL, "NULL miss list");
    DeviceGuard guard(c->device);
    int rc = ensure_capacity(c, n_ids);
    if (rc) return rc;
    return gather_impl(c, ids, Count{nullptr, n_ids}, out, miss_pos, miss_id, miss_slot, miss_cap, stats);
}

int helios_gather_miss(helios_ctx* c, const int32_t* miss_pos, const int32_t* miss_slot, int64_t n_miss_max,
                       const int64_t* n_miss_dev, void* out) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_cache) return fail(c, HELIOS_ESTATE, "helios_gather_miss before helios_cache_build");
    if (n_miss_max < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (n_miss_max == 0) return HELIOS_OK;
    if (!miss_pos || !miss_slot || !out) return fail(c, HELIOS_EINVAL, "NULL pointer");
    if (c->n_hbm + c->n_host >= c->g.n_nodes) return HELIOS_OK;      // every node is cached: nothing can miss
    if (!c->standin_table) return fail(c, HELIOS_ESTATE, "no stand-in table was given to helios_cache_build");
    DeviceGuard guard(c->device);
    HIP_TRY(c, launch_gather_rows(c->stream, c->standin_table, miss_pos, miss_slot, Count{n_miss_dev, n_miss_max},
                                  n_miss_max, c->row_bytes, out, true, nullptr, nullptr, c->host_blocks));
    return HELIOS_OK;
}

static int prepare_batch_impl(helios_ctx* c, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                         uint64_t rng_seed, const helios_hop_out* hops, int64_t* sizes, int32_t* unique,
                         int64_t unique_cap, int32_t* inverse, int64_t* n_unique, void* out, int32_t* miss_pos,
                         int32_t* miss_id, int32_t* miss_slot, int64_t miss_cap, helios_gather_stats* stats) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph || !c->has_cache) return fail(c, HELIOS_ESTATE, "helios_prepare_batch needs the graph and the cache");
    HopPlan p;
    int rc = plan_hops(c, n_seeds, fanouts, n_hops, hops, &p);
    if (rc) return rc;
    if (n_seeds > 0 && !seeds) return fail(c, HELIOS_EINVAL, "seeds is NULL");
    if (unique_cap < 0 || miss_cap < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (unique_cap > 0 && (!unique || !out)) return fail(c, HELIOS_EINVAL, "NULL pointer");
    if (miss_cap > 0 && (!miss_pos || !miss_id || !miss_slot)) return fail(c, HELIOS_EINVAL, "NULL miss list");
    rc = ensure_capacity(c, p.ids_max);
    if (rc) return rc;
    const int64_t batch_max = p.cat_max > 0 ? p.cat_max : 1;
    rc = sample_impl(c, seeds, n_seeds, fanouts, n_hops, rng_seed, hops, sizes, p, batch_max);
    if (rc) return rc;
    SegLens lens{};
    lens.n_seg = n_hops + 1;
    lens.len[0] = Count{nullptr, n_seeds};
    for (int h = 0; h < n_hops; ++h) lens.len[h + 1] = Count{c->cnt + kCntFlat + h, p.flat_max[h]};
    // the sampling passes have filled the table; the compaction classifies the unique IDs by cache tier on the way
    LookupOut look{c->rank, c->n_hbm, c->n_host, tier_lists(c), miss_pos, miss_id, miss_slot, miss_cap,
                   reinterpret_cast<int64_t*>(stats)};
    ScanState scan;
    rc = next_scan(c, &scan);
    if (rc) return rc;
    DedupScratch s = c->dd;
    s.n_slots = dedup_slots(c, batch_max);
    c->last_slots = s.n_slots;
    HIP_TRY(c, launch_dedup_compact(c->stream, c->cat, lens, p.cat_max, c->cnt + kCntCat, s, unique, unique_cap,
                                    c->cnt + kCntUnique, n_unique, nullptr, &look, scan, c->err));
    const int64_t u_max = p.cat_max < unique_cap ? p.cat_max : unique_cap;
    if (c->missq) {                 // the misses are on their way while the cached tiers are copied
        const int64_t m_max = miss_cap < u_max ? miss_cap : u_max;
        rc = missq_submit_from_batch(c, miss_pos, miss_slot, Count{c->cnt + kCntTier + 2, m_max}, m_max);
        if (rc) return rc;
    }
    c->blocks_ready = true;
    c->last_n_seeds = n_seeds;
    c->last_n_hops = n_hops;
    for (int h = 0; h < n_hops; ++h) {
        c->last_frontier_max[h] = p.frontier_max[h];
        c->last_flat_max[h] = p.flat_max[h];
    }
    rc = copy_tiers(c, Count{c->cnt + kCntUnique, u_max}, out);
    if (rc) return rc;
    // last, so that the row copies (and with them the host link) start one launch earlier
    if (inverse) HIP_TRY(c, launch_dedup_inverse(c->stream, c->cnt + kCntCat, p.cat_max, s, inverse));
    return HELIOS_OK;
}

int helios_prepare_batch(helios_ctx* c, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                         uint64_t rng_seed, const helios_hop_out* hops, int64_t* sizes, int32_t* unique,
                         int64_t unique_cap, int32_t* inverse, int64_t* n_unique, void* out, int32_t* miss_pos,
                         int32_t* miss_id, int32_t* miss_slot, int64_t miss_cap, helios_gather_stats* stats) {
    if (!c) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    return prepare_batch_impl(c, seeds, n_seeds, fanouts, n_hops, rng_seed, hops, sizes, unique, unique_cap, inverse,
                              n_unique, out, miss_pos, miss_id, miss_slot, miss_cap, stats);
}

struct helios_plan {
    helios_ctx* ctx = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    uint32_t n_scans = 0;
    uint64_t scratch_generation = 0;
    int64_t n_seeds = 0;
    int32_t n_hops = 0;
    int64_t frontier_max[HELIOS_MAX_HOPS] = {0};
    int64_t flat_max[HELIOS_MAX_HOPS] = {0};
    uint32_t slots = 0;
    helios_missq* missq = nullptr;     // the queue attached when the batch was recorded
    hipEvent_t done = nullptr;         // recorded behind every launch
    uint64_t launch_seq = 0;           // the context's launch count at this plan's last launch
};

int helios_plan_create(helios_ctx* c, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                       const helios_hop_out* hops, int64_t* sizes, int32_t* unique, int64_t unique_cap,
                       int32_t* inverse, int64_t* n_unique, void* out, int32_t* miss_pos, int32_t* miss_id,
                       int32_t* miss_slot, int64_t miss_cap, helios_gather_stats* stats, helios_plan** plan_out) {
    if (!c || !plan_out) return HELIOS_EINVAL;
    *plan_out = nullptr;
    if (!c->has_graph || !c->has_cache) return fail(c, HELIOS_ESTATE, "helios_plan_create needs the graph and the cache");
    if (!c->stream) return fail(c, HELIOS_EINVAL, "a batch cannot be recorded on the default (NULL) stream");
    if (c->timing > 1) return fail(c, HELIOS_ESTATE, "event timing cannot be recorded; use timing level 0 or 1");
    DeviceGuard guard(c->device);
    HopPlan p;
    int rc = plan_hops(c, n_seeds, fanouts, n_hops, hops, &p);
    if (rc) return rc;
    rc = ensure_capacity(c, p.ids_max);          // allocate before recording starts
    if (rc) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    helios_plan* pl = new helios_plan();
    pl->ctx = c;
    c->recording = true;
    c->rec_scans = 0;
    hipError_t e = hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal);
    if (e == hipSuccess) {
        // the seeds pointer and rng_seed passed here are placeholders: recorded kernels read both from c->vars
        rc = prepare_batch_impl(c, reinterpret_cast<const int32_t*>(c->vars), n_seeds, fanouts, n_hops, 0, hops, sizes,
                                unique, unique_cap, inverse, n_unique, out, miss_pos, miss_id, miss_slot, miss_cap, stats);
        hipError_t e2 = hipStreamEndCapture(c->stream, &pl->graph);
        if (rc == HELIOS_OK && e2 != hipSuccess) e = e2;
    }
    c->recording = false;
    pl->n_scans = c->rec_scans;
    if (e == hipSuccess && rc == HELIOS_OK) e = hipGraphInstantiate(&pl->exec, pl->graph, nullptr, nullptr, 0);
    if (e == hipSuccess && rc == HELIOS_OK) e = hipEventCreateWithFlags(&pl->done, hipEventDisableTiming);
    if (e != hipSuccess || rc != HELIOS_OK) {
        if (pl->exec) (void)hipGraphExecDestroy(pl->exec);
        if (pl->graph) (void)hipGraphDestroy(pl->graph);
        delete pl;
        c->blocks_ready = false;
        if (rc != HELIOS_OK) return rc;
        return fail(c, HELIOS_EHIP, "recording the batch failed: %s", hipGetErrorString(e));
    }
    pl->scratch_generation = c->scratch_generation;
    pl->n_seeds = n_seeds;
    pl->n_hops = n_hops;
    for (int h = 0; h < n_hops; ++h) {
        pl->frontier_max[h] = p.frontier_max[h];
        pl->flat_max[h] = p.flat_max[h];
    }
    pl->slots = c->last_slots;
    pl->missq = c->missq;
    c->blocks_ready = false;                     // nothing has run yet
    c->n_children += 1;
    *plan_out = pl;
    return HELIOS_OK;
}

int helios_plan_launch(helios_plan* pl, const int32_t* seeds, uint64_t rng_seed) {
    if (!pl || !pl->ctx) return HELIOS_EINVAL;
    helios_ctx* c = pl->ctx;
    if (pl->n_seeds > 0 && !seeds) return fail(c, HELIOS_EINVAL, "seeds is NULL");
    if (pl->scratch_generation != c->scratch_generation)
        return fail(c, HELIOS_ESTATE, "the context's scratch was regrown after the batch was recorded; record it again");
    if (pl->missq != c->missq)
        return fail(c, HELIOS_ESTATE, "the miss queue attached to the context is not the one the batch was recorded with");
    DeviceGuard guard(c->device);
    uint32_t io_round = 0;
    if (pl->missq) {
        int rc = missq_open_round(c, pl->missq, &io_round);
        if (rc) return rc;
    }
    if (c->epoch + pl->n_scans >= (1u << 30) - 64) {
        HIP_TRY(c, hipMemsetAsync(c->scan_status, 0, sizeof(unsigned long long) * 3 * c->scan_stride, c->stream));
        c->epoch = 0;
    }
    if (c->vars_unsynced + 1 >= kVarsRing) {     // the ring slot about to be reused may still be in flight
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        c->vars_unsynced = 0;
    }
    BatchVars* slot = c->vars_ring + (c->vars_next % kVarsRing);
    slot->rng_seed = rng_seed;
    slot->seeds = seeds;
    slot->epoch_base = c->epoch;
    slot->io_round = io_round;
    __atomic_thread_fence(__ATOMIC_RELEASE);     // the slot is written before the launch is rung in
    HIP_TRY(c, hipGraphLaunch(pl->exec, c->stream));
    // only a batch that was launched takes its slot: the device counts the batches it runs, and the two
    // counts select the slot
    c->vars_next += 1;
    c->vars_unsynced += 1;
    c->epoch += pl->n_scans;
    HIP_TRY(c, hipEventRecord(pl->done, c->stream));
    c->launch_seq += 1;
    pl->launch_seq = c->launch_seq;
    c->blocks_ready = true;
    c->last_slots = pl->slots;
    c->last_n_seeds = pl->n_seeds;
    c->last_n_hops = pl->n_hops;
    for (int h = 0; h < pl->n_hops; ++h) {
        c->last_frontier_max[h] = pl->frontier_max[h];
        c->last_flat_max[h] = pl->flat_max[h];
    }
    c->timed_hbm = c->timing != 0 && c->n_hbm > 0 && pl->n_seeds > 0;
    c->timed_host = c->timing != 0 && c->n_host > 0 && pl->n_seeds > 0;
    return HELIOS_OK;
}

int helios_plan_wait(helios_plan* pl) {
    if (!pl || !pl->ctx) return HELIOS_EINVAL;
    helios_ctx* c = pl->ctx;
    if (pl->launch_seq == 0) return HELIOS_OK;           // never launched
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipEventSynchronize(pl->done));
    // everything launched on the context up to this plan's launch has finished
    const uint64_t later = c->launch_seq - pl->launch_seq;
    if (later < c->vars_unsynced) c->vars_unsynced = static_cast<uint32_t>(later);
    return check_device_error(c);
}

int helios_plan_destroy(helios_plan* pl) {
    if (!pl) return HELIOS_EINVAL;
    if (pl->ctx) {
        DeviceGuard guard(pl->ctx->device);
        (void)hipStreamSynchronize(pl->ctx->stream);
        pl->ctx->n_children -= 1;
    }
    if (pl->exec) (void)hipGraphExecDestroy(pl->exec);
    if (pl->graph) (void)hipGraphDestroy(pl->graph);
    if (pl->done) (void)hipEventDestroy(pl->done);
    delete pl;
    return HELIOS_OK;
}

int helios_make_blocks(helios_ctx* c, const helios_hop_out* hops, int32_t n_hops, const helios_block_out* blocks) {
    if (!c) return HELIOS_EINVAL;
    if (!c->blocks_ready) return fail(c, HELIOS_ESTATE, "helios_make_blocks must follow helios_prepare_batch on this context");
    if (!hops || !blocks || n_hops != c->last_n_hops) return fail(c, HELIOS_EINVAL, "hops / blocks do not match the last batch");
    DeviceGuard guard(c->device);
    DedupScratch s = c->dd;
    s.n_slots = c->last_slots;
    for (int h = 0; h < n_hops; ++h) {
        if (!blocks[h].row_local || !blocks[h].col_local) return fail(c, HELIOS_EINVAL, "hop %d: NULL block buffer", h);
        const Count nf = h == 0 ? Count{nullptr, c->last_n_seeds} : Count{c->cnt + kCntFrontier + h, c->last_frontier_max[h]};
        HIP_TRY(c, launch_local_ids(c->stream, hops[h].frontier, nf, c->last_frontier_max[h], s, blocks[h].row_local, c->err));
        HIP_TRY(c, launch_local_ids(c->stream, hops[h].flat, Count{c->cnt + kCntFlat + h, c->last_flat_max[h]},
                                    c->last_flat_max[h], s, blocks[h].col_local, c->err));
    }
    return HELIOS_OK;
}

int helios_hotness_add(helios_ctx* c, const int32_t* ids, int64_t n_max, const int64_t* n_dev, int32_t* counts) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph) return fail(c, HELIOS_ESTATE, "helios_hotness_add before helios_csr_load");
    if (n_max < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (n_max == 0) return HELIOS_OK;
    if (!ids || !counts) return fail(c, HELIOS_EINVAL, "NULL pointer");
    DeviceGuard guard(c->device);
    HIP_TRY(c, launch_hotness_add(c->stream, ids, Count{n_dev, n_max}, n_max, c->g.n_nodes, counts, c->err));
    return HELIOS_OK;
}

int helios_hotness_order(helios_ctx* c, const int32_t* counts, int32_t* order) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph) return fail(c, HELIOS_ESTATE, "helios_hotness_order before helios_csr_load");
    const int64_t n = c->g.n_nodes;
    if (n == 0) return HELIOS_OK;
    if (!counts || !order) return fail(c, HELIOS_EINVAL, "NULL pointer");
    DeviceGuard guard(c->device);
    const size_t temp_bytes = hotness_order_temp_bytes(n);
    void* temp = nullptr;
    int32_t *ids_in = nullptr, *counts_sorted = nullptr;
    HIP_TRY(c, hipMalloc(&temp, temp_bytes ? temp_bytes : 16));
    hipError_t e = hipMalloc(&ids_in, sizeof(int32_t) * n);
    if (e == hipSuccess) e = hipMalloc(&counts_sorted, sizeof(int32_t) * n);
    if (e == hipSuccess) e = launch_hotness_order(c->stream, counts, n, ids_in, counts_sorted, order, temp, temp_bytes);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);     // the scratch is freed below
    (void)hipFree(temp);
    (void)hipFree(ids_in);
    (void)hipFree(counts_sorted);
    if (e != hipSuccess) return fail(c, HELIOS_EHIP, "helios_hotness_order: %s", hipGetErrorString(e));
    return HELIOS_OK;
}

int helios_calibration_copy(helios_ctx* c, const void* src, void* dst, int64_t bytes) {
    if (!c || !src || !dst || bytes < 0 || bytes % 16 != 0) return fail(c, HELIOS_EINVAL, "helios_calibration_copy: bad argument");
    DeviceGuard guard(c->device);
    HIP_TRY(c, launch_calibration_copy(c->stream, src, dst, bytes));
    return HELIOS_OK;
}

void* helios_host_alloc(int64_t bytes) {
    if (bytes <= 0) return nullptr;
    void* p = nullptr;
    if (hipHostMalloc(&p, static_cast<size_t>(bytes), hipHostMallocMapped | hipHostMallocPortable) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return p;
}

int helios_host_free(void* p) {
    if (!p) return HELIOS_OK;
    return hipHostFree(p) == hipSuccess ? HELIOS_OK : HELIOS_EHIP;
}

int helios_set_param(helios_ctx* c, int param, int64_t value) {
    if (!c) return HELIOS_EINVAL;
    if (value < 0) return fail(c, HELIOS_EINVAL, "helios_set_param: negative value");
    switch (param) {
        case HELIOS_PARAM_HBM_GATHER_BLOCKS:
            c->hbm_blocks = static_cast<unsigned>(value > kGatherMaxBlocks ? kGatherMaxBlocks : value);
            return HELIOS_OK;
        case HELIOS_PARAM_HOST_GATHER_BLOCKS:
            c->host_blocks = static_cast<unsigned>(value > kGatherMaxBlocks ? kGatherMaxBlocks : value);
            return HELIOS_OK;
        case HELIOS_PARAM_SERIAL_TIERS:
            c->serial_tiers = value != 0;
            return HELIOS_OK;
        case HELIOS_PARAM_MISSQ_TIMEOUT_US:
            c->missq_timeout_us = value < 1 ? 1 : value > 60000000 ? 60000000 : value;
            return HELIOS_OK;
        case HELIOS_PARAM_MISSQ_WAVES:
            c->missq_waves = static_cast<unsigned>(value > 4096 ? 4096 : value);
            return HELIOS_OK;
        default:
            return fail(c, HELIOS_EINVAL, "helios_set_param: unknown parameter %d", param);
    }
}

int helios_set_timing(helios_ctx* c, int enabled) {
    if (!c) return HELIOS_EINVAL;
    c->timing = enabled < 0 ? 0 : enabled > 2 ? 2 : enabled;
    c->timed_hbm = c->timed_host = false;
    return HELIOS_OK;
}

int helios_gather_times(helios_ctx* c, float* hbm_ms, float* host_ms, float* hbm_event_ms, float* host_event_ms) {
    if (!c || !hbm_ms || !host_ms) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    *hbm_ms = *host_ms = 0.f;
    if (hbm_event_ms) *hbm_event_ms = 0.f;
    if (host_event_ms) *host_event_ms = 0.f;
    if (!c->timed_hbm && !c->timed_host) return HELIOS_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));          // the publish kernels have written the pinned words
    for (int t = 0; t < 2; ++t) {
        if (!(t == 0 ? c->timed_hbm : c->timed_host)) continue;
        const volatile uint64_t* k = c->clock_host + 2 * t;
        const uint64_t lo = k[0], hi = k[1];
        const float ms = hi >= lo && lo != ~0ull ? static_cast<float>(static_cast<double>(hi - lo) / c->clock_khz) : 0.f;
        float ev = 0.f;
        if (c->timing > 1)
            HIP_TRY(c, hipEventElapsedTime(&ev, t == 0 ? c->t_hbm[0] : c->t_host[0], t == 0 ? c->t_hbm[1] : c->t_host[1]));
        if (t == 0) { *hbm_ms = ms; if (hbm_event_ms) *hbm_event_ms = ev; }
        else { *host_ms = ms; if (host_event_ms) *host_event_ms = ev; }
    }
    return HELIOS_OK;
}

int helios_gather_ticks(helios_ctx* c, uint64_t* ticks4, double* ticks_per_us) {
    if (!c || !ticks4) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    for (int i = 0; i < 4; ++i) ticks4[i] = 0;
    if (ticks_per_us) *ticks_per_us = c->clock_khz / 1000.0;
    if (!c->timed_hbm && !c->timed_host) return HELIOS_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int t = 0; t < 2; ++t) {
        if (!(t == 0 ? c->timed_hbm : c->timed_host)) continue;
        const volatile uint64_t* k = c->clock_host + 2 * t;
        if (k[0] != ~0ull && k[1] >= k[0]) {
            ticks4[2 * t] = k[0];
            ticks4[2 * t + 1] = k[1];
        }
    }
    return HELIOS_OK;
}

}  // extern "C"
