// Host runtime and C ABI of the Helios library: context, scratch memory,
// launch order of the kernels, device-side error word.  See include/helios.h
// for the contract of every entry point.
#include "context.hpp"
#include "missq.hpp"
#include "noalloc.hpp"

#include <algorithm>

using namespace helios;

static_assert(kMaxGang == HELIOS_MAX_GANG, "the header's limit is the kernels' limit");

struct helios_plan {
    helios_ctx* ctx = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    uint32_t n_scans = 0;
    uint64_t scratch_generation = 0;
    uint64_t cache_generation = 0, graph_generation = 0;   // the recording holds the graph's and the cache's pointers and sizes
    int64_t n_seeds = 0;
    int32_t n_hops = 0;
    int64_t frontier_max[HELIOS_MAX_HOPS] = {0};
    int64_t flat_max[HELIOS_MAX_HOPS] = {0};
    helios_hop_out hops[HELIOS_MAX_HOPS] = {};
    const int64_t* sizes = nullptr;    // the caller's size array (device-accessible, nullable)
    uint32_t slots = 0;                // slots of the batch table the recording uses
    uint32_t clear_slots = 0;          // slots of the next batch's table it empties on the way
    helios_missq* missq = nullptr;     // the queue attached when the batch was recorded
    hipEvent_t done = nullptr;         // recorded behind every launch
    uint64_t launch_seq = 0;           // the context's launch count at this plan's last launch
    uint64_t batch_seq = 0;            // the context's batch count right after this plan's last launch
    int32_t* err = nullptr;            // pinned int32[2]: the device-side error word of this plan's batches
    StampRole stamp_roles[kMaxStampRoles];
    StampTable stamp_table{};
    int n_stamps = 0;
    helios_gang* gang = nullptr;       // the gang this plan is a member of: it owns the recording and the event
};

// Mini-batches of several contexts recorded into the same launches (see helios_gang_create).
struct helios_gang {
    int n = 0;
    helios_plan* member[kMaxGang] = {nullptr, nullptr, nullptr, nullptr};
    int device = 0;
    hipStream_t stream = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipEvent_t done = nullptr;
    bool launched = false;
};

namespace {

uint32_t pow2_at_least(int64_t n) {
    uint32_t p = 1024;
    while (static_cast<int64_t>(p) < n && p < (1u << 31)) p <<= 1;
    return p;
}

void free_scratch(helios_ctx* c) {
    (void)hipFree(c->batch_tables);
    (void)hipFree(c->batch_iof);
    (void)hipFree(c->batch_slot_of);
    for (int t = 0; t < 2; ++t) {
        (void)hipFree(c->list_pos[t]);
        (void)hipFree(c->list_slot[t]);
        (void)hipFree(c->hop_table[t]);
        c->list_pos[t] = c->list_slot[t] = nullptr;
        c->hop_table[t] = nullptr;
    }
    (void)hipFree(c->cat);
    (void)hipFree(c->scan_status);
    (void)hipFree(c->hop_slot_of);
    c->batch_tables = nullptr;
    c->batch_iof = c->batch_slot_of = c->hop_slot_of = c->cat = nullptr;
    c->scan_status = nullptr;
    c->cap_ids = 0;
    c->table_slots = 0;
    c->scan_stride = 0;
}

unsigned long long* batch_table(const helios_ctx* c, uint32_t t) { return c->batch_tables + static_cast<size_t>(t) * c->table_slots; }
int32_t* batch_iof(const helios_ctx* c, uint32_t t) { return c->batch_iof + static_cast<size_t>(t) * c->cap_ids; }

// Scratch for calls with up to n IDs.  Growing waits for the stream first: the
// old buffers may still be in use.  Every hash table starts out empty.
int ensure_capacity(helios_ctx* c, int64_t n) {
    if (n < 1) n = 1;                           // an empty call still gets its (smallest) scratch
    if (n <= c->cap_ids) return HELIOS_OK;
    if (c->recording) return fail(c, HELIOS_ESTATE, "scratch must be reserved before a batch is recorded");
    c->scratch_generation += 1;
    if (n >= (1ll << 31) - 1024) return fail(c, HELIOS_EINVAL, "a call handles fewer than 2^31 IDs (got %lld)", (long long)n);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    free_scratch(c);
    c->blocks_ready = false;
    const int64_t cap = (n + 4095) / 4096 * 4096;
    const uint32_t slots = pow2_at_least(2 * cap);
    const uint32_t stride = static_cast<uint32_t>(cap / kTileItems + 2);
    HIP_TRY(c, hipMalloc(&c->batch_tables, sizeof(unsigned long long) * slots * kBatchTables));
    HIP_TRY(c, hipMalloc(&c->batch_iof, sizeof(int32_t) * cap * kBatchTables));
    HIP_TRY(c, hipMalloc(&c->batch_slot_of, sizeof(int32_t) * cap));
    HIP_TRY(c, hipMalloc(&c->hop_table[0], sizeof(unsigned long long) * slots));
    HIP_TRY(c, hipMalloc(&c->hop_table[1], sizeof(unsigned long long) * slots));
    HIP_TRY(c, hipMalloc(&c->hop_slot_of, sizeof(int32_t) * cap));
    for (int t = 0; t < 2; ++t) {
        HIP_TRY(c, hipMalloc(&c->list_pos[t], sizeof(int32_t) * cap));
        HIP_TRY(c, hipMalloc(&c->list_slot[t], sizeof(int32_t) * cap));
    }
    HIP_TRY(c, hipMalloc(&c->cat, sizeof(int32_t) * cap));
    HIP_TRY(c, hipMalloc(&c->scan_status, sizeof(unsigned long long) * kScanRows * stride));
    HIP_TRY(c, hipMemsetAsync(c->scan_status, 0, sizeof(unsigned long long) * kScanRows * stride, c->stream));
    c->table_slots = slots;
    c->scan_stride = stride;
    c->epoch = 0;
    c->cap_ids = cap;
    for (uint32_t t = 0; t < kBatchTables; ++t) {
        HIP_TRY(c, launch_clear(c->stream, ClearJob{batch_table(c, t), slots}));
        c->batch_dirty[t] = 0;
    }
    for (int t = 0; t < 2; ++t) {
        HIP_TRY(c, launch_clear(c->stream, ClearJob{c->hop_table[t], slots}));
        c->hop_dirty[t] = 0;
    }
    return HELIOS_OK;
}

// A fresh epoch for the scans of one launch; stale status words of earlier launches read as
// unpublished.  In a recording the batch's base epoch is added on the device.
int next_epoch(helios_ctx* c, uint32_t* out) {
    if (c->recording) {
        c->rec_scans += 1;
        *out = c->rec_scans;
        return HELIOS_OK;
    }
    if (c->epoch >= (1u << 30) - 64) {
        HIP_TRY(c, hipMemsetAsync(c->scan_status, 0, sizeof(unsigned long long) * kScanRows * c->scan_stride, c->stream));
        c->epoch = 0;
    }
    c->epoch += 1;
    *out = c->epoch;
    return HELIOS_OK;
}

// scan state over the status rows from `first_row` on; the two row groups have a ticket counter each
ScanState scan_state(const helios_ctx* c, uint32_t epoch, int first_row) {
    return ScanState{c->scan_status + static_cast<size_t>(first_row) * c->scan_stride,
                     c->scan_ticket + (first_row == kScanRowsHop ? 0 : 16), c->scan_stride, epoch,
                     c->recording ? c->vars : nullptr};
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
// table is cheaper to empty and stays in cache)
uint32_t dedup_slots(const helios_ctx* c, int64_t n_max) {
    const uint32_t want = pow2_at_least(2 * n_max);
    return want < c->table_slots ? want : c->table_slots;
}

unsigned tiles_for(int64_t n_max) {
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    return static_cast<unsigned>(tiles < 1 ? 1 : tiles);
}

// ---- timing of roles
constexpr uint64_t kStampWords = 2ull * kMaxRoleBlocks * 16;     // ticks of all timed roles of one batch (8 MiB)

void reset_stamps(helios_ctx* c) {
    c->n_stamps = 0;
    c->stamp_words = 0;
    c->timed_events = false;
}

// Room in the clock buffer for a role of `workgroups` workgroups, if roles are being timed.
Stamps take_stamps(helios_ctx* c, int kind, int stage, unsigned workgroups) {
    if (c->timing != 1 || !c->clock || c->n_stamps >= kMaxStampRoles || workgroups == 0 || workgroups > kMaxRoleBlocks) return Stamps{nullptr};
    if (c->stamp_words + 2ull * workgroups > kStampWords) return Stamps{nullptr};
    const int q = c->n_stamps++;
    c->stamp_roles[q] = StampRole{kind, stage, workgroups};
    c->stamp_table.offset[q] = c->stamp_words;
    c->stamp_table.workgroups[q] = workgroups;
    Stamps s{reinterpret_cast<unsigned long long*>(c->clock) + c->stamp_words};
    c->stamp_words += 2 * workgroups;
    return s;
}

int publish_stamps(helios_ctx* c) {
    if (c->n_stamps > 0) HIP_TRY(c, launch_clock_publish(c->stream, c->clock, c->stamp_table, c->n_stamps, c->clock_host));
    return HELIOS_OK;
}

// ---- emptiness of the hash tables
// Every table is empty between calls, except the batch tables of the last two batches (kept for
// helios_make_blocks; `batch_dirty` says how much of each may be in use).  A call that failed half way
// leaves its tables marked as in use: the next call empties them first.
int clean_for_call(helios_ctx* c, int batch_table_needed /* -1: none */) {
    for (int t = 0; t < 2; ++t)
        if (c->hop_dirty[t]) {
            HIP_TRY(c, launch_clear(c->stream, ClearJob{c->hop_table[t], c->hop_dirty[t]}));
            c->hop_dirty[t] = 0;
        }
    if (batch_table_needed >= 0 && c->batch_dirty[batch_table_needed]) {
        HIP_TRY(c, launch_clear(c->stream, ClearJob{batch_table(c, batch_table_needed), c->batch_dirty[batch_table_needed]}));
        c->batch_dirty[batch_table_needed] = 0;
    }
    return HELIOS_OK;
}

struct BatchOut {                // the outputs of the whole-path call beyond those of the sampling
    int32_t* unique;
    int64_t unique_cap;
    int32_t* inverse;
    int64_t* n_unique;
    void* out;
    int32_t *miss_pos, *miss_id, *miss_slot;
    int64_t miss_cap;
    helios_gather_stats* stats;
};

int64_t* stage_words(const helios_ctx* c, int stage) { return c->cnt + kCntStage + stage * kStageWords; }

GatherArgs tier_copy_args(helios_ctx* c, int tier, const int64_t* begin, Count end, void* out, Stamps stamps) {
    return GatherArgs{static_cast<const chunk16*>(tier == 0 ? c->hbm_table : c->host_table), c->list_pos[tier], c->list_slot[tier],
                      begin, end, c->row_bytes / 16, static_cast<chunk16*>(out), -1, -1, c->err_now, stamps};
}

// Workgroups of a host-tier copy role over a list of at most n_max rows.  The members of a gang copy at the same
// time: they share what one copy alone would take to fill the link (at least 8 workgroups each).
unsigned link_role_blocks(const helios_ctx* c, int64_t n_max) {
    const int32_t chunks = c->row_bytes / 16;
    unsigned limit = c->host_blocks;
    if (limit == 0 && c->link_share > 1) {
        const unsigned alone = copy_role_blocks(chunks, true, int64_t{1} << 40, 0, 0);
        limit = std::max(8u, (alone + c->link_share - 1) / c->link_share);
    }
    return copy_role_blocks(chunks, true, n_max, limit, 0);
}

// The HBM hits of the context's last finished lookup: the best guess for the next batch's (0 = none yet).  The
// word is written by the lookup's last workgroup and read here without waiting: it only sizes a grid.
int64_t expected_hbm_rows(const helios_ctx* c) {
    const int64_t v = *reinterpret_cast<const volatile int64_t*>(c->learn + 1);
    return v > 0 ? v : 0;
}

// Workgroups of the HBM-tier copy role over a list of at most n_max rows.  Alone, the copy is quickest with one step
// per workgroup (a grid that follows the expected length of the list).  The short lists of a gang's members are copied
// at the same time, and together such grids would be several times what the chip holds at once: each member then
// takes its share, at least 1024 workgroups, and loops (measured with four members of 34 k rows of 512 B: the four
// copies take 31 us with 1024 workgroups each against 41 us with 4.4 k each).  A long list fills the chip by itself
// and keeps its grid.
unsigned hbm_role_blocks(const helios_ctx* c, int64_t n_max) {
    const int32_t chunks = c->row_bytes / 16;
    const unsigned alone = copy_role_blocks(chunks, false, n_max, c->hbm_blocks, expected_hbm_rows(c));
    if (c->hbm_blocks > 0 || c->link_share <= 1 || alone >= 16384) return alone;
    return std::min(alone, std::max(1024u, alone / static_cast<unsigned>(c->link_share)));
}

// The two row copies as kernels of their own over the per-tier lists that a lookup has left behind
// (helios_gather, and the whole-path call with split copies); n_max bounds the lists.
int copy_tiers_split(helios_ctx* c, int64_t n_max, void* out) {
    const bool events = c->timing > 1 && !c->recording;
    if (c->n_hbm > 0 && n_max > 0) {
        const int64_t expected = expected_hbm_rows(c);
        const unsigned nb = copy_role_blocks(c->row_bytes / 16, false, n_max, c->hbm_blocks, expected);
        const GatherArgs a = tier_copy_args(c, 0, nullptr, Count{c->cnt + kCntTier + 0, n_max}, out, take_stamps(c, HELIOS_ROLE_COPY_HBM, 0, nb));
        HIP_TRY(c, launch_gather_rows(c->stream, a, n_max, false, false, c->hbm_blocks, expected, events ? c->t_hbm[0] : nullptr,
                                      events ? c->t_hbm[1] : nullptr, nullptr));
    }
    if (c->n_host > 0 && n_max > 0) {
        const unsigned nb = copy_role_blocks(c->row_bytes / 16, true, n_max, c->host_blocks, 0);
        const GatherArgs a = tier_copy_args(c, 1, nullptr, Count{c->cnt + kCntTier + 1, n_max}, out, take_stamps(c, HELIOS_ROLE_COPY_HOST, 0, nb));
        HIP_TRY(c, launch_gather_rows(c->stream, a, n_max, true, false, c->host_blocks, 0, events ? c->t_host[0] : nullptr,
                                      events ? c->t_host[1] : nullptr, nullptr));
    }
    c->timed_events = events;
    return HELIOS_OK;
}

// The launches of the pipeline go out at once, or, while a gang is being recorded, onto the member's list.
int emit_sample(helios_ctx* c, const SampleJob& j) {
    if (c->defer) {
        PendingStep s{};
        s.kind = kStepSample;
        s.sample = j;
        c->defer->push_back(s);
        return HELIOS_OK;
    }
    HIP_TRY(c, launch_sample(c->stream, &j, 1));
    return HELIOS_OK;
}
int emit_compact(helios_ctx* c, const CompactJob& j) {
    if (c->defer) {
        PendingStep s{};
        s.kind = kStepCompact;
        s.compact = j;
        c->defer->push_back(s);
        return HELIOS_OK;
    }
    HIP_TRY(c, launch_compact(c->stream, &j, 1));
    return HELIOS_OK;
}
int emit_finish(helios_ctx* c, const FinishJob& j) {
    if (c->defer) {
        PendingStep s{};
        s.kind = kStepFinish;
        s.finish = j;
        c->defer->push_back(s);
        return HELIOS_OK;
    }
    HIP_TRY(c, launch_finish(c->stream, &j, 1));
    return HELIOS_OK;
}

// The sampling pipeline, and with `b` the whole path: see pipeline.hip for the launches and their roles.
int run_pipeline(helios_ctx* c, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                 uint64_t rng_seed, const helios_hop_out* hops, int64_t* sizes, const HopPlan& p, const BatchOut* b) {
    const bool rec = c->recording;
    const BatchVars* vars = rec ? c->vars : nullptr;
    const BatchFeed feed = rec ? BatchFeed{c->vars_ring, kVarsRing, c->batches_run, c->vars} : BatchFeed{nullptr, 0, nullptr, nullptr};
    int32_t* err = c->err_now;
    const int32_t chunks = c->row_bytes / 16;
    reset_stamps(c);
    c->blocks_ready = false;

    const int64_t batch_max = p.cat_max > 0 ? p.cat_max : 1;
    const uint32_t which = static_cast<uint32_t>(c->batch_seq % kBatchTables), next = (which + 1) % kBatchTables;
    BatchTables bt{nullptr, 0, nullptr, 0, 0, nullptr, 0};
    uint32_t slots_b = 0;
    if (b) {
        slots_b = dedup_slots(c, batch_max);
        bt = BatchTables{c->batch_tables, c->table_slots, c->batch_iof, static_cast<uint64_t>(c->cap_ids), slots_b, c->batch_slot_of, which};
    }
    uint32_t hop_slots[HELIOS_MAX_HOPS];
    for (int h = 0; h < n_hops; ++h) hop_slots[h] = dedup_slots(c, p.flat_max[h]);
    if (!rec) {
        int rc = clean_for_call(c, b ? static_cast<int>(which) : -1);
        if (rc) return rc;
        // until the call has been enqueued completely, its tables count as in use
        for (int h = 0; h + 1 < n_hops; ++h) c->hop_dirty[h % 2] = std::max(c->hop_dirty[h % 2], hop_slots[h]);
        if (b) c->batch_dirty[which] = slots_b;
    }
    const int64_t u_max = b ? std::min(p.cat_max, b->unique_cap) : 0;
    // What the kernels' own guards rely on (they bound every index by these): a list never outgrows the buffer it
    // is written to, and the scratch holds the longest list.  Cheap enough to check on every call.
    for (int h = 0; h < n_hops; ++h) {
        const bool fits = p.frontier_max[h] <= hops[h].frontier_cap && p.flat_max[h] <= hops[h].flat_cap &&
                          p.flat_max[h] <= c->cap_ids && 2 * p.flat_max[h] <= static_cast<int64_t>(c->table_slots) &&
                          (h == 0 || p.frontier_max[h] <= p.flat_max[h - 1]);
        if (!fits) return fail(c, HELIOS_EINTERNAL, "launch bounds of hop %d do not fit its buffers", h);
    }
    if (p.cat_max > c->cap_ids || 2 * p.cat_max > static_cast<int64_t>(c->table_slots) || (b && u_max > b->unique_cap) ||
        c->scan_stride < static_cast<uint32_t>(p.ids_max / kTileItems + 2))
        return fail(c, HELIOS_EINTERNAL, "launch bounds of the batch do not fit the scratch");

    const bool fold = n_seeds <= kFoldMaxSeeds;
    if (c->defer && (!fold || !b || c->split_copies || c->missq || c->timing > 1))
        return fail(c, HELIOS_EINTERNAL, "this call cannot be part of a gang");       // (refused earlier, with the reason)
    if (!fold) {
        uint32_t epoch;
        int rc = next_epoch(c, &epoch);
        if (rc) return rc;
        HIP_TRY(c, launch_frontier_count(c->stream, c->g, seeds, feed, hops[0].frontier, Count{nullptr, n_seeds}, n_seeds,
                                         fanouts[0], hops[0].indptr, hops[0].flat_cap, c->cnt + kCntFlat + 0, sizes,
                                         scan_state(c, epoch, kScanRowsHop), err));
    }
    Count prev_flat[HELIOS_MAX_HOPS];
    Count nf{nullptr, n_seeds};
    for (int h = 0; h < n_hops; ++h) {
        const bool last = h + 1 == n_hops;
        // ---- sampling pass of hop h; beside it the host-tier copy of the stage that the compaction before it listed
        HopArgs ha{};
        ha.offsets = c->g.offsets;
        ha.indices = c->g.indices;
        ha.n_nodes = c->g.n_nodes;
        ha.fold = h == 0 && fold;
        ha.frontier = ha.fold ? seeds : hops[h].frontier;
        ha.indptr = hops[h].indptr;
        ha.n_frontier = nf;
        ha.fanout = fanouts[h];
        ha.hop = h;
        ha.rng_seed = rng_seed;
        ha.vars = ha.fold ? nullptr : vars;          // the folded hop 0 of a recorded batch reads the ring itself
        ha.flat = hops[h].flat;
        ha.flat_cap = p.flat_max[h];
        ha.clear = h > 0 ? ClearJob{c->hop_table[(h - 1) % 2], hop_slots[h - 1]} : ClearJob{nullptr, 0};
        ha.hop_table = !last ? InsertInto{c->hop_table[h % 2], hop_slots[h], c->hop_slot_of} : InsertInto{nullptr, 0, nullptr};
        ha.batch = bt;
        ha.cat_out = c->cat;
        ha.n_seeds = n_seeds;
        for (int k = 0; k < h; ++k) ha.prev_flat[k] = prev_flat[k];
        ha.err = err;
        if (ha.fold) {
            ha.feed = feed;
            ha.frontier_out = hops[0].frontier;
            ha.indptr_out = hops[0].indptr;
            ha.n_flat_dev = c->cnt + kCntFlat + 0;
            ha.size_out = sizes;
        }
        const unsigned hop_blocks = sample_role_blocks(fanouts[h], p.frontier_max[h]);
        ha.stamps = take_stamps(c, HELIOS_ROLE_SAMPLE, h, hop_blocks);
        GatherArgs link{};
        unsigned link_blocks = 0;
        if (b && h > 0 && !c->split_copies && c->n_host > 0 && u_max > 0) {
            const int stage = h - 1;
            const int64_t stage_max = std::min(u_max, stage == 0 ? n_seeds + p.flat_max[0] : p.flat_max[stage]);
            link_blocks = link_role_blocks(c, stage_max);
            link = tier_copy_args(c, 1, stage > 0 ? stage_words(c, stage - 1) + kStageHostCopy : nullptr,
                                  Count{stage_words(c, stage) + kStageHostCopy, u_max}, b->out,
                                  take_stamps(c, HELIOS_ROLE_COPY_HOST, stage, link_blocks));
        }
        int rs = emit_sample(c, SampleJob{ha, hop_blocks, link, link_blocks});
        if (rs) return rs;
        prev_flat[h] = Count{c->cnt + kCntFlat + h, p.flat_max[h]};

        // ---- compaction: this hop's samples into the next frontier, and stage h of the batch's ID list
        if (last && !b) break;
        uint32_t epoch;
        int rc = next_epoch(c, &epoch);
        if (rc) return rc;
        CompactArgs hopc{}, look{};
        unsigned hopc_blocks = 0, look_blocks = 0;
        if (!last) {
            hopc.ids = hops[h].flat;
            hopc.lens.n_seg = 1;
            hopc.lens.first_here = 0;
            hopc.lens.len[0] = prev_flat[h];
            hopc.n_max = p.flat_max[h];
            hopc.n_total_dev = c->cnt + kCntHopTotal;
            hopc.s = DedupScratch{c->hop_table[h % 2], hop_slots[h], c->hop_slot_of, nullptr};
            hopc.unique = hops[h + 1].frontier;
            hopc.unique_cap = hops[h + 1].frontier_cap;
            hopc.last = true;
            hopc.n_unique_dev = c->cnt + kCntFrontier + h + 1;
            hopc.next = NextHopCount{c->g.offsets, c->g.n_nodes, fanouts[h + 1], hops[h + 1].indptr, hops[h + 1].flat_cap,
                                     c->cnt + kCntFlat + h + 1, sizes ? sizes + 2 * (h + 1) : nullptr};
            hopc.scan = scan_state(c, epoch, kScanRowsHop);
            hopc.err = err;
            hopc_blocks = tiles_for(p.flat_max[h]);
            hopc.stamps = take_stamps(c, HELIOS_ROLE_COMPACT_HOP, h, hopc_blocks);
        }
        if (b) {
            look.ids = c->cat;
            look.lens.n_seg = h + 2;
            look.lens.first_here = h == 0 ? 0 : h + 1;
            look.lens.len[0] = Count{nullptr, n_seeds};
            for (int k = 0; k <= h; ++k) look.lens.len[k + 1] = prev_flat[k];
            look.n_max = h == 0 ? n_seeds + p.flat_max[0] : p.flat_max[h];
            look.n_total_dev = c->cnt + kCntCat;
            look.batch = bt;
            look.vars = vars;
            look.unique = b->unique;
            look.unique_cap = b->unique_cap;
            look.prev = h > 0 ? stage_words(c, h - 1) : nullptr;
            look.mine = stage_words(c, h);
            look.last = last;
            look.n_unique_dev = c->cnt + kCntUnique;
            look.n_unique_out = b->n_unique;
            look.look = LookupOut{c->rank, c->n_hbm, c->n_host,
                                  TierLists{{c->list_pos[0], c->list_pos[1]}, {c->list_slot[0], c->list_slot[1]}, c->cnt + kCntTier},
                                  b->miss_pos, b->miss_id, b->miss_slot, b->miss_cap, reinterpret_cast<int64_t*>(b->stats), c->learn};
            look.batches_run = rec && h == 0 ? c->batches_run : nullptr;
            look.scan = scan_state(c, epoch, kScanRowsLook);
            look.err = err;
            look_blocks = tiles_for(look.n_max);
            look.stamps = take_stamps(c, HELIOS_ROLE_COMPACT_LOOKUP, h, look_blocks);
        }
        rc = emit_compact(c, CompactJob{hopc, hopc_blocks, look, look_blocks});
        if (rc) return rc;
        nf = Count{c->cnt + kCntFrontier + h + 1, !last ? p.frontier_max[h + 1] : 0};
    }
    if (!b) {
        if (!rec) for (int t = 0; t < 2; ++t) c->hop_dirty[t] = 0;         // every hop table was emptied on the way
        return publish_stamps(c);
    }

    // ---- the end of the batch: the rest of the row copies, the inverse map, the next batch's table
    const int64_t standin_rows = c->g.n_nodes - c->n_hbm - c->n_host;
    const int64_t served_max = c->serve_misses && standin_rows > 0 ? std::min(b->miss_cap, u_max) : 0;
    if (c->serve_misses && c->missq) return fail(c, HELIOS_ESTATE, "HELIOS_PARAM_SERVE_MISSES and an attached miss queue exclude each other");
    if (served_max > 0 && !c->standin_table) return fail(c, HELIOS_ESTATE, "no stand-in table was given to helios_cache_build");
    // the batch's own miss list, served from the stand-in; its entries are checked like a caller's (a node whose rank the
    // cache map does not know has slot -1)
    const GatherArgs miss_args{static_cast<const chunk16*>(c->standin_table), b->miss_pos, b->miss_slot, nullptr,
                               Count{c->cnt + kCntTier + 2, served_max}, chunks, static_cast<chunk16*>(b->out), standin_rows,
                               b->unique_cap, err, Stamps{nullptr}};
    if (c->missq) {                 // the misses are on their way while the cached tiers are copied
        const int64_t m_max = std::min(b->miss_cap, u_max);
        int rc = missq_submit_from_batch(c, b->miss_pos, b->miss_slot, Count{c->cnt + kCntTier + 2, m_max}, m_max, b->unique_cap);
        if (rc) return rc;
    }
    const uint32_t clear_slots = rec ? slots_b : c->batch_dirty[next];
    InverseArgs inv{Count{c->cnt + kCntCat, p.cat_max}, DedupScratch{nullptr, 0, nullptr, nullptr}, bt, vars, b->inverse, Stamps{nullptr}};
    if (c->split_copies) {
        int rc = copy_tiers_split(c, u_max, b->out);
        if (rc) return rc;
        if (served_max > 0)
            HIP_TRY(c, launch_gather_rows(c->stream, miss_args, served_max, true, true, c->host_blocks, 0, nullptr, nullptr, nullptr));
        if (b->inverse) HIP_TRY(c, launch_dedup_inverse(c->stream, inv, p.cat_max));
        // (a recording with split copies leaves the emptying of the next table to helios_plan_launch)
        if (!rec && clear_slots) HIP_TRY(c, launch_clear(c->stream, ClearJob{batch_table(c, next), clear_slots}));
    } else {
        const int stage = n_hops - 1;
        GatherArgs hbm{}, link{}, miss{};
        unsigned hbm_blocks = 0, link_blocks = 0, miss_blocks = 0, inv_blocks = 0, clear_blocks = 0;
        if (served_max > 0) {
            miss = miss_args;
            miss_blocks = link_role_blocks(c, served_max);
            miss.stamps = take_stamps(c, HELIOS_ROLE_COPY_STANDIN, stage, miss_blocks);
        }
        if (c->n_hbm > 0 && u_max > 0) {
            hbm_blocks = hbm_role_blocks(c, u_max);
            hbm = tier_copy_args(c, 0, nullptr, Count{c->cnt + kCntTier + 0, u_max}, b->out, take_stamps(c, HELIOS_ROLE_COPY_HBM, stage, hbm_blocks));
        }
        if (c->n_host > 0 && u_max > 0) {
            const int64_t stage_max = std::min(u_max, stage == 0 ? n_seeds + p.flat_max[0] : p.flat_max[stage]);
            link_blocks = link_role_blocks(c, stage_max);
            link = tier_copy_args(c, 1, stage > 0 ? stage_words(c, stage - 1) + kStageHostCopy : nullptr,
                                  Count{c->cnt + kCntTier + 1, u_max}, b->out, take_stamps(c, HELIOS_ROLE_COPY_HOST, stage, link_blocks));
        }
        if (b->inverse) {
            inv_blocks = static_cast<unsigned>(std::min<int64_t>(1024, (p.cat_max + kBlock - 1) / kBlock));
            inv_blocks = inv_blocks < 1 ? 1 : inv_blocks;
            inv.stamps = take_stamps(c, HELIOS_ROLE_INVERSE, stage, inv_blocks);
        }
        ClearJob clear{nullptr, 0};
        if (clear_slots) {
            clear = ClearJob{batch_table(c, next), clear_slots};      // a recording picks the table on the device
            clear_blocks = std::min(256u, (clear_slots + kBlock * 16 - 1) / (kBlock * 16));
        }
        int rf = emit_finish(c, FinishJob{hbm, hbm_blocks, link, link_blocks, miss, miss_blocks, inv, inv_blocks, clear, clear_blocks, bt, vars});
        if (rf) return rf;
    }
    int rc = c->defer ? HELIOS_OK : publish_stamps(c);      // (a gang publishes after its launches have gone out)
    if (rc) return rc;
    if (!rec) {
        for (int t = 0; t < 2; ++t) c->hop_dirty[t] = 0;
        c->batch_dirty[next] = 0;
        c->batch_seq += 1;
        c->blocks_ready = true;
        c->last_table = which;
    }
    c->rec_clear_slots = c->split_copies ? 0 : clear_slots;
    c->last_slots = slots_b;
    c->last_n_seeds = n_seeds;
    c->last_n_hops = n_hops;
    for (int h = 0; h < n_hops; ++h) {
        c->last_frontier_max[h] = p.frontier_max[h];
        c->last_flat_max[h] = p.flat_max[h];
    }
    return HELIOS_OK;
}

int prepare_batch_impl(helios_ctx* c, const int32_t* seeds, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                       uint64_t rng_seed, const helios_hop_out* hops, int64_t* sizes, int32_t* unique,
                       int64_t unique_cap, int32_t* inverse, int64_t* n_unique, void* out, int32_t* miss_pos,
                       int32_t* miss_id, int32_t* miss_slot, int64_t miss_cap, helios_gather_stats* stats) {
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
    const BatchOut b{unique, unique_cap, inverse, n_unique, out, miss_pos, miss_id, miss_slot, miss_cap, stats};
    return run_pipeline(c, seeds, n_seeds, fanouts, n_hops, rng_seed, hops, sizes, p, &b);
}

// a device-side error word: reports and clears what kernels have recorded since the last check
int check_error_word(helios_ctx* c, int32_t* word) {
    const int code = *reinterpret_cast<volatile int32_t*>(word);
    if (code != 0) {
        word[0] = 0;
        return fail(c, code, code == HELIOS_ECAPACITY ? "an output did not fit its capacity"
                             : code == HELIOS_EINTERNAL ? "a workgroup gave up waiting (chained scan, or a miss queue that stopped answering)"
                             : "a node ID outside [0, n_nodes), an order that is not a permutation, or a list entry outside its table");
    }
    return HELIOS_OK;
}

int make_blocks_impl(helios_ctx* c, uint32_t table, uint32_t slots, int64_t n_seeds, int32_t n_hops, const int64_t* frontier_max,
                     const int64_t* flat_max, const int64_t* sizes, const helios_hop_out* hops, const helios_block_out* blocks,
                     int32_t* err) {
    const DedupScratch s{batch_table(c, table), slots, nullptr, batch_iof(c, table)};
    for (int h = 0; h < n_hops; ++h)
        if (!blocks[h].row_local || !blocks[h].col_local) return fail(c, HELIOS_EINVAL, "hop %d: NULL block buffer", h);
    for (int h = 0; h < n_hops; ++h) {
        // the sizes of the batch: the caller's size array if there is one (it belongs to the batch's buffers), else
        // the context's counters, which hold those of the context's last batch
        const Count nf = h == 0 ? Count{nullptr, n_seeds}
                                : Count{sizes ? sizes + 2 * h : c->cnt + kCntFrontier + h, frontier_max[h]};
        const Count nfl{sizes ? sizes + 2 * h + 1 : c->cnt + kCntFlat + h, flat_max[h]};
        HIP_TRY(c, launch_local_ids(c->stream, hops[h].frontier, nf, frontier_max[h], s, blocks[h].row_local, err));
        HIP_TRY(c, launch_local_ids(c->stream, hops[h].flat, nfl, flat_max[h], s, blocks[h].col_local, err));
    }
    return HELIOS_OK;
}

// ---- recorded batches: the parts that a plan of its own and a member of a gang share
helios_plan* new_plan(helios_ctx* c) {
    helios_plan* pl = new helios_plan();
    pl->ctx = c;
    if (hipHostMalloc(reinterpret_cast<void**>(&pl->err), 64, hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess || !pl->err) {
        (void)hipGetLastError();
        delete pl;
        fail(c, HELIOS_EHIP, "no pinned memory for the plan's error word");
        return nullptr;
    }
    pl->err[0] = pl->err[1] = 0;
    return pl;
}

void free_plan(helios_plan* pl) {
    if (pl->exec) (void)hipGraphExecDestroy(pl->exec);
    if (pl->graph) (void)hipGraphDestroy(pl->graph);
    if (pl->done) (void)hipEventDestroy(pl->done);
    if (pl->err) (void)hipHostFree(pl->err);
    delete pl;
}

// what the recording that has just ended left in the context goes into the plan
void fill_plan(helios_plan* pl, helios_ctx* c, const HopPlan& p, int64_t n_seeds, int32_t n_hops, const helios_hop_out* hops,
               int64_t* sizes) {
    pl->n_scans = c->rec_scans;
    pl->scratch_generation = c->scratch_generation;
    pl->cache_generation = c->cache_generation;
    pl->graph_generation = c->graph_generation;
    pl->n_seeds = n_seeds;
    pl->n_hops = n_hops;
    for (int h = 0; h < n_hops; ++h) {
        pl->frontier_max[h] = p.frontier_max[h];
        pl->flat_max[h] = p.flat_max[h];
        pl->hops[h] = hops[h];
    }
    pl->sizes = sizes;
    pl->slots = c->last_slots;
    pl->clear_slots = c->rec_clear_slots;
    pl->missq = c->missq;
    pl->n_stamps = c->n_stamps;
    pl->stamp_table = c->stamp_table;
    for (int q = 0; q < c->n_stamps; ++q) pl->stamp_roles[q] = c->stamp_roles[q];
    reset_stamps(c);
}

// Everything of a launch up to the launch itself: the checks, the tables that the recording expects to be empty,
// the batch's variables in the next ring slot.  Nothing is committed: if the launch does not happen, nothing has.
int plan_prelaunch(helios_plan* pl, const int32_t* seeds, uint64_t rng_seed, uint32_t* io_round_out) {
    helios_ctx* c = pl->ctx;
    if (pl->n_seeds > 0 && !seeds) return fail(c, HELIOS_EINVAL, "seeds is NULL");
    if (pl->scratch_generation != c->scratch_generation)
        return fail(c, HELIOS_ESTATE, "the context's scratch was regrown after the batch was recorded; record it again");
    if (pl->graph_generation != c->graph_generation || pl->cache_generation != c->cache_generation || !c->has_cache)
        return fail(c, HELIOS_ESTATE, "helios_csr_load / helios_cache_build was called after the batch was recorded; record it again");
    if (pl->missq != c->missq)
        return fail(c, HELIOS_ESTATE, "the miss queue attached to the context is not the one the batch was recorded with");
    uint32_t io_round = 0;
    if (pl->missq) {
        int rc = missq_next_round(c, pl->missq, &io_round);      // opened once the launch has succeeded
        if (rc) return rc;
    }
    if (c->epoch + pl->n_scans >= (1u << 30) - 64) {
        HIP_TRY(c, hipMemsetAsync(c->scan_status, 0, sizeof(unsigned long long) * kScanRows * c->scan_stride, c->stream));
        c->epoch = 0;
    }
    if (c->vars_unsynced + 1 >= kVarsRing) {     // the ring slot about to be reused may still be in flight
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        c->vars_unsynced = 0;
    }
    // The recording assumes that its own batch table and both hop tables are empty, and it empties clear_slots slots
    // of the next batch's table.  What that leaves out is emptied here, by launches of their own (rare: only when
    // batches of different sizes, or direct and recorded calls, alternate on a context).
    const uint32_t which = static_cast<uint32_t>(c->batch_seq % kBatchTables), next = (which + 1) % kBatchTables;
    int rc = clean_for_call(c, static_cast<int>(which));
    if (rc) return rc;
    if (c->batch_dirty[next] > pl->clear_slots) {
        HIP_TRY(c, launch_clear(c->stream, ClearJob{batch_table(c, next), c->batch_dirty[next]}));
        c->batch_dirty[next] = 0;
    }
    BatchVars* slot = c->vars_ring + (c->vars_next % kVarsRing);
    slot->rng_seed = rng_seed;
    slot->seeds = seeds;
    slot->epoch_base = c->epoch;
    slot->io_round = io_round;
    slot->table = which;
    slot->reserved = 0;
    __atomic_thread_fence(__ATOMIC_RELEASE);     // the slot is written before the launch is rung in
    *io_round_out = io_round;
    return HELIOS_OK;
}

// The launch has happened: only a batch that was launched takes its ring slot (the device counts the batches it
// runs, and the two counts select the slot), its tables, its miss-queue round.
void plan_postlaunch(helios_plan* pl, uint32_t io_round) {
    helios_ctx* c = pl->ctx;
    const uint32_t which = static_cast<uint32_t>(c->batch_seq % kBatchTables), next = (which + 1) % kBatchTables;
    c->vars_next += 1;
    c->vars_unsynced += 1;
    c->epoch += pl->n_scans;
    if (pl->missq) missq_commit_round(pl->missq, io_round);
    c->batch_dirty[which] = pl->slots;
    c->batch_dirty[next] = 0;
    c->batch_seq += 1;
    pl->batch_seq = c->batch_seq;
    c->launch_seq += 1;
    pl->launch_seq = c->launch_seq;
    c->blocks_ready = true;
    c->last_table = which;
    c->last_slots = pl->slots;
    c->last_n_seeds = pl->n_seeds;
    c->last_n_hops = pl->n_hops;
    for (int h = 0; h < pl->n_hops; ++h) {
        c->last_frontier_max[h] = pl->frontier_max[h];
        c->last_flat_max[h] = pl->flat_max[h];
    }
    c->n_stamps = pl->n_stamps;
    c->stamp_table = pl->stamp_table;
    for (int q = 0; q < pl->n_stamps; ++q) c->stamp_roles[q] = pl->stamp_roles[q];
    c->timed_events = false;
}

// after the event behind the plan's last launch has been waited for
int plan_retire(helios_plan* pl) {
    helios_ctx* c = pl->ctx;
    // everything launched on the context up to this plan's launch has finished
    const uint64_t later = c->launch_seq - pl->launch_seq;
    if (later < c->vars_unsynced) c->vars_unsynced = static_cast<uint32_t>(later);
    return check_error_word(c, pl->err);                 // the errors of this plan's batches, not of others queued behind them
}

int plan_make_blocks(helios_plan* pl, const helios_block_out* blocks) {
    helios_ctx* c = pl->ctx;
    if (!blocks) return fail(c, HELIOS_EINVAL, "blocks is NULL");
    if (pl->launch_seq == 0) return fail(c, HELIOS_ESTATE, "the plan has not been launched");
    if (pl->scratch_generation != c->scratch_generation) return fail(c, HELIOS_ESTATE, "the context's scratch was regrown since");
    // the plan's batch was number batch_seq - 1 of the context; its table is kept until the second batch after it
    // is launched (that one empties it for the third)
    const uint32_t table = static_cast<uint32_t>((pl->batch_seq - 1) % kBatchTables);
    if (c->batch_seq - pl->batch_seq > 1 || c->batch_dirty[table] < pl->slots)
        return fail(c, HELIOS_ESTATE, "two or more batches were launched on the context since this plan's: its table is gone");
    if (!pl->sizes && c->batch_seq != pl->batch_seq)
        return fail(c, HELIOS_ESTATE, "a plan recorded without a size array can only make blocks right after its launch");
    DeviceGuard guard(c->device);
    return make_blocks_impl(c, table, pl->slots, pl->n_seeds, pl->n_hops, pl->frontier_max, pl->flat_max, pl->sizes, pl->hops,
                            blocks, pl->err);
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
    bool ok = hipEventCreate(&c->t_hbm[0]) == hipSuccess && hipEventCreate(&c->t_hbm[1]) == hipSuccess &&
              hipEventCreate(&c->t_host[0]) == hipSuccess && hipEventCreate(&c->t_host[1]) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->err), 64, hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess &&
              hipMalloc(&c->cnt, sizeof(int64_t) * kNumCounters) == hipSuccess &&
              hipMalloc(&c->vars, sizeof(BatchVars)) == hipSuccess &&
              hipMalloc(&c->scan_ticket, 128) == hipSuccess &&
              hipMalloc(&c->batches_run, 64) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->vars_ring), sizeof(BatchVars) * kVarsRing,
                            hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->learn), 64, hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&c->clock_host), sizeof(uint64_t) * 2 * kMaxStampRoles,
                            hipHostMallocMapped | hipHostMallocCoherent) == hipSuccess;
    ok = ok && c->err && c->cnt && c->vars && c->scan_ticket && c->batches_run && c->vars_ring && c->learn && c->clock_host;
    ok = ok && noalloc_init(device) == HELIOS_OK;      // address of this device's static scratch (helios_dedup_noalloc)
    if (ok) {
        int khz = 0;
        if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, device) == hipSuccess && khz > 0) c->clock_khz = khz;
        c->err[0] = c->err[1] = 0;
        c->err_now = c->err;
        for (int k = 0; k < 4; ++k) c->learn[k] = 0;
        ok = hipMemsetAsync(c->cnt, 0, sizeof(int64_t) * kNumCounters, c->stream) == hipSuccess &&
             hipMemsetAsync(c->scan_ticket, 0, 128, c->stream) == hipSuccess &&
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
    free_scratch(c);
    (void)hipFree(c->rank);
    (void)hipFree(c->cnt);
    (void)hipFree(c->vars);
    (void)hipFree(c->scan_ticket);
    (void)hipFree(c->batches_run);
    (void)hipFree(c->hot_temp);
    if (c->vars_ring) (void)hipHostFree(c->vars_ring);
    (void)hipFree(c->clock);
    if (c->clock_host) (void)hipHostFree(c->clock_host);
    if (c->err) (void)hipHostFree(c->err);
    if (c->learn) (void)hipHostFree(c->learn);
    for (hipEvent_t e : {c->t_hbm[0], c->t_hbm[1], c->t_host[0], c->t_host[1]})
        if (e) (void)hipEventDestroy(e);
    delete c;
    return HELIOS_OK;
}

const char* helios_last_error(const helios_ctx* c) { return c ? c->errmsg : "no context"; }

int helios_reserve(helios_ctx* c, int64_t max_ids) {
    if (!c || max_ids < 0) return fail(c, HELIOS_EINVAL, "helios_reserve: bad argument");
    DeviceGuard guard(c->device);
    return ensure_capacity(c, max_ids);
}

int helios_sync(helios_ctx* c) {
    if (!c) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->vars_unsynced = 0;
    int rc = check_error_word(c, c->err);
    for (helios_plan* pl : c->plans) {           // every batch launched on the context has finished: its errors count
        const int rp = check_error_word(c, pl->err);
        if (rc == HELIOS_OK) rc = rp;
    }
    return rc;
}

int helios_csr_load(helios_ctx* c, int64_t n_nodes, int64_t n_edges, const int64_t* offsets, const int32_t* indices) {
    if (!c) return HELIOS_EINVAL;
    if (n_nodes < 0 || n_edges < 0 || n_nodes > 0x7fffffffLL) return fail(c, HELIOS_EINVAL, "bad graph size");
    if (!offsets || (n_edges > 0 && !indices)) return fail(c, HELIOS_EINVAL, "offsets / indices is NULL");
    c->g = CsrView{offsets, indices, n_nodes};
    c->n_edges = n_edges;
    c->has_graph = true;
    c->graph_generation += 1;
    c->has_cache = false;              // the cache map belongs to the graph it was built for
    c->blocks_ready = false;
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
    const GatherArgs a{static_cast<const chunk16*>(src_table), nullptr, order + first_rank, nullptr, Count{nullptr, n_rows},
                       row_bytes / 16, static_cast<chunk16*>(dst), -1, -1, c->err, Stamps{nullptr}};
    HIP_TRY(c, launch_gather_rows(c->stream, a, n_rows, false, false, 0, n_rows, nullptr, nullptr, nullptr));
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
    return run_pipeline(c, seeds, n_seeds, fanouts, n_hops, rng_seed, hops, sizes, p, nullptr);
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
    // the table that the context's next batch would use: not one that helios_make_blocks may still need
    const uint32_t which = static_cast<uint32_t>(c->batch_seq % kBatchTables);
    rc = clean_for_call(c, static_cast<int>(which));
    if (rc) return rc;
    uint32_t epoch;
    rc = next_epoch(c, &epoch);
    if (rc) return rc;
    const DedupScratch s{batch_table(c, which), dedup_slots(c, n_ids), c->batch_slot_of, batch_iof(c, which)};
    c->batch_dirty[which] = s.n_slots;
    const Count n{nullptr, n_ids};
    HIP_TRY(c, launch_dedup_insert(c->stream, ids, n, n_ids, c->g.n_nodes, s, c->err));
    CompactArgs a{};
    a.ids = ids;
    a.lens.n_seg = 1;
    a.lens.first_here = 0;
    a.lens.len[0] = n;
    a.n_max = n_ids;
    a.n_total_dev = c->cnt + kCntCat;
    a.s = s;
    a.unique = unique;
    a.unique_cap = unique_cap;
    a.last = true;
    a.n_unique_dev = c->cnt + kCntUnique;
    a.n_unique_out = n_unique;
    a.scan = scan_state(c, epoch, kScanRowsLook);
    a.err = c->err;
    HIP_TRY(c, launch_dedup_compact_plain(c->stream, a, n_ids));
    if (inverse) {
        const InverseArgs inv{Count{c->cnt + kCntCat, n_ids}, s, BatchTables{nullptr, 0, nullptr, 0, 0, nullptr, 0}, nullptr, inverse,
                              Stamps{nullptr}};
        HIP_TRY(c, launch_dedup_inverse(c->stream, inv, n_ids));
    }
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
    reset_stamps(c);
    uint32_t epoch;
    rc = next_epoch(c, &epoch);
    if (rc) return rc;
    const TierLists lists{{c->list_pos[0], c->list_pos[1]}, {c->list_slot[0], c->list_slot[1]}, c->cnt + kCntTier};
    HIP_TRY(c, launch_lookup_partition(c->stream, ids, Count{nullptr, n_ids}, n_ids, c->rank, c->g.n_nodes, c->n_hbm, c->n_host,
                                       lists, miss_pos, miss_id, miss_slot, miss_cap, reinterpret_cast<int64_t*>(stats), c->learn,
                                       scan_state(c, epoch, kScanRowsLook), c->err));
    rc = copy_tiers_split(c, n_ids, out);
    if (rc) return rc;
    return publish_stamps(c);
}

int helios_gather_miss(helios_ctx* c, const int32_t* miss_pos, const int32_t* miss_slot, int64_t n_miss_max,
                       const int64_t* n_miss_dev, void* out, int64_t out_rows) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_cache) return fail(c, HELIOS_ESTATE, "helios_gather_miss before helios_cache_build");
    if (n_miss_max < 0 || out_rows < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (n_miss_max == 0) return HELIOS_OK;
    if (!miss_pos || !miss_slot || !out) return fail(c, HELIOS_EINVAL, "NULL pointer");
    const int64_t standin_rows = c->g.n_nodes - c->n_hbm - c->n_host;
    if (standin_rows > 0 && !c->standin_table) return fail(c, HELIOS_ESTATE, "no stand-in table was given to helios_cache_build");
    DeviceGuard guard(c->device);
    // (with every node cached nothing can miss: any entry is then reported by the kernel as outside its table)
    const GatherArgs a{static_cast<const chunk16*>(c->standin_table), miss_pos, miss_slot, nullptr, Count{n_miss_dev, n_miss_max},
                       c->row_bytes / 16, static_cast<chunk16*>(out), standin_rows, out_rows, c->err, Stamps{nullptr}};
    HIP_TRY(c, launch_gather_rows(c->stream, a, n_miss_max, true, true, c->host_blocks, 0, nullptr, nullptr, nullptr));
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
    helios_plan* pl = new_plan(c);
    if (!pl) return HELIOS_EHIP;
    c->recording = true;
    c->rec_scans = 0;
    c->err_now = pl->err;
    const bool was_ready = c->blocks_ready;
    hipError_t e = hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal);
    if (e == hipSuccess) {
        // the seeds pointer and rng_seed passed here are placeholders: recorded kernels read both from the batch's variables
        rc = prepare_batch_impl(c, reinterpret_cast<const int32_t*>(c->vars), n_seeds, fanouts, n_hops, 0, hops, sizes,
                                unique, unique_cap, inverse, n_unique, out, miss_pos, miss_id, miss_slot, miss_cap, stats);
        hipError_t e2 = hipStreamEndCapture(c->stream, &pl->graph);
        if (rc == HELIOS_OK && e2 != hipSuccess) e = e2;
    }
    c->recording = false;
    c->err_now = c->err;
    c->blocks_ready = was_ready;                 // nothing has run
    if (e == hipSuccess && rc == HELIOS_OK) e = hipGraphInstantiate(&pl->exec, pl->graph, nullptr, nullptr, 0);
    if (e == hipSuccess && rc == HELIOS_OK) e = hipEventCreateWithFlags(&pl->done, hipEventDisableTiming);
    if (e != hipSuccess || rc != HELIOS_OK) {
        reset_stamps(c);                             // whatever the failed recording took
        free_plan(pl);
        if (rc != HELIOS_OK) return rc;
        return fail(c, HELIOS_EHIP, "recording the batch failed: %s", hipGetErrorString(e));
    }
    fill_plan(pl, c, p, n_seeds, n_hops, hops, sizes);
    c->n_children += 1;
    c->plans.push_back(pl);
    *plan_out = pl;
    return HELIOS_OK;
}

int helios_plan_launch(helios_plan* pl, const int32_t* seeds, uint64_t rng_seed) {
    if (!pl || !pl->ctx || pl->gang) return HELIOS_EINVAL;
    helios_ctx* c = pl->ctx;
    DeviceGuard guard(c->device);
    uint32_t io_round = 0;
    int rc = plan_prelaunch(pl, seeds, rng_seed, &io_round);
    if (rc) return rc;
    HIP_TRY(c, hipGraphLaunch(pl->exec, c->stream));
    plan_postlaunch(pl, io_round);
    HIP_TRY(c, hipEventRecord(pl->done, c->stream));
    return HELIOS_OK;
}

int helios_plan_wait(helios_plan* pl) {
    if (!pl || !pl->ctx || pl->gang) return HELIOS_EINVAL;
    helios_ctx* c = pl->ctx;
    if (pl->launch_seq == 0) return HELIOS_OK;           // never launched
    DeviceGuard guard(c->device);
    HIP_TRY(c, hipEventSynchronize(pl->done));
    return plan_retire(pl);
}

int helios_plan_destroy(helios_plan* pl) {
    if (!pl) return HELIOS_EINVAL;
    if (pl->gang) return HELIOS_EINVAL;                  // a gang's members go with the gang
    if (pl->ctx) {
        helios_ctx* c = pl->ctx;
        DeviceGuard guard(c->device);
        (void)hipStreamSynchronize(c->stream);
        c->n_children -= 1;
        c->plans.erase(std::remove(c->plans.begin(), c->plans.end(), pl), c->plans.end());
    }
    free_plan(pl);
    return HELIOS_OK;
}

int helios_gang_create(helios_ctx* const* ctxs, int32_t n_members, int64_t n_seeds, const int32_t* fanouts, int32_t n_hops,
                       const helios_batch_buffers* buffers, helios_gang** gang_out) {
    if (!ctxs || !gang_out || n_members < 1 || !ctxs[0]) return HELIOS_EINVAL;
    *gang_out = nullptr;
    helios_ctx* c0 = ctxs[0];
    if (n_members > kMaxGang) return fail(c0, HELIOS_EINVAL, "a gang has at most %d members", kMaxGang);
    if (!buffers) return fail(c0, HELIOS_EINVAL, "buffers is NULL");
    if (!c0->stream) return fail(c0, HELIOS_EINVAL, "a gang cannot be recorded on the default (NULL) stream");
    if (n_seeds > kFoldMaxSeeds) return fail(c0, HELIOS_EINVAL, "a batch of a gang has at most %d seeds", kFoldMaxSeeds);
    for (int m = 0; m < n_members; ++m) {
        helios_ctx* c = ctxs[m];
        if (!c) return fail(c0, HELIOS_EINVAL, "member %d is NULL", m);
        for (int k = 0; k < m; ++k)
            if (ctxs[k] == c) return fail(c0, HELIOS_EINVAL, "members %d and %d are the same context", k, m);
        if (c->stream != c0->stream || c->device != c0->device)
            return fail(c0, HELIOS_EINVAL, "member %d is not on the stream of member 0: a gang's contexts share one stream", m);
        if (!c->has_graph || !c->has_cache) return fail(c0, HELIOS_ESTATE, "member %d has no graph or no cache", m);
        if (c->row_bytes != c0->row_bytes) return fail(c0, HELIOS_EINVAL, "member %d has rows of another size", m);
        if (c->timing > 1 || c->split_copies || c->missq)
            return fail(c0, HELIOS_ESTATE, "member %d: event timing, split copies and an attached miss queue do not go with a gang", m);
        if (c->recording) return fail(c0, HELIOS_ESTATE, "member %d is being recorded", m);
    }
    DeviceGuard guard(c0->device);
    HopPlan p[kMaxGang];
    for (int m = 0; m < n_members; ++m) {
        helios_ctx* c = ctxs[m];
        int rc = plan_hops(c, n_seeds, fanouts, n_hops, buffers[m].hops, &p[m]);
        if (rc == HELIOS_OK) rc = ensure_capacity(c, p[m].ids_max);          // allocate before recording starts
        if (rc) return c == c0 ? rc : fail(c0, rc, "member %d: %s", m, c->errmsg);
    }
    HIP_TRY(c0, hipStreamSynchronize(c0->stream));
    helios_gang* g = new helios_gang();
    g->n = n_members;
    g->device = c0->device;
    g->stream = c0->stream;
    int rc = HELIOS_OK;
    for (int m = 0; m < n_members && rc == HELIOS_OK; ++m) {
        g->member[m] = new_plan(ctxs[m]);
        if (!g->member[m]) rc = fail(c0, HELIOS_EHIP, "no pinned memory for a member's error word");
    }
    std::vector<PendingStep> steps[kMaxGang];
    bool was_ready[kMaxGang] = {false, false, false, false};
    hipError_t e = hipSuccess;
    if (rc == HELIOS_OK) {
        for (int m = 0; m < n_members; ++m) {
            helios_ctx* c = ctxs[m];
            c->recording = true;
            c->rec_scans = 0;
            c->err_now = g->member[m]->err;
            c->defer = &steps[m];
            c->link_share = n_members;
            was_ready[m] = c->blocks_ready;
        }
        e = hipStreamBeginCapture(c0->stream, hipStreamCaptureModeThreadLocal);
        if (e == hipSuccess) {
            // every member prepares its launches (the seeds pointer and rng_seed are placeholders: recorded kernels
            // read both from the batch's variables) ...
            for (int m = 0; m < n_members && rc == HELIOS_OK; ++m) {
                helios_ctx* c = ctxs[m];
                const helios_batch_buffers& bb = buffers[m];
                rc = prepare_batch_impl(c, reinterpret_cast<const int32_t*>(c->vars), n_seeds, fanouts, n_hops, 0, bb.hops, bb.sizes,
                                        bb.unique, bb.unique_cap, bb.inverse, bb.n_unique, bb.out, bb.miss_pos, bb.miss_id,
                                        bb.miss_slot, bb.miss_cap, bb.stats);
                if (rc && c != c0) rc = fail(c0, rc, "member %d: %s", m, c->errmsg);
            }
            // ... and step by step the launches of all members go out as one
            for (int m = 1; m < n_members && rc == HELIOS_OK; ++m) {
                bool same = steps[m].size() == steps[0].size();
                for (size_t k = 0; same && k < steps[0].size(); ++k) same = steps[m][k].kind == steps[0][k].kind;
                if (!same) rc = fail(c0, HELIOS_EINTERNAL, "the members of a gang do not take the same steps");
            }
            for (size_t k = 0; k < steps[0].size() && rc == HELIOS_OK && e == hipSuccess; ++k) {
                if (steps[0][k].kind == kStepSample) {
                    SampleJob jobs[kMaxGang];
                    for (int m = 0; m < n_members; ++m) jobs[m] = steps[m][k].sample;
                    e = launch_sample(c0->stream, jobs, n_members);
                } else if (steps[0][k].kind == kStepCompact) {
                    CompactJob jobs[kMaxGang];
                    for (int m = 0; m < n_members; ++m) jobs[m] = steps[m][k].compact;
                    e = launch_compact(c0->stream, jobs, n_members);
                } else {
                    FinishJob jobs[kMaxGang];
                    for (int m = 0; m < n_members; ++m) jobs[m] = steps[m][k].finish;
                    e = launch_finish(c0->stream, jobs, n_members);
                }
            }
            // members whose roles are timed (timing level 1 at creation) publish their ticks behind the last launch
            for (int m = 0; m < n_members && rc == HELIOS_OK && e == hipSuccess; ++m) rc = publish_stamps(ctxs[m]);
            hipError_t e2 = hipStreamEndCapture(c0->stream, &g->graph);
            if (rc == HELIOS_OK && e == hipSuccess && e2 != hipSuccess) e = e2;
        }
        for (int m = 0; m < n_members; ++m) {
            helios_ctx* c = ctxs[m];
            c->recording = false;
            c->err_now = c->err;
            c->defer = nullptr;
            c->link_share = 1;
            c->blocks_ready = was_ready[m];          // nothing has run
        }
    }
    if (e == hipSuccess && rc == HELIOS_OK) e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
    if (e == hipSuccess && rc == HELIOS_OK) e = hipEventCreateWithFlags(&g->done, hipEventDisableTiming);
    if (e != hipSuccess || rc != HELIOS_OK) {
        for (int m = 0; m < n_members; ++m) {
            reset_stamps(ctxs[m]);                   // whatever the failed recording took
            if (g->member[m]) free_plan(g->member[m]);
        }
        if (g->exec) (void)hipGraphExecDestroy(g->exec);
        if (g->graph) (void)hipGraphDestroy(g->graph);
        if (g->done) (void)hipEventDestroy(g->done);
        delete g;
        (void)hipGetLastError();
        if (rc != HELIOS_OK) return rc;
        return fail(c0, HELIOS_EHIP, "recording the gang failed: %s", hipGetErrorString(e));
    }
    for (int m = 0; m < n_members; ++m) {
        helios_ctx* c = ctxs[m];
        helios_plan* pl = g->member[m];
        fill_plan(pl, c, p[m], n_seeds, n_hops, buffers[m].hops, buffers[m].sizes);
        pl->gang = g;
        c->n_children += 1;
        c->plans.push_back(pl);
    }
    *gang_out = g;
    return HELIOS_OK;
}

int helios_gang_launch(helios_gang* g, const int32_t* const* seeds, const uint64_t* rng_seeds) {
    if (!g || g->n < 1) return HELIOS_EINVAL;
    helios_ctx* c0 = g->member[0]->ctx;
    if (!seeds || !rng_seeds) return fail(c0, HELIOS_EINVAL, "seeds / rng_seeds is NULL");
    DeviceGuard guard(g->device);
    uint32_t io_round[kMaxGang] = {0, 0, 0, 0};
    for (int m = 0; m < g->n; ++m) {
        helios_plan* pl = g->member[m];
        int rc = plan_prelaunch(pl, seeds[m], rng_seeds[m], &io_round[m]);
        if (rc) return pl->ctx == c0 ? rc : fail(c0, rc, "member %d: %s", m, pl->ctx->errmsg);
    }
    HIP_TRY(c0, hipGraphLaunch(g->exec, g->stream));
    for (int m = 0; m < g->n; ++m) plan_postlaunch(g->member[m], io_round[m]);
    g->launched = true;
    HIP_TRY(c0, hipEventRecord(g->done, g->stream));
    return HELIOS_OK;
}

int helios_gang_wait(helios_gang* g, int32_t* member_status) {
    if (!g || g->n < 1) return HELIOS_EINVAL;
    helios_ctx* c0 = g->member[0]->ctx;
    for (int m = 0; member_status && m < g->n; ++m) member_status[m] = HELIOS_OK;
    if (!g->launched) return HELIOS_OK;
    DeviceGuard guard(g->device);
    HIP_TRY(c0, hipEventSynchronize(g->done));
    int first = HELIOS_OK;
    for (int m = 0; m < g->n; ++m) {
        const int rc = plan_retire(g->member[m]);
        if (member_status) member_status[m] = rc;
        if (rc != HELIOS_OK && first == HELIOS_OK) first = g->member[m]->ctx == c0 ? rc : fail(c0, rc, "member %d: %s", m, g->member[m]->ctx->errmsg);
    }
    return first;
}

int helios_gang_make_blocks(helios_gang* g, int32_t member, const helios_block_out* blocks) {
    if (!g || member < 0 || member >= g->n) return HELIOS_EINVAL;
    return plan_make_blocks(g->member[member], blocks);
}

int helios_gang_destroy(helios_gang* g) {
    if (!g) return HELIOS_EINVAL;
    {
        DeviceGuard guard(g->device);
        (void)hipStreamSynchronize(g->stream);
    }
    for (int m = 0; m < g->n; ++m) {
        helios_plan* pl = g->member[m];
        helios_ctx* c = pl->ctx;
        c->n_children -= 1;
        c->plans.erase(std::remove(c->plans.begin(), c->plans.end(), pl), c->plans.end());
        free_plan(pl);
    }
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    if (g->done) (void)hipEventDestroy(g->done);
    delete g;
    return HELIOS_OK;
}

int helios_make_blocks(helios_ctx* c, const helios_hop_out* hops, int32_t n_hops, const helios_block_out* blocks) {
    if (!c) return HELIOS_EINVAL;
    if (!c->blocks_ready) return fail(c, HELIOS_ESTATE, "helios_make_blocks must follow helios_prepare_batch on this context");
    if (!hops || !blocks || n_hops != c->last_n_hops) return fail(c, HELIOS_EINVAL, "hops / blocks do not match the last batch");
    DeviceGuard guard(c->device);
    return make_blocks_impl(c, c->last_table, c->last_slots, c->last_n_seeds, n_hops, c->last_frontier_max, c->last_flat_max,
                            nullptr, hops, blocks, c->err);
}

int helios_plan_make_blocks(helios_plan* pl, const helios_block_out* blocks) {
    if (!pl || !pl->ctx) return HELIOS_EINVAL;
    return plan_make_blocks(pl, blocks);
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
    // scratch of the sort: allocated on the first call for a graph of this size, kept until the context is destroyed
    const size_t bytes = hotness_order_scratch_bytes(n);
    if (bytes > c->hot_temp_bytes) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        (void)hipFree(c->hot_temp);
        c->hot_temp = nullptr;
        c->hot_temp_bytes = 0;
        HIP_TRY(c, hipMalloc(&c->hot_temp, bytes));
        c->hot_temp_bytes = bytes;
    }
    HIP_TRY(c, launch_hotness_order(c->stream, counts, n, order, c->hot_temp, c->err));
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
            c->hbm_blocks = static_cast<unsigned>(value > kMaxRoleBlocks ? kMaxRoleBlocks : value);
            return HELIOS_OK;
        case HELIOS_PARAM_HOST_GATHER_BLOCKS:
            c->host_blocks = static_cast<unsigned>(value > kMaxRoleBlocks ? kMaxRoleBlocks : value);
            return HELIOS_OK;
        case HELIOS_PARAM_SPLIT_COPIES:
            c->split_copies = value != 0;
            return HELIOS_OK;
        case HELIOS_PARAM_SERVE_MISSES:
            c->serve_misses = value != 0;
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

int helios_set_timing(helios_ctx* c, int level) {
    if (!c) return HELIOS_EINVAL;
    if (level == 1 && !c->clock) {              // room for the ticks of every workgroup of every timed role of a batch
        DeviceGuard guard(c->device);
        HIP_TRY(c, hipMalloc(&c->clock, sizeof(uint64_t) * kStampWords));
    }
    c->timing = level < 0 ? 0 : level > 2 ? 2 : level;
    reset_stamps(c);
    return HELIOS_OK;
}

int helios_batch_ticks(helios_ctx* c, helios_role_ticks* out, int32_t cap, int32_t* n_out, double* ticks_per_us) {
    if (!c || !n_out || cap < 0 || (cap > 0 && !out)) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    *n_out = 0;
    if (ticks_per_us) *ticks_per_us = c->clock_khz / 1000.0;
    if (c->n_stamps == 0) return HELIOS_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));          // the publish kernel has written the pinned words
    for (int q = 0; q < c->n_stamps && *n_out < cap; ++q) {
        const volatile uint64_t* k = c->clock_host + 2 * q;
        helios_role_ticks& r = out[(*n_out)++];
        const bool ok = k[0] != ~0ull && k[1] >= k[0];
        r.kind = c->stamp_roles[q].kind;
        r.stage = c->stamp_roles[q].stage;
        r.workgroups = c->stamp_roles[q].workgroups;
        r.start = ok ? k[0] : 0;
        r.end = ok ? k[1] : 0;
    }
    return HELIOS_OK;
}

int helios_gather_times(helios_ctx* c, float* hbm_ms, float* host_ms, float* hbm_event_ms, float* host_event_ms) {
    if (!c || !hbm_ms || !host_ms) return HELIOS_EINVAL;
    DeviceGuard guard(c->device);
    *hbm_ms = *host_ms = 0.f;
    if (hbm_event_ms) *hbm_event_ms = 0.f;
    if (host_event_ms) *host_event_ms = 0.f;
    if (c->n_stamps == 0 && !c->timed_events) return HELIOS_OK;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int q = 0; q < c->n_stamps; ++q) {
        const volatile uint64_t* k = c->clock_host + 2 * q;
        if (k[0] == ~0ull || k[1] < k[0]) continue;
        const float ms = static_cast<float>(static_cast<double>(k[1] - k[0]) / c->clock_khz);
        if (c->stamp_roles[q].kind == HELIOS_ROLE_COPY_HBM) *hbm_ms += ms;
        if (c->stamp_roles[q].kind == HELIOS_ROLE_COPY_HOST) *host_ms += ms;
    }
    if (c->timed_events) {
        float ev = 0.f;
        if (c->n_hbm > 0 && hbm_event_ms && hipEventElapsedTime(&ev, c->t_hbm[0], c->t_hbm[1]) == hipSuccess) *hbm_event_ms = ev;
        if (c->n_host > 0 && host_event_ms && hipEventElapsedTime(&ev, c->t_host[0], c->t_host[1]) == hipSuccess) *host_event_ms = ev;
        (void)hipGetLastError();
    }
    return HELIOS_OK;
}

}  // extern "C"
