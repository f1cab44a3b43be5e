// Device code of the second pass of the order-preserving de-duplication (see dedup.hip for the
// whole scheme): the inputs have been inserted into a hash table that keeps, per distinct ID, the
// smallest input position holding it, and the slot of every input is remembered.  Input j is a
// first occurrence iff its slot's position is j.  A thread takes four consecutive inputs; the flags
// are scanned in the workgroup and chained across workgroups (scan.hpp), so `unique` comes out in
// input order.  The pass has the new unique IDs in registers, so two things that need them ride on
// it instead of being kernels of their own:
//   kCompactNextHop  the unique list is the frontier of the next hop: read every new frontier node's
//                    row bounds and scan the sample counts min(deg, fanout) as a second counter,
//                    which gives that hop its indptr;
//   kCompactLookup   the unique list is (a stage of) the batch's ID list: read rank[id], classify into
//                    HBM tier, host tier or miss, and scan the two hit classes as further counters
//                    (the miss rank is what is left), which gives the stable per-tier lists and the
//                    miss list that cache.hip's stand-alone lookup kernel would produce from `unique`.
//
// Stages.  The list may be compacted piece by piece: a stage handles the inputs [begin, begin + n)
// and continues the numbering where the stage before it stopped (its totals are read from device
// memory; this stage leaves its own for the next).  Because `unique` is in order of first occurrence,
// the unique IDs of a prefix of the list are a prefix of the final unique list, so a stage's part of
// `unique`, of the tier lists and of the miss list is final as soon as the inputs of that stage are
// in the table: the whole-path call compacts [seeds | flat_0] right after hop 0, flat_1 after hop 1,
// and so on, and the row copies of a stage run while the next hop is being sampled.
#pragma once
#include "common.hpp"
#include "hashtable.hpp"
#include "scan.hpp"

#define HELIOS_KERNELS_MAX_SEG 9

namespace helios {

enum CompactMode { kCompactPlain = 0, kCompactNextHop = 1, kCompactLookup = 2 };

struct DedupScratch {
    unsigned long long* table;   // n_slots entries {id:32, first position:32}; all ones = empty
    uint32_t n_slots;            // power of two
    int32_t* slot_of;            // [n] table slot of every input position
    int32_t* index_of_first;     // [n] index in `unique` of a first occurrence (nullable: not wanted)
};

// The rotating tables of the batch de-duplication: batch b of a context uses table b mod kBatchTables,
// so that the table of a finished batch stays readable (helios_make_blocks) while the next batch
// runs, and a table is emptied, off the critical path, by the batch before the one that uses it.
constexpr uint32_t kBatchTables = 3;
struct BatchTables {
    unsigned long long* table0;  // nullable: no batch de-duplication; table t starts at table0 + t * table_stride
    uint64_t table_stride;       // in slots
    int32_t* iof0;               // index_of_first of table t starts at iof0 + t * iof_stride
    uint64_t iof_stride;
    uint32_t n_slots;            // slots in use (power of two)
    int32_t* slot_of;            // [position in the batch's ID list]
    uint32_t which;              // the batch's table, unless BatchVars say otherwise
    __device__ __forceinline__ uint32_t pick(const BatchVars* vars) const { return vars ? vars->table % kBatchTables : which; }
    __device__ __forceinline__ unsigned long long* table(uint32_t t) const { return table0 + t * table_stride; }
    __device__ __forceinline__ int32_t* iof(uint32_t t) const { return iof0 + t * iof_stride; }
};

// The lengths of up to HELIOS_KERNELS_MAX_SEG segments whose concatenation is de-duplicated (each may be
// known only on the device).  The stage handles the segments [first_here, n_seg); those before it only
// fix where it begins.
struct SegLens {
    Count len[HELIOS_KERNELS_MAX_SEG];
    int n_seg;
    int first_here;
};

// What the de-duplication between two hops also computes for the hop that follows: the sample
// counts min(deg, fanout) of the new frontier, scanned into indptr (indptr[n_unique] = total, also
// to *n_flat_dev); size_out (nullable, device-accessible) gets {n_unique, total}.
struct NextHopCount {
    const int64_t* offsets;
    int64_t n_nodes;
    int32_t fanout;
    int64_t* indptr;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;
};
struct TierLists {
    int32_t* pos[2];    // positions in the ID list, per cached tier (0 = HBM, 1 = host)
    int32_t* slot[2];   // row in the tier table
    int64_t* count;     // device int64[3]: entries to copy from tier 0 and tier 1, misses to serve
};
// What the batch's de-duplication also computes: the cache lookup of the unique IDs (see
// launch_lookup_partition, whose outputs these are, with positions = indices into `unique`).
struct LookupOut {
    const int32_t* rank;
    int64_t n_hbm, n_host;
    TierLists lists;
    int32_t *miss_pos, *miss_id, *miss_slot;
    int64_t miss_cap;
    int64_t* stats_out;          // device-accessible int64[4], nullable; written by the last stage
    int64_t* learn;              // pinned int64[4], nullable: the library's own copy of the stats, from which the host
                                 // sizes the grids of the batches that follow
};
// Totals a stage leaves behind in device memory (int64[kStageWords]).
constexpr int kStageUnique = 0, kStageHbm = 1, kStageHost = 2;      // unique IDs, HBM hits, host hits so far
constexpr int kStageHbmCopy = 3, kStageHostCopy = 4;                // list entries that may be copied (none of a stage
                                                                    // whose part of `unique` did not fit its capacity)
constexpr int kStageWords = 8;

struct CompactArgs {
    const int32_t* ids;
    SegLens lens;
    int64_t n_max;               // bound on the inputs of this stage
    int64_t* n_total_dev;        // receives begin + n: the inputs compacted so far (nullable)
    DedupScratch s;              // table / index_of_first are overridden by `batch` when that is set
    BatchTables batch;
    const BatchVars* vars;
    int32_t* unique;
    int64_t unique_cap;
    const int64_t* prev;         // totals of the stage before (nullable: this is the first)
    int64_t* mine;               // totals after this stage (nullable)
    bool last;                   // the last stage writes the outputs below
    int64_t* n_unique_dev;
    int64_t* n_unique_out;       // device-accessible, nullable
    union {                      // a pass is either the batch's (look) or the one between two hops (next), or neither
        LookupOut look;
        NextHopCount next;
    };
    uint32_t* batches_run;       // nullable: the first compaction of a recorded batch counts the batch
    ScanState scan;
    int32_t* err;
    Stamps stamps;
};

template <int MODE>
__device__ __forceinline__ void compact_role(const CompactArgs& a, uint32_t rb, uint32_t nrb) {
    constexpr int NC = MODE == kCompactNextHop ? 2 : MODE == kCompactLookup ? 3 : 1;
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[NC], s_excl[NC];
    __shared__ ScanLookbackLds<NC> s_look;
    stamp_start(a.stamps, rb);
    if (a.batches_run && rb == 0 && threadIdx.x == 0) *a.batches_run += 1;   // every workgroup of the batch's first kernel has read its slot
    DedupScratch s = a.s;
    if (a.batch.table0) {
        const uint32_t t = a.batch.pick(a.vars);
        s = DedupScratch{a.batch.table(t), a.batch.n_slots, a.batch.slot_of, a.batch.iof(t)};
    }
    int64_t begin = 0, n = 0;
#pragma unroll
    for (int k = 0; k < HELIOS_KERNELS_MAX_SEG; ++k) {
        if (k < a.lens.first_here) begin += a.lens.len[k].get();
        else if (k < a.lens.n_seg) n += a.lens.len[k].get();
    }
    n = n < a.n_max ? n : a.n_max;
    const int64_t end = begin + n;
    int64_t base[3] = {0, 0, 0};
    if (a.prev) { base[0] = a.prev[kStageUnique]; base[1] = a.prev[kStageHbm]; base[2] = a.prev[kStageHost]; }
    const int64_t n_tiles = (n + kTileItems - 1) / kTileItems;
    if (rb == 0 && threadIdx.x == 0) {
        if (a.n_total_dev) *a.n_total_dev = end;
        if (n == 0) {                              // an empty stage: the totals pass through
            if (a.mine) {
                a.mine[kStageUnique] = base[0]; a.mine[kStageHbm] = base[1]; a.mine[kStageHost] = base[2];
                a.mine[kStageHbmCopy] = a.prev ? a.prev[kStageHbmCopy] : 0;
                a.mine[kStageHostCopy] = a.prev ? a.prev[kStageHostCopy] : 0;
            }
            if (a.last) {
                *a.n_unique_dev = base[0];
                if (a.n_unique_out) *a.n_unique_out = base[0];
            }
            if (MODE == kCompactNextHop) {
                a.next.indptr[0] = 0;
                *a.next.n_flat_dev = 0;
                if (a.next.size_out) { a.next.size_out[0] = 0; a.next.size_out[1] = 0; }
            }
            if (MODE == kCompactLookup && a.last) {
                const int64_t c2 = base[0] - base[1] - base[2];
                const bool fits = base[0] <= a.unique_cap;
                a.look.lists.count[0] = a.prev ? a.prev[kStageHbmCopy] : 0;
                a.look.lists.count[1] = a.prev ? a.prev[kStageHostCopy] : 0;
                a.look.lists.count[2] = fits ? c2 : 0;
                if (a.look.stats_out) { a.look.stats_out[0] = base[0]; a.look.stats_out[1] = base[1]; a.look.stats_out[2] = base[2]; a.look.stats_out[3] = c2; }
            }
        }
    }
    if (static_cast<int64_t>(rb) >= n_tiles) {
        stamp_end(a.stamps, rb, nrb);
        return;
    }
    const uint32_t tile = scan_take_ticket(a.scan, static_cast<uint32_t>(n_tiles), &s_ticket);
    const int64_t j0 = begin + static_cast<int64_t>(tile) * kTileItems + static_cast<int64_t>(threadIdx.x) * kItemsPerThread;
    int32_t slot[kItemsPerThread], id[kItemsPerThread];
    uint32_t first[kItemsPerThread], cnt[kItemsPerThread];
    int64_t r[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        slot[k] = j0 + k < end ? s.slot_of[j0 + k] : -1;
        id[k] = j0 + k < end ? a.ids[j0 + k] : 0;
    }
    // The table word and the row bounds / the rank are fetched together: those of a repeated ID are
    // read for nothing, but they are in cache and nobody waits for the flag first.  (A slot >= 0
    // means the insert pass found the ID to be a node ID.)
    unsigned long long word[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        if (static_cast<uint32_t>(slot[k]) >= s.n_slots) slot[k] = -1;      // never a slot of this table
        word[k] = slot[k] >= 0 ? s.table[slot[k]] : ~0ull;
        cnt[k] = 0;
        r[k] = 0;
        if (MODE == kCompactNextHop && slot[k] >= 0) cnt[k] = sample_count(a.next.offsets, a.next.n_nodes, id[k], a.next.fanout, a.err);
        if (MODE == kCompactLookup && slot[k] >= 0) r[k] = a.look.rank[id[k]];
    }
    uint32_t n_first = 0, n_second = 0;          // second counter: sample counts, or hits packed as hbm | host << 16
    int tier[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        first[k] = slot[k] >= 0 && static_cast<uint32_t>(word[k]) == static_cast<uint32_t>(j0 + k) ? 1u : 0u;
        if (!first[k]) cnt[k] = 0;
        tier[k] = -1;
        if (MODE == kCompactLookup && first[k]) {
            // a negative rank (the hotness order was no permutation; reported when the map was built, and
            // here) counts as a miss whose slot no table has
            if (r[k] < 0) raise(a.err, kErrData);
            tier[k] = r[k] < 0 ? 2 : r[k] < a.look.n_hbm ? 0 : r[k] < a.look.n_hbm + a.look.n_host ? 1 : 2;
            n_second += tier[k] == 0 ? 1u : tier[k] == 1 ? (1u << 16) : 0u;
        }
        n_first += first[k];
        if (MODE == kCompactNextHop) n_second += cnt[k];
    }

    uint32_t tile_first, tile_second = 0;
    const uint32_t local_first = block_exclusive_scan(n_first, s_wave, tile_first);
    uint32_t local_second = 0;
    if (MODE != kCompactPlain) local_second = block_exclusive_scan(n_second, s_wave, tile_second);
    if (threadIdx.x == 0) {
        s_agg[0] = tile_first;
        if (MODE == kCompactNextHop) s_agg[NC - 1] = tile_second;
        if (MODE == kCompactLookup) {
            s_agg[NC - 2] = tile_second & 0xffffu;
            s_agg[NC - 1] = tile_second >> 16;
        }
    }
    scan_chained_prefix<NC>(a.scan, tile, s_agg, s_excl, &s_look, a.err);
    int64_t at = base[0] + static_cast<int64_t>(s_excl[0]) + local_first;
    int64_t at_cnt = MODE == kCompactNextHop ? static_cast<int64_t>(s_excl[NC - 1]) + local_second : 0;
    int64_t at_tier[3] = {0, 0, 0};
    if (MODE == kCompactLookup) {
        at_tier[0] = base[1] + static_cast<int64_t>(s_excl[NC - 2]) + (local_second & 0xffffu);
        at_tier[1] = base[2] + static_cast<int64_t>(s_excl[NC - 1]) + (local_second >> 16);
        at_tier[2] = at - at_tier[0] - at_tier[1];           // every unique ID is in exactly one class
    }
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        if (first[k]) {
            if (s.index_of_first) s.index_of_first[j0 + k] = static_cast<int32_t>(at);
            if (MODE == kCompactNextHop && at == a.unique_cap) {
                // the frontier is cut off here: the next hop samples the nodes that fit, and its sample list
                // ends where this node's samples would have begun
                a.next.indptr[a.unique_cap] = at_cnt;
                *a.next.n_flat_dev = at_cnt;
            }
            if (at < a.unique_cap) {
                a.unique[at] = id[k];
                if (MODE == kCompactNextHop) a.next.indptr[at] = at_cnt;
                if (MODE == kCompactLookup) {
                    const int t = tier[k];
                    const int64_t w = at_tier[t];
                    const int32_t sl = static_cast<int32_t>(t == 0 ? r[k] : t == 1 ? r[k] - a.look.n_hbm
                                                             : r[k] < 0 ? -1 : r[k] - a.look.n_hbm - a.look.n_host);
                    if (t < 2) {
                        a.look.lists.pos[t][w] = static_cast<int32_t>(at);
                        a.look.lists.slot[t][w] = sl;
                    } else if (w < a.look.miss_cap) {
                        a.look.miss_pos[w] = static_cast<int32_t>(at);
                        a.look.miss_id[w] = id[k];
                        a.look.miss_slot[w] = sl;
                    }
                }
            }
            if (MODE == kCompactLookup) at_tier[tier[k]] += 1;
            at += 1;
            at_cnt += cnt[k];
        }
    }
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = base[0] + static_cast<int64_t>(s_excl[0]) + tile_first;
        const bool fits = total <= a.unique_cap;
        if (a.last) {
            *a.n_unique_dev = total;
            if (a.n_unique_out) *a.n_unique_out = total;
        }
        if (!fits) raise(a.err, kErrCapacity);
        if (a.mine) a.mine[kStageUnique] = total;
        if (MODE == kCompactNextHop) {
            const int64_t total_cnt = static_cast<int64_t>(s_excl[NC - 1]) + tile_second;
            if (fits) {                          // else the thread at the cut has written both
                a.next.indptr[total] = total_cnt;
                *a.next.n_flat_dev = total_cnt;
            }
            if (a.next.size_out) { a.next.size_out[0] = total; a.next.size_out[1] = total_cnt; }
            if (total_cnt > a.next.flat_cap) raise(a.err, kErrCapacity);
        }
        if (MODE == kCompactLookup) {
            const int64_t c0 = base[1] + static_cast<int64_t>(s_excl[NC - 2]) + (tile_second & 0xffffu);
            const int64_t c1 = base[2] + static_cast<int64_t>(s_excl[NC - 1]) + (tile_second >> 16);
            const int64_t c2 = total - c0 - c1;
            // if `unique` overflowed, list entries past its capacity were not written: this stage's are not copied
            const int64_t copy0 = fits ? c0 : (a.prev ? a.prev[kStageHbmCopy] : 0);
            const int64_t copy1 = fits ? c1 : (a.prev ? a.prev[kStageHostCopy] : 0);
            if (a.mine) {
                a.mine[kStageHbm] = c0; a.mine[kStageHost] = c1;
                a.mine[kStageHbmCopy] = copy0; a.mine[kStageHostCopy] = copy1;
            }
            if (a.last) {
                a.look.lists.count[0] = copy0; a.look.lists.count[1] = copy1; a.look.lists.count[2] = fits ? c2 : 0;
                if (a.look.stats_out) { a.look.stats_out[0] = total; a.look.stats_out[1] = c0; a.look.stats_out[2] = c1; a.look.stats_out[3] = c2; }
                if (a.look.learn) { a.look.learn[0] = total; a.look.learn[1] = c0; a.look.learn[2] = c1; a.look.learn[3] = c2; }
                if (c2 > a.look.miss_cap) raise(a.err, kErrCapacity);
            }
        }
    }
    stamp_end(a.stamps, rb, nrb);
}

struct InverseArgs {
    Count n;                     // inputs of the list (a device count written by the compaction)
    DedupScratch s;
    BatchTables batch;
    const BatchVars* vars;
    int32_t* inverse;
    Stamps stamps;
};

// Third pass (optional): inverse[j] = index in unique of input j.
__device__ __forceinline__ void inverse_role(const InverseArgs& a, uint32_t rb, uint32_t nrb) {
    stamp_start(a.stamps, rb);
    DedupScratch s = a.s;
    if (a.batch.table0) {
        const uint32_t t = a.batch.pick(a.vars);
        s = DedupScratch{a.batch.table(t), a.batch.n_slots, a.batch.slot_of, a.batch.iof(t)};
    }
    const int64_t n = a.n.get();
    for (int64_t j = static_cast<int64_t>(rb) * kBlock + threadIdx.x; j < n; j += static_cast<int64_t>(nrb) * kBlock) {
        const int32_t slot = s.slot_of[j];
        int32_t inv = -1;
        if (static_cast<uint32_t>(slot) < s.n_slots) {
            const uint32_t first = static_cast<uint32_t>(s.table[slot]);      // position of the ID's first occurrence
            if (static_cast<int64_t>(first) < n) inv = s.index_of_first[first];
        }
        a.inverse[j] = inv;
    }
    stamp_end(a.stamps, rb, nrb);
}

}  // namespace helios
