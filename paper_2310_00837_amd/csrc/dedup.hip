// Order-preserving de-duplication of an ID list.
//
// unique = the distinct IDs in order of first occurrence.  The order is made
// independent of thread scheduling by keeping, per distinct ID, the smallest
// input position that holds it:
//   1. insert: an open-addressing hash table of 64-bit words {id:32 | pos:32}
//      (hashtable.hpp).  The slot of every input is remembered.  For IDs that
//      the sampling kernel produces, that kernel does the inserting as it writes
//      them (sample.hip); the insert kernel here serves helios_dedup.
//   2. compact: input j is a first occurrence iff its slot's position is j; the
//      flags are scanned in-workgroup and chained across workgroups, so the
//      unique list comes out in input order in the same pass.  Between hops
//      this pass also counts the samples of every new frontier node.
//   3. inverse (optional): every input looks up the unique index of its ID's
//      first occurrence.
// The table has at least twice as many slots as inputs and is cleared by the
// same stream before use; at the sizes of one mini-batch (at most 16 MB) it
// stays in L2 / MALL.  It is not staged through LDS: a batch's ID list has few
// repeats (3-20 % in the power-law workloads; the hubs that repeat are spread
// over the whole list), so a per-workgroup LDS table would catch little and
// every survivor would go to the global table anyway.
#include "kernels.hpp"

namespace helios {

namespace {

__global__ __launch_bounds__(kBlock) void dedup_clear_kernel(ClearJob c) { clear_slots(c); }

__global__ __launch_bounds__(kBlock) void dedup_insert_kernel(const int32_t* __restrict__ ids, Count n_in, int64_t n_nodes,
                                                              DedupScratch s, int32_t* err) {
    // The first ID is fetched before the device-side count has arrived (the buffer holds n_in.host
    // entries, so the read is in bounds whatever the count turns out to be).
    const int64_t j0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    int32_t early = 0;
    if (j0 < n_in.host) early = ids[j0];
    const int64_t n = n_in.get();
    const uint32_t mask = s.n_slots - 1;
    for (int64_t j = j0; j < n; j += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int32_t id = j == j0 ? early : ids[j];
        if (id < 0 || static_cast<int64_t>(id) >= n_nodes) {
            raise(err, kErrData);
            s.slot_of[j] = -1;
            continue;
        }
        s.slot_of[j] = static_cast<int32_t>(table_insert(s.table, mask, static_cast<uint32_t>(id), static_cast<uint32_t>(j)));
    }
}

// Pass 2.  Input j is a first occurrence iff its slot's position is j.  A thread takes four
// consecutive inputs; the flags are scanned in the workgroup and chained across workgroups, so
// `unique` comes out in input order.  The pass has the new unique IDs in registers, so two things
// that need them ride on it instead of being kernels of their own:
//   kCompactNextHop  the unique list is the frontier of the next hop: read every new frontier node's
//                    row bounds and scan the sample counts min(deg, fanout) as a second counter,
//                    which gives that hop its indptr;
//   kCompactLookup   the unique list is the batch's ID list: read rank[id], classify into HBM tier,
//                    host tier or miss, and scan the two hit classes as further counters (the miss
//                    rank is what is left), which gives the stable per-tier lists and the miss list
//                    that cache.hip's stand-alone lookup kernel would produce from `unique`.
enum CompactMode { kCompactPlain = 0, kCompactNextHop = 1, kCompactLookup = 2 };

template <int MODE>
__global__ __launch_bounds__(kBlock) void dedup_compact_kernel(const int32_t* __restrict__ ids, SegLens lens, int64_t n_max,
                                                               int64_t* n_total_dev, DedupScratch s,
                                                               int32_t* unique, int64_t unique_cap,
                                                               int64_t* n_unique_dev, int64_t* n_unique_out,
                                                               NextHopCount next, LookupOut look, ScanState scan,
                                                               int32_t* err) {
    constexpr int NC = MODE == kCompactNextHop ? 2 : MODE == kCompactLookup ? 3 : 1;
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[NC], s_excl[NC];
    __shared__ ScanLookbackLds<NC> s_look;
    int64_t n = 0;
#pragma unroll
    for (int k = 0; k < HELIOS_KERNELS_MAX_SEG; ++k)
        if (k < lens.n_seg) n += lens.len[k].get();
    n = n < n_max ? n : n_max;
    const int64_t n_tiles = (n + kTileItems - 1) / kTileItems;
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_total_dev = n;
    if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        *n_unique_dev = 0;
        if (n_unique_out) *n_unique_out = 0;
        if (MODE == kCompactNextHop) {
            next.indptr[0] = 0;
            *next.n_flat_dev = 0;
            if (next.size_out) { next.size_out[0] = 0; next.size_out[1] = 0; }
        }
        if (MODE == kCompactLookup) {
            look.lists.count[0] = look.lists.count[1] = look.lists.count[2] = 0;
            if (look.stats_out) { look.stats_out[0] = 0; look.stats_out[1] = 0; look.stats_out[2] = 0; look.stats_out[3] = 0; }
        }
    }
    if (static_cast<int64_t>(blockIdx.x) >= n_tiles) return;
    const uint32_t tile = scan_take_ticket(scan, static_cast<uint32_t>(n_tiles), &s_ticket);
    const int64_t j0 = static_cast<int64_t>(tile) * kTileItems + static_cast<int64_t>(threadIdx.x) * kItemsPerThread;
    int32_t slot[kItemsPerThread], id[kItemsPerThread];
    uint32_t first[kItemsPerThread], cnt[kItemsPerThread];
    int64_t r[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        slot[k] = j0 + k < n ? s.slot_of[j0 + k] : -1;
        id[k] = j0 + k < n ? ids[j0 + k] : 0;
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
        if (MODE == kCompactNextHop && slot[k] >= 0) cnt[k] = sample_count(next.offsets, next.n_nodes, id[k], next.fanout, err);
        if (MODE == kCompactLookup && slot[k] >= 0) r[k] = look.rank[id[k]];
    }
    uint32_t n_first = 0, n_second = 0;          // second counter: sample counts, or hits packed as hbm | host << 16
    int tier[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        first[k] = slot[k] >= 0 && static_cast<uint32_t>(word[k]) == static_cast<uint32_t>(j0 + k) ? 1u : 0u;
        if (!first[k]) cnt[k] = 0;
        tier[k] = -1;
        if (MODE == kCompactLookup && first[k]) {
            tier[k] = r[k] < look.n_hbm ? 0 : r[k] < look.n_hbm + look.n_host ? 1 : 2;
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
    scan_chained_prefix<NC>(scan, tile, s_agg, s_excl, &s_look, err);
    int64_t at = static_cast<int64_t>(s_excl[0]) + local_first;
    int64_t at_cnt = MODE == kCompactNextHop ? static_cast<int64_t>(s_excl[NC - 1]) + local_second : 0;
    int64_t at_tier[3] = {0, 0, 0};
    if (MODE == kCompactLookup) {
        at_tier[0] = static_cast<int64_t>(s_excl[NC - 2]) + (local_second & 0xffffu);
        at_tier[1] = static_cast<int64_t>(s_excl[NC - 1]) + (local_second >> 16);
        at_tier[2] = at - at_tier[0] - at_tier[1];           // every unique ID is in exactly one class
    }
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        if (first[k]) {
            s.index_of_first[j0 + k] = static_cast<int32_t>(at);
            if (MODE == kCompactNextHop && at == unique_cap) {
                // the frontier is cut off here: the next hop samples the nodes that fit, and its sample list
                // ends where this node's samples would have begun
                next.indptr[unique_cap] = at_cnt;
                *next.n_flat_dev = at_cnt;
            }
            if (at < unique_cap) {
                unique[at] = id[k];
                if (MODE == kCompactNextHop) next.indptr[at] = at_cnt;
                if (MODE == kCompactLookup) {
                    const int t = tier[k];
                    const int64_t w = at_tier[t];
                    const int32_t sl = static_cast<int32_t>(t == 0 ? r[k] : t == 1 ? r[k] - look.n_hbm
                                                                                   : r[k] - look.n_hbm - look.n_host);
                    if (t < 2) {
                        look.lists.pos[t][w] = static_cast<int32_t>(at);
                        look.lists.slot[t][w] = sl;
                    } else if (w < look.miss_cap) {
                        look.miss_pos[w] = static_cast<int32_t>(at);
                        look.miss_id[w] = id[k];
                        look.miss_slot[w] = sl;
                    }
                }
            }
            if (MODE == kCompactLookup) at_tier[tier[k]] += 1;
            at += 1;
            at_cnt += cnt[k];
        }
    }
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = static_cast<int64_t>(s_excl[0]) + tile_first;
        *n_unique_dev = total;
        if (n_unique_out) *n_unique_out = total;
        if (total > unique_cap) raise(err, kErrCapacity);
        if (MODE == kCompactNextHop) {
            const int64_t total_cnt = static_cast<int64_t>(s_excl[NC - 1]) + tile_second;
            if (total <= unique_cap) {           // else the thread at the cut has written both
                next.indptr[total] = total_cnt;
                *next.n_flat_dev = total_cnt;
            }
            if (next.size_out) { next.size_out[0] = total; next.size_out[1] = total_cnt; }
            if (total_cnt > next.flat_cap) raise(err, kErrCapacity);
        }
        if (MODE == kCompactLookup) {
            const int64_t c0 = static_cast<int64_t>(s_excl[NC - 2]) + (tile_second & 0xffffu);
            const int64_t c1 = static_cast<int64_t>(s_excl[NC - 1]) + (tile_second >> 16);
            const int64_t c2 = total - c0 - c1;
            // if `unique` overflowed, list entries past its capacity were not written: copy nothing then
            const bool fits = total <= unique_cap;
            look.lists.count[0] = fits ? c0 : 0; look.lists.count[1] = fits ? c1 : 0; look.lists.count[2] = c2;
            if (look.stats_out) { look.stats_out[0] = total; look.stats_out[1] = c0; look.stats_out[2] = c1; look.stats_out[3] = c2; }
            if (c2 > look.miss_cap) raise(err, kErrCapacity);
        }
    }
}

__global__ __launch_bounds__(kBlock) void dedup_inverse_kernel(Count n_in, DedupScratch s, int32_t* inverse) {
    const int64_t n = n_in.get();      // written by the compaction pass
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; j < n;
         j += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int32_t slot = s.slot_of[j];
        int32_t inv = -1;
        if (static_cast<uint32_t>(slot) < s.n_slots) {
            const uint32_t first = static_cast<uint32_t>(s.table[slot]);      // position of the ID's first occurrence
            if (static_cast<int64_t>(first) < n) inv = s.index_of_first[first];
        }
        inverse[j] = inv;
    }
}

unsigned grid_for(int64_t n_max, unsigned cap_blocks) {
    int64_t b = (n_max + kBlock - 1) / kBlock;
    if (b < 1) b = 1;
    if (b > cap_blocks) b = cap_blocks;
    return static_cast<unsigned>(b);
}

}  // namespace

hipError_t launch_dedup_insert(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                               const DedupScratch& s, bool table_is_clear, int32_t* err) {
    const dim3 block(kBlock);
    if (!table_is_clear)
        hipLaunchKernelGGL(dedup_clear_kernel, dim3(grid_for(s.n_slots, 2048)), block, 0, stream, ClearJob{s.table, s.n_slots});
    hipLaunchKernelGGL(dedup_insert_kernel, dim3(grid_for(n_max, 4096)), block, 0, stream, ids, n, n_nodes, s, err);
    return hipGetLastError();
}

hipError_t launch_dedup_compact(hipStream_t stream, const int32_t* ids, const SegLens& lens, int64_t n_max,
                                int64_t* n_total_dev, const DedupScratch& s, int32_t* unique, int64_t unique_cap,
                                int64_t* n_unique_dev, int64_t* n_unique_out, const NextHopCount* next, const LookupOut* look,
                                const ScanState& scan, int32_t* err) {
    const dim3 block(kBlock);
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    if (tiles < 1) tiles = 1;
    const dim3 grid(static_cast<unsigned>(tiles));
    if (next)
        hipLaunchKernelGGL(dedup_compact_kernel<kCompactNextHop>, grid, block, 0, stream, ids, lens, n_max, n_total_dev, s,
                           unique, unique_cap, n_unique_dev, n_unique_out, *next, LookupOut{}, scan, err);
    else if (look)
        hipLaunchKernelGGL(dedup_compact_kernel<kCompactLookup>, grid, block, 0, stream, ids, lens, n_max, n_total_dev, s,
                           unique, unique_cap, n_unique_dev, n_unique_out, NextHopCount{}, *look, scan, err);
    else
        hipLaunchKernelGGL(dedup_compact_kernel<kCompactPlain>, grid, block, 0, stream, ids, lens, n_max, n_total_dev, s,
                           unique, unique_cap, n_unique_dev, n_unique_out, NextHopCount{}, LookupOut{}, scan, err);
    return hipGetLastError();
}

hipError_t launch_dedup_inverse(hipStream_t stream, const int64_t* n_total_dev, int64_t n_max, const DedupScratch& s,
                                int32_t* inverse) {
    hipLaunchKernelGGL(dedup_inverse_kernel, dim3(grid_for(n_max, 4096)), dim3(kBlock), 0, stream, Count{n_total_dev, n_max},
                       s, inverse);
    return hipGetLastError();
}

}  // namespace helios
