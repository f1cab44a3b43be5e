// Cache map and cache lookup.
//
// rank_build: rank[order[r]] = r, with a check that order is a permutation.
//
// lookup_partition: one thread per ID reads rank[id] (one random 4-byte read),
// classifies it into the HBM tier, the host tier or a miss by two compares, and
// the three classes are compacted *stably* in one pass: a thread takes four
// consecutive IDs, a workgroup scan gives the in-tile ranks and a three-counter
// chained scan (scan.hpp) the ranks across workgroups.  The two hit lists (position, slot)
// feed the row-copy kernels; the miss list (position, id, slot) is the request
// list of the storage tier and comes out ascending in position.
#include "kernels.hpp"

namespace helios {

namespace {

__global__ __launch_bounds__(kBlock) void rank_fill_kernel(int32_t* rank, int64_t n) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * kBlock)
        rank[i] = -1;
}

__global__ __launch_bounds__(kBlock) void rank_scatter_kernel(const int32_t* __restrict__ order, int64_t n, int32_t* rank,
                                                              int32_t* err) {
    for (int64_t r = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; r < n;
         r += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int32_t v = order[r];
        if (v < 0 || static_cast<int64_t>(v) >= n) raise(err, kErrData);
        else rank[v] = static_cast<int32_t>(r);
    }
}

// a node that no rank points to means `order` repeated another node
__global__ __launch_bounds__(kBlock) void rank_check_kernel(const int32_t* __restrict__ rank, int64_t n, int32_t* err) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * kBlock)
        if (rank[i] < 0) raise(err, kErrData);
}

struct PartitionArgs {
    const int32_t* ids;
    Count n;
    const int32_t* rank;
    int64_t n_nodes, n_hbm, n_host;
    TierLists lists;
    int32_t *miss_pos, *miss_id, *miss_slot;
    int64_t miss_cap;
    int64_t* stats_out;          // device-accessible int64[4], nullable
    int64_t* learn;              // pinned int64[4], nullable: a copy of the stats for the host's grid sizing
    ScanState scan;
    int32_t* err;
};

__global__ __launch_bounds__(kBlock) void lookup_partition_kernel(PartitionArgs a) {
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[3], s_excl[3];
    __shared__ ScanLookbackLds<3> s_look;
    const int64_t n = a.n.get();
    const int64_t n_tiles = (n + kTileItems - 1) / kTileItems;
    if (n == 0 && blockIdx.x == 0 && threadIdx.x == 0) {
        a.lists.count[0] = a.lists.count[1] = a.lists.count[2] = 0;
        if (a.stats_out) { a.stats_out[0] = 0; a.stats_out[1] = 0; a.stats_out[2] = 0; a.stats_out[3] = 0; }
    }
    if (static_cast<int64_t>(blockIdx.x) >= n_tiles) return;
    const uint32_t tile = scan_take_ticket(a.scan, static_cast<uint32_t>(n_tiles), &s_ticket);

    // a thread takes four consecutive IDs: all four rank reads are in flight together
    const int64_t j0 = static_cast<int64_t>(tile) * kTileItems + static_cast<int64_t>(threadIdx.x) * kItemsPerThread;
    int32_t id[kItemsPerThread], slot[kItemsPerThread];
    int tier[kItemsPerThread];               // -1: no ID here (tail of the last tile, or a bad ID)
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) id[k] = j0 + k < n ? a.ids[j0 + k] : -1;
    int64_t r[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        const bool ok = id[k] >= 0 && static_cast<int64_t>(id[k]) < a.n_nodes;
        if (j0 + k < n && !ok) raise(a.err, kErrData);
        r[k] = ok ? static_cast<int64_t>(a.rank[id[k]]) : -1;
    }
    uint32_t c_hbm = 0, c_host = 0, c_miss = 0;
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        tier[k] = -1;
        slot[k] = 0;
        if (r[k] >= 0) {
            if (r[k] < a.n_hbm) { tier[k] = 0; slot[k] = static_cast<int32_t>(r[k]); ++c_hbm; }
            else if (r[k] < a.n_hbm + a.n_host) { tier[k] = 1; slot[k] = static_cast<int32_t>(r[k] - a.n_hbm); ++c_host; }
            else { tier[k] = 2; slot[k] = static_cast<int32_t>(r[k] - a.n_hbm - a.n_host); ++c_miss; }
        }
    }
    // ranks inside the workgroup: the two hit classes share one scan (16 bits each, a tile has 1024 IDs)
    uint32_t tot_hits, tot_miss;
    const uint32_t before_hits = block_exclusive_scan(c_hbm | (c_host << 16), s_wave, tot_hits);
    const uint32_t before_miss = block_exclusive_scan(c_miss, s_wave, tot_miss);
    if (threadIdx.x == 0) {
        s_agg[0] = tot_hits & 0xffffu;
        s_agg[1] = tot_hits >> 16;
        s_agg[2] = tot_miss;
    }
    scan_chained_prefix<3>(a.scan, tile, s_agg, s_excl, &s_look, a.err);
    int64_t at[3] = {static_cast<int64_t>(s_excl[0]) + (before_hits & 0xffffu),
                     static_cast<int64_t>(s_excl[1]) + (before_hits >> 16),
                     static_cast<int64_t>(s_excl[2]) + before_miss};
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        if (tier[k] < 0) continue;
        const int64_t w = tier[k] == 0 ? at[0]++ : tier[k] == 1 ? at[1]++ : at[2]++;
        if (tier[k] < 2) {
            a.lists.pos[tier[k]][w] = static_cast<int32_t>(j0 + k);
            a.lists.slot[tier[k]][w] = slot[k];
        } else if (w < a.miss_cap) {
            a.miss_pos[w] = static_cast<int32_t>(j0 + k);
            a.miss_id[w] = id[k];
            a.miss_slot[w] = slot[k];
        }
    }
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t c0 = static_cast<int64_t>(s_excl[0]) + s_agg[0];
        const int64_t c1 = static_cast<int64_t>(s_excl[1]) + s_agg[1];
        const int64_t c2 = static_cast<int64_t>(s_excl[2]) + s_agg[2];
        a.lists.count[0] = c0; a.lists.count[1] = c1; a.lists.count[2] = c2;
        if (a.stats_out) { a.stats_out[0] = n; a.stats_out[1] = c0; a.stats_out[2] = c1; a.stats_out[3] = c2; }
        if (a.learn) { a.learn[0] = n; a.learn[1] = c0; a.learn[2] = c1; a.learn[3] = c2; }
        if (c2 > a.miss_cap) raise(a.err, kErrCapacity);
    }
}

unsigned grid_for(int64_t n, unsigned cap_blocks) {
    int64_t b = (n + kBlock - 1) / kBlock;
    if (b < 1) b = 1;
    if (b > cap_blocks) b = cap_blocks;
    return static_cast<unsigned>(b);
}

}  // namespace

hipError_t launch_rank_build(hipStream_t stream, const int32_t* order, int64_t n_nodes, int32_t* rank, int32_t* err) {
    const dim3 grid(grid_for(n_nodes, 8192)), block(kBlock);
    hipLaunchKernelGGL(rank_fill_kernel, grid, block, 0, stream, rank, n_nodes);
    hipLaunchKernelGGL(rank_scatter_kernel, grid, block, 0, stream, order, n_nodes, rank, err);
    hipLaunchKernelGGL(rank_check_kernel, grid, block, 0, stream, rank, n_nodes, err);
    return hipGetLastError();
}

hipError_t launch_lookup_partition(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max,
                                   const int32_t* rank, int64_t n_nodes, int64_t n_hbm, int64_t n_host,
                                   const TierLists& lists, int32_t* miss_pos, int32_t* miss_id,
                                   int32_t* miss_slot, int64_t miss_cap, int64_t* stats_out, int64_t* learn,
                                   const ScanState& scan, int32_t* err) {
    PartitionArgs a{ids, n, rank, n_nodes, n_hbm, n_host, lists, miss_pos, miss_id, miss_slot, miss_cap,
                    stats_out, learn, scan, err};
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    if (tiles < 1) tiles = 1;
    hipLaunchKernelGGL(lookup_partition_kernel, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
