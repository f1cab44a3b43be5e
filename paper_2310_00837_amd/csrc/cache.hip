// Cache map and cache lookup.
//
// rank_build: rank[order[r]] = r, with a check that order is a permutation.
//
// lookup_partition: one thread per ID reads rank[id] (one random 4-byte read),
// classifies it into the HBM tier, the host tier or a miss by two compares, and
// the three classes are compacted *stably* in one pass: wave ballots give the
// in-wave ranks, LDS the in-workgroup ranks, and a three-counter chained scan
// (scan.hpp) the ranks across workgroups.  The two hit lists (position, slot)
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
    ScanState scan;
    int32_t* err;
};

__global__ __launch_bounds__(kBlock) void lookup_partition_kernel(PartitionArgs a) {
    __shared__ uint32_t s_wave_cnt[3][kWavesPerBlock];
    __shared__ uint32_t s_agg[3], s_excl[3];
    __shared__ ScanLookbackLds<3> s_look;
    const uint32_t tile = blockIdx.x;
    const int64_t j = static_cast<int64_t>(tile) * kBlock + threadIdx.x;
    // the ID and its rank are fetched before the device-side count has arrived (ids has room for
    // a.n.host entries; a value that is no node ID is simply not looked up)
    int32_t id = j < a.n.host ? a.ids[j] : -1;
    const bool id_ok = id >= 0 && static_cast<int64_t>(id) < a.n_nodes;
    const int64_t r = id_ok ? static_cast<int64_t>(a.rank[id]) : 0;
    const int64_t n = a.n.get();
    const int64_t n_tiles = (n + kBlock - 1) / kBlock;
    if (n == 0 && tile == 0 && threadIdx.x == 0) {
        a.lists.count[0] = a.lists.count[1] = a.lists.count[2] = 0;
        if (a.stats_out) { a.stats_out[0] = 0; a.stats_out[1] = 0; a.stats_out[2] = 0; a.stats_out[3] = 0; }
    }
    if (static_cast<int64_t>(tile) >= n_tiles) return;

    int tier = -1;                       // -1: no ID here (tail of the last tile, or a bad ID)
    int32_t slot = 0;
    if (j < n) {
        if (!id_ok) {
            raise(a.err, kErrData);
        } else {
            if (r < a.n_hbm) { tier = 0; slot = static_cast<int32_t>(r); }
            else if (r < a.n_hbm + a.n_host) { tier = 1; slot = static_cast<int32_t>(r - a.n_hbm); }
            else { tier = 2; slot = static_cast<int32_t>(r - a.n_hbm - a.n_host); }
        }
    }
    // rank inside the wave, per class
    const int lane = lane_id();
    const unsigned long long below = (1ull << lane) - 1ull;
    uint32_t in_wave = 0;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        const unsigned long long m = __ballot(tier == c);
        if (tier == c) in_wave = static_cast<uint32_t>(__popcll(m & below));
        if (lane == 0) s_wave_cnt[c][wave_id()] = static_cast<uint32_t>(__popcll(m));
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        uint32_t t = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) t += s_wave_cnt[threadIdx.x][w];
        s_agg[threadIdx.x] = t;
    }
    scan_chained_prefix<3>(a.scan, tile, s_agg, s_excl, &s_look, a.err);
    if (tier >= 0) {
        uint32_t before = 0;
        for (int w = 0; w < wave_id(); ++w) before += s_wave_cnt[tier][w];
        const int64_t at = static_cast<int64_t>(s_excl[tier]) + before + in_wave;
        if (tier < 2) {
            a.lists.pos[tier][at] = static_cast<int32_t>(j);
            a.lists.slot[tier][at] = slot;
        } else if (at < a.miss_cap) {
            a.miss_pos[at] = static_cast<int32_t>(j);
            a.miss_id[at] = id;
            a.miss_slot[at] = slot;
        }
    }
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t c0 = static_cast<int64_t>(s_excl[0]) + s_agg[0];
        const int64_t c1 = static_cast<int64_t>(s_excl[1]) + s_agg[1];
        const int64_t c2 = static_cast<int64_t>(s_excl[2]) + s_agg[2];
        a.lists.count[0] = c0; a.lists.count[1] = c1; a.lists.count[2] = c2;
        if (a.stats_out) { a.stats_out[0] = n; a.stats_out[1] = c0; a.stats_out[2] = c1; a.stats_out[3] = c2; }
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
                                   int32_t* miss_slot, int64_t miss_cap, int64_t* stats_out,
                                   const ScanState& scan, int32_t* err) {
    PartitionArgs a{ids, n, rank, n_nodes, n_hbm, n_host, lists, miss_pos, miss_id, miss_slot, miss_cap,
                    stats_out, scan, err};
    int64_t tiles = (n_max + kBlock - 1) / kBlock;
    if (tiles < 1) tiles = 1;
    hipLaunchKernelGGL(lookup_partition_kernel, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
