// Count pass of hop 0 as a kernel of its own, for seed lists too long for the count that the
// sampling pass folds in (sample_dev.hpp): one thread per four frontier nodes reads the row bounds,
// the sample counts min(deg, fanout) are scanned in the workgroup and chained across workgroups
// (scan.hpp) into indptr, each node's place in `flat`.
#include "kernels.hpp"

namespace helios {

namespace {

struct CountArgs {
    const int64_t* offsets;
    int64_t n_nodes;
    const int32_t* frontier;
    BatchFeed feed;               // recorded batch: the batch's variables come from the host's ring, and the frontier is their seeds
    int32_t* frontier_out;        // nullable: receives a copy of the frontier
    Count n;
    int32_t fanout;
    int64_t* indptr;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;            // nullable: [0] = frontier size, [1] = sample-list size
    ScanState scan;
    int32_t* err;
};

__global__ __launch_bounds__(kBlock) void frontier_count_kernel(CountArgs a) {
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[1], s_excl[1];
    __shared__ ScanLookbackLds<1> s_look;
    // A recorded batch starts here: every workgroup reads the batch's variables from the slot of the host's ring
    // that the count of batches run so far selects, and the first workgroup leaves them in device memory for the
    // kernels that follow (the batch's first compaction advances the count).
    BatchVars bv{};
    if (a.feed.ring) bv = a.feed.ring[*a.feed.batches_run % a.feed.ring_slots];
    ScanState scan = a.scan;
    if (a.feed.ring) {
        scan.vars = nullptr;
        scan.epoch += bv.epoch_base;
        if (blockIdx.x == 0 && threadIdx.x == 0) *a.feed.vars_out = bv;
    }
    const int64_t n = a.n.get();
    const int64_t n_tiles = (n + kTileItems - 1) / kTileItems;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (a.size_out) a.size_out[0] = n;
        if (n == 0) {                            // empty frontier: empty hop
            a.indptr[0] = 0;
            *a.n_flat_dev = 0;
            if (a.size_out) a.size_out[1] = 0;
        }
    }
    if (static_cast<int64_t>(blockIdx.x) >= n_tiles) return;
    const uint32_t tile = scan_take_ticket(scan, static_cast<uint32_t>(n_tiles), &s_ticket);
    const int32_t* frontier = a.feed.ring ? bv.seeds : a.frontier;
    const int64_t j0 = static_cast<int64_t>(tile) * kTileItems + static_cast<int64_t>(threadIdx.x) * kItemsPerThread;
    int32_t v[kItemsPerThread];
    uint32_t cnt[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) v[k] = j0 + k < n ? frontier[j0 + k] : -1;
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        cnt[k] = 0;
        if (j0 + k < n) {
            if (a.frontier_out && a.frontier_out != frontier) a.frontier_out[j0 + k] = v[k];
            cnt[k] = sample_count(a.offsets, a.n_nodes, v[k], a.fanout, a.err);
        }
        sum += cnt[k];
    }
    uint32_t tile_total;
    const uint32_t local = block_exclusive_scan(sum, s_wave, tile_total);
    if (threadIdx.x == 0) s_agg[0] = tile_total;
    scan_chained_prefix<1>(scan, tile, s_agg, s_excl, &s_look, a.err);
    int64_t at = static_cast<int64_t>(s_excl[0]) + local;
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        if (j0 + k < n) a.indptr[j0 + k] = at;
        at += cnt[k];
    }
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = static_cast<int64_t>(s_excl[0]) + tile_total;
        a.indptr[n] = total;
        *a.n_flat_dev = total;
        if (a.size_out) a.size_out[1] = total;
        if (total > a.flat_cap) raise(a.err, kErrCapacity);
    }
}

}  // namespace

hipError_t launch_frontier_count(hipStream_t stream, const CsrView& g, const int32_t* frontier, const BatchFeed& feed,
                                 int32_t* frontier_out, Count n, int64_t n_max, int32_t fanout, int64_t* indptr,
                                 int64_t flat_cap, int64_t* n_flat_dev, int64_t* size_out, const ScanState& scan, int32_t* err) {
    CountArgs a{g.offsets, g.n_nodes, frontier, feed, frontier_out, n, fanout, indptr, flat_cap, n_flat_dev, size_out, scan, err};
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    if (tiles < 1) tiles = 1;                  // the first workgroup also writes the sizes of an empty hop
    hipLaunchKernelGGL(frontier_count_kernel, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
