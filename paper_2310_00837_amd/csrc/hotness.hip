// Pre-sampling hotness: per-node counters and the hotness order.
//
// hotness_add: one batch's de-duplicated ID list adds one to each of its nodes'
// counters.  The IDs of a call are distinct, so the atomic adds of one call
// never meet on an address; calls on different streams may.
//
// hotness_order: nodes sorted by counter, descending, ties by ascending ID: a
// stable least-significant-digit radix sort of (count, id) pairs whose ids
// start out ascending.  A digit is two bits, so a pass is a stable four-way
// partition: one kernel counts every digit of every pass beforehand (where
// each class of a pass begins), and a pass then places every pair by a
// three-counter chained scan (scan.hpp; the fourth class is what is left),
// which keeps the order inside a class.  Classes go out in descending digit
// order, so the last pass leaves the counts descending.  Sixteen passes over
// the node list, once per cache build, not on the per-batch path.
#include "kernels.hpp"

namespace helios {

namespace {

constexpr int kSortItems = 8;                             // pairs per thread
constexpr int kSortTile = kBlock * kSortItems;            // 2048
constexpr int kSortPasses = 16;                           // 32-bit counts, 2 bits a pass

__global__ __launch_bounds__(kBlock) void hotness_add_kernel(const int32_t* __restrict__ ids, Count n_in, int64_t n_nodes,
                                                             int32_t* counts, int32_t* err) {
    const int64_t n = n_in.get();
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; j < n;
         j += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int32_t id = ids[j];
        if (id < 0 || static_cast<int64_t>(id) >= n_nodes) raise(err, kErrData);
        else atomicAdd(counts + id, 1);
    }
}

// hist[pass][digit] = how many counts have that digit in that pass (zeroed before the launch)
__global__ __launch_bounds__(kBlock) void digit_histogram_kernel(const int32_t* __restrict__ counts, int64_t n,
                                                                 unsigned long long* hist) {
    __shared__ unsigned int s_hist[kSortPasses * 4];
    for (int k = threadIdx.x; k < kSortPasses * 4; k += kBlock) s_hist[k] = 0;
    __syncthreads();
    unsigned int mine[kSortPasses * 4];
#pragma unroll
    for (int k = 0; k < kSortPasses * 4; ++k) mine[k] = 0;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * kBlock) {
        const uint32_t key = static_cast<uint32_t>(counts[i]);
#pragma unroll
        for (int p = 0; p < kSortPasses; ++p) {
            const uint32_t d = (key >> (2 * p)) & 3u;
#pragma unroll
            for (int q = 0; q < 4; ++q) mine[p * 4 + q] += d == static_cast<uint32_t>(q) ? 1u : 0u;
        }
    }
#pragma unroll
    for (int k = 0; k < kSortPasses * 4; ++k) {
        const unsigned int w = wave_sum(mine[k]);
        if (lane_id() == 0 && w) atomicAdd(s_hist + k, w);
    }
    __syncthreads();
    for (int k = threadIdx.x; k < kSortPasses * 4; k += kBlock)
        if (s_hist[k]) atomicAdd(hist + k, static_cast<unsigned long long>(s_hist[k]));
}

struct SplitArgs {
    const int32_t* keys_in;
    const int32_t* vals_in;      // nullable: the values are the positions 0 .. n-1 (the first pass)
    int32_t* keys_out;
    int32_t* vals_out;
    int64_t n;
    int shift;
    const unsigned long long* hist;   // this pass's four digit counts
    ScanState scan;
    int32_t* err;
};

// One pass: a stable partition by the two bits at `shift`, digit 3 first.
__global__ __launch_bounds__(kBlock) void radix_split_kernel(SplitArgs a) {
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[3], s_excl[3];
    __shared__ ScanLookbackLds<3> s_look;
    const int64_t n_tiles = (a.n + kSortTile - 1) / kSortTile;
    if (static_cast<int64_t>(blockIdx.x) >= n_tiles) return;
    const uint32_t tile = scan_take_ticket(a.scan, static_cast<uint32_t>(n_tiles), &s_ticket);
    const int64_t j0 = static_cast<int64_t>(tile) * kSortTile + static_cast<int64_t>(threadIdx.x) * kSortItems;
    int32_t key[kSortItems], val[kSortItems];
    uint32_t cls[kSortItems];            // 0: digit 3, 1: digit 2, 2: digit 1, 3: digit 0; 4: no pair here
    uint32_t c[3] = {0, 0, 0};
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        cls[k] = 4;
        if (j0 + k < a.n) {
            key[k] = a.keys_in[j0 + k];
            val[k] = a.vals_in ? a.vals_in[j0 + k] : static_cast<int32_t>(j0 + k);
            cls[k] = 3u - ((static_cast<uint32_t>(key[k]) >> a.shift) & 3u);
            if (cls[k] < 3) c[cls[k]] += 1;
        }
    }
    // ranks inside the workgroup: classes 0 and 1 share one scan (16 bits each, a tile has 2048 pairs)
    uint32_t tot01, tot2;
    const uint32_t before01 = block_exclusive_scan(c[0] | (c[1] << 16), s_wave, tot01);
    const uint32_t before2 = block_exclusive_scan(c[2], s_wave, tot2);
    if (threadIdx.x == 0) {
        s_agg[0] = tot01 & 0xffffu;
        s_agg[1] = tot01 >> 16;
        s_agg[2] = tot2;
    }
    scan_chained_prefix<3>(a.scan, tile, s_agg, s_excl, &s_look, a.err);
    // where each class begins in the output, and how many pairs of it lie before this thread's
    const int64_t base[4] = {0, static_cast<int64_t>(a.hist[3]), static_cast<int64_t>(a.hist[3] + a.hist[2]),
                             static_cast<int64_t>(a.hist[3] + a.hist[2] + a.hist[1])};
    int64_t at[4];
    at[0] = static_cast<int64_t>(s_excl[0]) + (before01 & 0xffffu);
    at[1] = static_cast<int64_t>(s_excl[1]) + (before01 >> 16);
    at[2] = static_cast<int64_t>(s_excl[2]) + before2;
    // pairs before this thread's first = j0; those not in classes 0..2 are in class 3
    at[3] = j0 - at[0] - at[1] - at[2];
#pragma unroll
    for (int k = 0; k < kSortItems; ++k) {
        if (cls[k] > 3) continue;
        int64_t w = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (cls[k] == static_cast<uint32_t>(q)) w = base[q] + at[q]++;
        if (w >= 0 && w < a.n) {                     // always, unless the counts changed between the two kernels
            a.keys_out[w] = key[k];
            a.vals_out[w] = val[k];
        } else {
            raise(a.err, kErrInternal);
        }
    }
}

unsigned grid_for(int64_t n, unsigned cap_blocks) {
    int64_t b = (n + kBlock - 1) / kBlock;
    if (b < 1) b = 1;
    if (b > cap_blocks) b = cap_blocks;
    return static_cast<unsigned>(b);
}

}  // namespace

hipError_t launch_hotness_add(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                              int32_t* counts, int32_t* err) {
    hipLaunchKernelGGL(hotness_add_kernel, dim3(grid_for(n_max, 4096)), dim3(kBlock), 0, stream, ids, n, n_nodes, counts, err);
    return hipGetLastError();
}

size_t hotness_order_scratch_bytes(int64_t n_nodes) {
    const size_t tiles = static_cast<size_t>((n_nodes + kSortTile - 1) / kSortTile) + 2;
    const size_t status = (sizeof(unsigned long long) * 3 * tiles + 255) / 256 * 256;
    const size_t ints = (sizeof(int32_t) * static_cast<size_t>(n_nodes) + 255) / 256 * 256;
    return 512 /* digit counts */ + 256 /* ticket */ + status + 3 * ints;
}

hipError_t launch_hotness_order(hipStream_t stream, const int32_t* counts, int64_t n_nodes, int32_t* order, void* scratch,
                                int32_t* err) {
    unsigned char* p = static_cast<unsigned char*>(scratch);
    const size_t tiles = static_cast<size_t>((n_nodes + kSortTile - 1) / kSortTile) + 2;
    const size_t status_bytes = (sizeof(unsigned long long) * 3 * tiles + 255) / 256 * 256;
    const size_t ints = (sizeof(int32_t) * static_cast<size_t>(n_nodes) + 255) / 256 * 256;
    unsigned long long* hist = reinterpret_cast<unsigned long long*>(p);
    uint32_t* ticket = reinterpret_cast<uint32_t*>(p + 512);
    unsigned long long* status = reinterpret_cast<unsigned long long*>(p + 768);
    int32_t* keys1 = reinterpret_cast<int32_t*>(p + 768 + status_bytes);
    int32_t* vals1 = reinterpret_cast<int32_t*>(p + 768 + status_bytes + ints);
    int32_t* keys2 = reinterpret_cast<int32_t*>(p + 768 + status_bytes + 2 * ints);
    // digit counts, ticket and scan status start from zero (this call is not part of any recorded batch)
    hipError_t e = hipMemsetAsync(p, 0, 768 + status_bytes, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(digit_histogram_kernel, dim3(grid_for(n_nodes, 2048)), dim3(kBlock), 0, stream, counts, n_nodes, hist);
    const unsigned n_tiles = static_cast<unsigned>((n_nodes + kSortTile - 1) / kSortTile);
    for (int pass = 0; pass < kSortPasses; ++pass) {
        SplitArgs a{};
        a.keys_in = pass == 0 ? counts : (pass % 2 == 1 ? keys1 : keys2);
        a.vals_in = pass == 0 ? nullptr : (pass % 2 == 1 ? vals1 : order);
        a.keys_out = pass % 2 == 0 ? keys1 : keys2;
        a.vals_out = pass % 2 == 0 ? vals1 : order;            // the last pass (odd) leaves the values in `order`
        a.n = n_nodes;
        a.shift = 2 * pass;
        a.hist = hist + 4 * pass;
        a.scan = ScanState{status, ticket, static_cast<uint32_t>(tiles), static_cast<uint32_t>(pass + 1), nullptr};
        a.err = err;
        hipLaunchKernelGGL(radix_split_kernel, dim3(n_tiles < 1 ? 1 : n_tiles), dim3(kBlock), 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace helios
