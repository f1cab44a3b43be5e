// Row copy: out[pos[k], :] = table[slot[k], :].
//
// The rows are 256 B - 2 KB, at random places of a table of tens of GB, so the
// kernel is bound by memory bandwidth (HBM for the GPU tier, the host link for
// the pinned-host tier and the storage stand-in).  A group of L lanes owns one
// row and moves it as 16-byte pieces, so a row is read and written as whole
// contiguous lines; L is the smallest power of two that covers the row (at most
// a wave).  Each group takes R list entries per step (R = 1 or 2: measured
// best; the 32 waves a CU holds supply the requests in flight) and issues all
// their loads before the first store.  The groups of the grid share the list
// evenly (entry k belongs to group k mod groups) and the
// count is read on the device, so no host round trip sits between the lookup
// and the copy.  For an HBM source the grid is up to 8192 workgroups, four
// times what the chip holds at once, so the dispatcher balances the load; a
// far (host-link) source is limited per CU by the requests a CU keeps in
// flight, not by waves, so it takes one workgroup on each of 32-128 CUs, which
// fills the link and leaves the other CUs alone.  Source and destination are
// touched once: non-temporal accesses keep them from displacing the graph and
// the cache map in L2.
#include "kernels.hpp"

namespace helios {

namespace {

typedef uint32_t chunk16 __attribute__((ext_vector_type(4)));   // one 16-byte piece of a row

struct GatherArgs {
    const chunk16* table;
    const int32_t* pos;     // nullable: identity
    const int32_t* slot;
    Count n;
    int32_t chunks;         // 16-byte pieces per row
    chunk16* out;
    unsigned long long* clock;   // nullable: [2 * gridDim.x] first and last tick of every workgroup
};

// Optional timing: every workgroup stores its first and last tick of the
// constant-rate device clock (clock[b], clock[gridDim.x + b]; plain stores, no
// contention); clock_publish_kernel reduces them to {earliest start, latest
// end} in pinned host memory.  Latest end minus earliest start is the kernel's
// duration.
__device__ __forceinline__ void stamp_start(unsigned long long* clock) {
    if (clock && threadIdx.x == 0) clock[blockIdx.x] = wall_clock64();
}
__device__ __forceinline__ void stamp_end(unsigned long long* clock) {
    if (clock) {
        __syncthreads();
        if (threadIdx.x == 0) clock[gridDim.x + blockIdx.x] = wall_clock64();
    }
}

constexpr int kPublishThreads = 1024;

__global__ __launch_bounds__(kPublishThreads) void clock_publish_kernel(const unsigned long long* clock, unsigned n_blocks,
                                                                        unsigned long long* host_out) {
    __shared__ unsigned long long s_lo[kPublishThreads / kWave], s_hi[kPublishThreads / kWave];
    unsigned long long lo = ~0ull, hi = 0ull;
#pragma unroll 8
    for (unsigned b = threadIdx.x; b < n_blocks; b += kPublishThreads) {      // independent loads, issued together
        const unsigned long long a = clock[b], z = clock[n_blocks + b];
        lo = a < lo ? a : lo;
        hi = z > hi ? z : hi;
    }
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) {
        const unsigned long long lo2 = __shfl_xor(lo, d, kWave), hi2 = __shfl_xor(hi, d, kWave);
        lo = lo2 < lo ? lo2 : lo;
        hi = hi2 > hi ? hi2 : hi;
    }
    if ((threadIdx.x & (kWave - 1)) == 0) {
        s_lo[threadIdx.x / kWave] = lo;
        s_hi[threadIdx.x / kWave] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kPublishThreads / kWave; ++w) {
            lo = s_lo[w] < lo ? s_lo[w] : lo;
            hi = s_hi[w] > hi ? s_hi[w] : hi;
        }
        host_out[0] = lo;
        host_out[1] = hi;
    }
}

__device__ __forceinline__ chunk16 load16(const chunk16* p) {
    return __builtin_nontemporal_load(p);
}
__device__ __forceinline__ void store16(chunk16* p, const chunk16& v) {
    __builtin_nontemporal_store(v, p);
}

// L lanes per row, CPL pieces per lane (L * CPL >= chunks), R rows per step.
template <int L, int CPL, int R>
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(GatherArgs a) {
    constexpr int kGroups = kBlock / L;
    stamp_start(a.clock);
    const int l = threadIdx.x % L;
    const int g = threadIdx.x / L;
    // Group j of the grid takes the list entries j, j + groups, j + 2 * groups, ..., R of them per step: every
    // group gets the same number of rows to within one, so all workgroups (for a far source: all the CUs
    // whose requests fill the link) stay busy until the list ends.
    const int64_t groups = static_cast<int64_t>(gridDim.x) * kGroups;
    const int64_t n = a.n.get();
    for (int64_t k0 = static_cast<int64_t>(blockIdx.x) * kGroups + g; k0 < n; k0 += groups * R) {
        chunk16 v[R][CPL];
        int64_t dst[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t k = k0 + r * groups;
            dst[r] = -1;
            if (k < n) {
                const int64_t s = a.slot[k];
                dst[r] = a.pos ? static_cast<int64_t>(a.pos[k]) : k;
                const chunk16* src = a.table + s * a.chunks;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int idx = l + c * L;
                    if (idx < a.chunks) v[r][c] = load16(src + idx);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (dst[r] >= 0) {
                chunk16* o = a.out + dst[r] * a.chunks;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int idx = l + c * L;
                    if (idx < a.chunks) store16(o + idx, v[r][c]);
                }
            }
        }
    }
    stamp_end(a.clock);
}

// any row length: a wave per row, looping over the pieces
__global__ __launch_bounds__(kBlock) void gather_rows_long_kernel(GatherArgs a) {
    stamp_start(a.clock);
    const int64_t n = a.n.get();
    const int l = lane_id();
    const int64_t step = static_cast<int64_t>(gridDim.x) * kWavesPerBlock;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave_id(); k < n; k += step) {
        const int64_t s = a.slot[k];
        const int64_t d = a.pos ? static_cast<int64_t>(a.pos[k]) : k;
        const chunk16* src = a.table + s * a.chunks;
        chunk16* o = a.out + d * a.chunks;
        for (int idx = l; idx < a.chunks; idx += kWave) store16(o + idx, load16(src + idx));
    }
    stamp_end(a.clock);
}

// plain streaming copy of known size: the yardstick for hardware counters and for the
// bandwidth a copy can reach on this part
__global__ __launch_bounds__(kBlock) void calibration_copy_kernel(const chunk16* __restrict__ src, chunk16* __restrict__ dst,
                                                                  int64_t n_chunks) {
    const int64_t step = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n_chunks; i += step)
        store16(dst + i, load16(src + i));
}

template <int L, int CPL, int R>
unsigned launch_shape(hipStream_t stream, const GatherArgs& a, int64_t n_max, unsigned max_blocks) {
    constexpr int kRowsPerBlockStep = (kBlock / L) * R;
    int64_t blocks = (n_max + kRowsPerBlockStep - 1) / kRowsPerBlockStep;
    if (blocks < 1) blocks = 1;
    if (blocks > max_blocks) blocks = max_blocks;
    hipLaunchKernelGGL((gather_rows_kernel<L, CPL, R>), dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream, a);
    return static_cast<unsigned>(blocks);
}

}  // namespace

hipError_t launch_calibration_copy(hipStream_t stream, const void* src, void* dst, int64_t bytes) {
    int64_t blocks = (bytes / 16 + kBlock - 1) / kBlock;
    blocks = blocks < 1 ? 1 : blocks > kGatherMaxBlocks ? kGatherMaxBlocks : blocks;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream,
                       static_cast<const chunk16*>(src), static_cast<chunk16*>(dst), bytes / 16);
    return hipGetLastError();
}

hipError_t launch_clock_publish(hipStream_t stream, const uint64_t* clock, unsigned n_blocks, uint64_t* host_out) {
    hipLaunchKernelGGL(clock_publish_kernel, dim3(1), dim3(kPublishThreads), 0, stream,
                       reinterpret_cast<const unsigned long long*>(clock), n_blocks,
                       reinterpret_cast<unsigned long long*>(host_out));
    return hipGetLastError();
}

hipError_t launch_gather_rows(hipStream_t stream, const void* table, const int32_t* pos, const int32_t* slot,
                              Count n, int64_t n_max, int32_t row_bytes, void* out, bool far_source,
                              uint64_t* clock, unsigned* blocks_out, unsigned blocks_limit) {
    GatherArgs a{static_cast<const chunk16*>(table), pos, slot, n, row_bytes / 16, static_cast<chunk16*>(out),
                 reinterpret_cast<unsigned long long*>(clock)};
    const int c = a.chunks;
    // far source: one workgroup per CU on as many CUs as fill the link (more for short rows)
    // HBM source: 8192 workgroups (four rounds of what the chip holds) balance long lists best; lists that can
    // hold at most a few hundred thousand rows are quicker with the 2048 that are resident at once (measured:
    // 17 k rows 4.4 vs 5.4 us, 35 k rows 8.2 vs 9.1 us; 1 M rows 2 % the other way).
    // (far source, 512 B rows: 64 workgroups copy a list alone 2 % faster than 44, but every kernel launched on
    // the GPU while the link is saturated starts some microseconds late, the later the more link waves are
    // in flight; with three mini-batches in flight 44 workgroups gave 4-6 % more mini-batches per second)
    unsigned max_blocks = far_source ? (c <= 16 ? 128u : c <= 32 ? 44u : 32u) : (n_max >= 500000 ? kGatherMaxBlocks : 2048u);
    if (blocks_limit > 0) max_blocks = blocks_limit < kGatherMaxBlocks ? blocks_limit : kGatherMaxBlocks;
    unsigned nb = 0;
    if (c <= 4) nb = launch_shape<4, 1, 2>(stream, a, n_max, max_blocks);
    else if (c <= 8) nb = launch_shape<8, 1, 2>(stream, a, n_max, max_blocks);
    else if (c <= 16) nb = launch_shape<16, 1, 2>(stream, a, n_max, max_blocks);
    else if (c <= 32 && far_source) nb = launch_shape<32, 1, 4>(stream, a, n_max, max_blocks);
    else if (c <= 32) nb = launch_shape<32, 1, 1>(stream, a, n_max, max_blocks);
    else if (c <= 64) nb = launch_shape<64, 1, 2>(stream, a, n_max, max_blocks);
    else if (c <= 128) nb = launch_shape<64, 2, 2>(stream, a, n_max, max_blocks);
    else if (c <= 256) nb = launch_shape<64, 4, 1>(stream, a, n_max, max_blocks);
    else {
        int64_t blocks = (n_max + kWavesPerBlock - 1) / kWavesPerBlock;
        if (blocks < 1) blocks = 1;
        if (blocks > max_blocks) blocks = max_blocks;
        hipLaunchKernelGGL(gather_rows_long_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream, a);
        nb = static_cast<unsigned>(blocks);
    }
    if (blocks_out) *blocks_out = nb;
    return hipGetLastError();
}

}  // namespace helios
