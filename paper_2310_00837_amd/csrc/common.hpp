// Shared device-side helpers of the Helios HIP kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace helios {

constexpr int kBlock = 256;          // threads per workgroup in every kernel
constexpr int kWave = 64;            // CDNA wavefront
constexpr int kWavesPerBlock = kBlock / kWave;

// device-side error codes, same values as helios_status
constexpr int kErrCapacity = -2;
constexpr int kErrData = -5;
constexpr int kErrInternal = -6;

// A count that is known either on the host (dev == nullptr: the count is
// `host`) or only on the device (read from *dev by the kernel and clamped to
// `host`, the most the buffers behind it can hold).
struct Count {
    const int64_t* dev;
    int64_t host;
    __device__ __forceinline__ int64_t get() const {
        if (!dev) return host;
        const int64_t v = *dev;
        return v < host ? (v < 0 ? 0 : v) : host;
    }
};

// What changes from one mini-batch to the next.  Kernels of a recorded (graph) batch read it
// from device memory, so that one recording serves every batch; directly launched kernels get
// the same values as arguments and a null pointer here.
struct BatchVars {
    uint64_t rng_seed;
    const int32_t* seeds;
    uint32_t epoch_base;     // added to the per-launch epoch of the chained scans
    uint32_t io_round;       // round number of the miss queue the batch submits to (0 if none)
    uint32_t table;          // which of the rotating batch tables this batch uses
    uint32_t reserved;
};

// How a recorded batch gets its BatchVars without a copy being part of the recording: the host writes
// them to the next slot of a ring in pinned memory before every launch; the workgroups of the batch's
// first kernel read the slot that the number of recorded batches run so far on the context selects (a
// device counter, advanced by the batch's second kernel) and the first of them leaves a copy in device
// memory for the kernels after it.
struct BatchFeed {
    const BatchVars* ring;        // pinned host memory, nullable (a directly launched batch)
    uint32_t ring_slots;
    const uint32_t* batches_run;  // device
    BatchVars* vars_out;          // device
};

// First error wins is not needed: any recorded error makes the call fail.
// err points to pinned, GPU-mapped host memory (int32[2]: code, detail).
__device__ __forceinline__ void raise(int32_t* err, int code) {
    *reinterpret_cast<volatile int32_t*>(err) = code;
}

// A role is a range of the workgroups of a launch that does one job; several roles share a launch
// when their jobs are independent and bound by different things (the host link, HBM, latency).
// Workgroup blockIdx.x belongs to the role with first <= blockIdx.x < first + blocks and is its
// workgroup number blockIdx.x - first.
struct Role {
    uint32_t first, blocks;
    __device__ __forceinline__ bool mine() const { return blockIdx.x - first < blocks; }   // unsigned wrap-around
    __device__ __forceinline__ uint32_t rb() const { return blockIdx.x - first; }
};
constexpr unsigned kMaxRoleBlocks = 32768;

// Optional timing of a role: workgroup rb of nrb stores its first and last tick of the constant-rate
// device clock at clock[rb] and clock[nrb + rb] (plain stores, no contention); a publish kernel
// reduces them to {earliest start, latest end} in pinned host memory.
struct Stamps {
    unsigned long long* clock;     // nullable
};
__device__ __forceinline__ void stamp_start(const Stamps& s, uint32_t rb) {
    if (s.clock && threadIdx.x == 0) s.clock[rb] = wall_clock64();
}
__device__ __forceinline__ void stamp_end(const Stamps& s, uint32_t rb, uint32_t nrb) {
    if (s.clock) {
        __syncthreads();
        if (threadIdx.x == 0) s.clock[nrb + rb] = wall_clock64();
    }
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// inclusive scan over the 64 lanes of a wave
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        uint32_t t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread over the block; `total` is the block
// sum (valid in every thread).  `s_wave` is kWavesPerBlock+1 words of LDS.
// Contains block barriers: call from uniform control flow.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* s_wave, uint32_t& total) {
    uint32_t inc = wave_inclusive_scan(v);
    if (lane_id() == kWave - 1) s_wave[wave_id()] = inc;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        uint32_t t = s_wave[w];
        if (w < wave_id()) base += t;
        sum += t;
    }
    total = sum;
    __syncthreads();            // s_wave may be reused by the caller
    return base + inc - v;
}

// Scan kernels give every thread kItemsPerThread consecutive items, so a tile is 1024 items and a
// launch has few tiles (each tile costs a ticket, see scan.hpp).
constexpr int kItemsPerThread = 4;
constexpr int kTileItems = kBlock * kItemsPerThread;

// min(deg(v), fanout): how many samples node v yields at a hop.  A value that is no node ID, or a
// row of 2^31 entries or more, is reported and yields nothing.
__device__ __forceinline__ uint32_t sample_count(const int64_t* offsets, int64_t n_nodes, int32_t v, int32_t fanout,
                                                 int32_t* err) {
    if (v < 0 || static_cast<int64_t>(v) >= n_nodes) {
        raise(err, kErrData);
        return 0;
    }
    const int64_t d = offsets[v + 1] - offsets[v];
    if (d < 0 || d > 0x7fffffffLL) {
        raise(err, kErrData);
        return 0;
    }
    const int64_t f = fanout > 0 ? fanout : 0;
    return static_cast<uint32_t>(d < f ? d : f);
}

}  // namespace helios
