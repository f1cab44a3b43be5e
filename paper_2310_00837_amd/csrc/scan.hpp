// Single-pass chained prefix sum across workgroups (decoupled look-back).
//
// Each participating workgroup owns one tile, taken in start order from a
// ticket counter.  A tile publishes its aggregate, then looks back over its
// predecessors, 256 at a time, until it meets one that has published a full
// inclusive prefix.  One 64-bit status word per tile and counter holds
// {epoch:30, flag:2, value:32}; the epoch changes on every launch, so a stale
// word reads as "not published" and the buffer never needs clearing between
// launches.
//
// Why tickets: a tile waits only for tiles with a smaller index, and with
// tickets those have all started already, whatever else runs on the GPU.  With
// tile = workgroup index that is not so once several scan kernels from
// different streams oversubscribe the chip: the waiting workgroups of one
// kernel can hold the slots of an XCD on which another kernel's lower tile is
// still to start, and the other way round (seen on this part with six streams:
// the bounded wait below fired).  The price is one device-scope atomic on one
// address per participating workgroup, which serialises at ~20 ns each, so the
// kernels keep the number of tiles low: 1024 items per tile, and only
// workgroups that own a tile take a ticket.
//
// The wait is bounded all the same: after kScanSpinBudget polls a tile gives up,
// records kErrInternal and carries on with a zero, so a launch always drains
// and the caller gets an error instead of a hang.
#pragma once
#include "common.hpp"

namespace helios {

struct ScanState {
    unsigned long long* status;   // [n_counters][stride]
    uint32_t* ticket;             // one counter, zero between launches
    uint32_t stride;              // tiles the status rows have room for
    uint32_t epoch;               // 1 .. 2^30-1, new for every launch
    const BatchVars* vars;        // nullable: if set, vars->epoch_base is added to epoch on the device
};

// the launch's epoch: the argument, plus the batch's base when the launch is part of a recorded batch
__device__ __forceinline__ ScanState scan_resolve(ScanState st) {
    if (st.vars) st.epoch += st.vars->epoch_base;
    return st;
}

constexpr uint32_t kFlagAggregate = 1u;
constexpr uint32_t kFlagPrefix = 2u;

__device__ __forceinline__ unsigned long long scan_pack(uint32_t epoch, uint32_t flag, uint32_t v) {
    return (static_cast<unsigned long long>(epoch) << 34) | (static_cast<unsigned long long>(flag) << 32) | v;
}

__device__ __forceinline__ void scan_store(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long scan_load(unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr uint32_t kScanSpinBudget = 1u << 20;     // polls of one status word before giving up (about a second)

// Tile index of this workgroup: its place in the start order of the n_tiles workgroups that take
// part (the caller lets exactly the workgroups with blockIdx.x < n_tiles call this).  The one that
// draws the last ticket puts the counter back to zero for the next launch: by then every other
// participant has drawn.  Contains barriers; s_ticket is one word of LDS.
__device__ __forceinline__ uint32_t scan_take_ticket(const ScanState& st, uint32_t n_tiles, uint32_t* s_ticket) {
    if (n_tiles == 1) return 0;               // a single tile waits for nobody: no ticket, no atomic
    if (threadIdx.x == 0) {
        const uint32_t t = atomicAdd(st.ticket, 1u);
        if (t == n_tiles - 1) __hip_atomic_store(st.ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_ticket = t;
    }
    __syncthreads();
    const uint32_t t = *s_ticket;
    __syncthreads();
    return t;
}

// LDS the look-back needs: per counter and wave, {prefix seen, partial sum}.
template <int NC>
struct ScanLookbackLds {
    uint32_t seen[NC][kWavesPerBlock];
    uint32_t part[NC][kWavesPerBlock];
};

// Exclusive prefix of this tile's aggregates over all earlier tiles, for NC
// counters at once.  s_agg[c] holds the tile aggregate (written by the caller
// before the call; a barrier comes first here); on return s_excl[c] holds the
// exclusive prefix.  The whole workgroup looks back, 256 predecessors per round
// and all counters in the same round: thread k reads the status words of tile
// (first - k); within a round each wave reduces its 64 words and the waves are
// combined in order, stopping at the nearest predecessor that has published a
// full prefix.  A round costs one device-scope read latency, so the look-back
// of a launch with T tiles takes about T/256 rounds at worst.  Call from
// uniform control flow; tile < st.stride is the caller's duty.
template <int NC>
__device__ __forceinline__ void scan_chained_prefix(const ScanState& st_in, uint32_t tile, const uint32_t* s_agg,
                                                    uint32_t* s_excl, ScanLookbackLds<NC>* lds, int32_t* err) {
    const ScanState st = scan_resolve(st_in);
    __syncthreads();
    if (threadIdx.x < NC) {
        const uint32_t c = threadIdx.x;
        scan_store(st.status + static_cast<size_t>(c) * st.stride + tile,
                   scan_pack(st.epoch, tile == 0 ? kFlagPrefix : kFlagAggregate, s_agg[c]));
        if (tile == 0) s_excl[c] = 0;
    }
    if (tile == 0) {
        __syncthreads();
        return;
    }
    const int lane = lane_id(), wave = wave_id();
    uint32_t excl[NC];
    bool done[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) { excl[c] = 0; done[c] = false; }
    int64_t first = static_cast<int64_t>(tile) - 1;          // nearest predecessor of the round
    while (true) {
        const int64_t idx = first - static_cast<int64_t>(threadIdx.x);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (done[c]) continue;                           // uniform over the workgroup
            uint32_t flag = kFlagPrefix, val = 0;            // positions before tile 0 act as an empty prefix
            if (idx >= 0) {
                unsigned long long* p = st.status + static_cast<size_t>(c) * st.stride + idx;
                unsigned long long w;
                uint32_t budget = kScanSpinBudget;
                do {
                    w = scan_load(p);
                    flag = static_cast<uint32_t>(w >> 32) & 3u;
                    if (static_cast<uint32_t>(w >> 34) != st.epoch) flag = 0;
                    if (flag == 0) __builtin_amdgcn_s_sleep(1);
                } while (flag == 0 && --budget != 0);
                val = static_cast<uint32_t>(w);
                if (flag == 0) {                             // gave up: report, and let the launch drain
                    raise(err, kErrInternal);
                    flag = kFlagPrefix;
                    val = 0;
                }
            }
            const unsigned long long has_prefix = __ballot(flag == kFlagPrefix);
            uint32_t part;
            if (has_prefix) {
                const int stop = __ffsll(static_cast<long long>(has_prefix)) - 1;
                part = wave_sum(lane <= stop ? val : 0u);
            } else {
                part = wave_sum(val);
            }
            if (lane == 0) {
                lds->seen[c][wave] = has_prefix ? 1u : 0u;
                lds->part[c][wave] = part;
            }
        }
        __syncthreads();
        bool all_done = true;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (done[c]) continue;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) {
                if (!done[c]) {
                    excl[c] += lds->part[c][w];
                    if (lds->seen[c][w]) done[c] = true;
                }
            }
            all_done = all_done && done[c];
        }
        __syncthreads();                                     // lds is rewritten in the next round
        if (all_done) break;
        first -= kBlock;
    }
    if (threadIdx.x < NC) {
        const uint32_t c = threadIdx.x;
        uint32_t e = 0;
#pragma unroll
        for (int q = 0; q < NC; ++q) if (q == static_cast<int>(c)) e = excl[q];
        scan_store(st.status + static_cast<size_t>(c) * st.stride + tile, scan_pack(st.epoch, kFlagPrefix, e + s_agg[c]));
        s_excl[c] = e;
    }
    __syncthreads();
}

}  // namespace helios
