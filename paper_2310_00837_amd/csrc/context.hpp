// The context behind the C ABI and the helpers every file of the host runtime uses.
#pragma once
#include "../../include/helios.h"
#include "kernels.hpp"

#include <cstdarg>
#include <cstdio>
#include <cstring>

namespace helios {

// device counters (int64 each)
constexpr int kCntFrontier = 0;     // [HELIOS_MAX_HOPS + 1] frontier sizes
constexpr int kCntFlat = 16;        // [HELIOS_MAX_HOPS] sample-list sizes
constexpr int kCntCat = 32;         // length of [seeds | flat_0 | ...]
constexpr int kCntUnique = 33;
constexpr int kCntHopTotal = 34;    // input length of a de-duplication between two hops (a copy of its flat size)
constexpr int kCntTier = 40;        // [3] HBM hits, host hits, misses
constexpr int kNumCounters = 64;
constexpr uint32_t kVarsRing = 256;   // batch launches that may be queued on a context without a helios_sync

}  // namespace helios

struct helios_missq;

struct helios_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    hipStream_t aux = nullptr;                 // host-tier row copies run here, beside the HBM-tier ones
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int timing = 0;                            // 0 off, 1 device clock, 2 device clock + HIP events
    hipEvent_t t_hbm[2] = {nullptr, nullptr}, t_host[2] = {nullptr, nullptr};
    bool timed_hbm = false, timed_host = false;
    uint64_t* clock = nullptr;                 // device [2][2 * kGatherMaxBlocks] workgroup ticks per tier copy
    unsigned clock_blocks[2] = {0, 0};
    uint64_t* clock_host = nullptr;            // pinned [2][2], written by the publish kernel
    double clock_khz = 100000.0;
    unsigned hbm_blocks = 0, host_blocks = 0;  // 0 = the launcher's default
    bool serial_tiers = true;                  // the host-tier copy follows the HBM-tier copy (see helios_set_param)
    char errmsg[256] = {0};

    helios::CsrView g{nullptr, nullptr, 0};
    int64_t n_edges = 0;
    bool has_graph = false;

    int32_t* rank = nullptr;
    int64_t rank_cap = 0;
    int64_t n_hbm = 0, n_host = 0;
    int32_t row_bytes = 0;
    const void *hbm_table = nullptr, *host_table = nullptr, *standin_table = nullptr;
    bool has_cache = false;
    uint64_t cache_generation = 0;             // bumped by every helios_cache_build

    int n_children = 0;                        // live plans and miss queues: they point back to the context
    helios_missq* missq = nullptr;             // attached miss queue: batches submit their misses by themselves
    int64_t missq_timeout_us = 2000000;        // how long the completion kernel waits without progress
    unsigned missq_waves = 0;                  // 0 = default

    int32_t* err = nullptr;                    // pinned, GPU-mapped int32[2]
    int64_t* cnt = nullptr;                    // device int64[kNumCounters]

    int64_t cap_ids = 0;                       // IDs per call the scratch below has room for
    helios::DedupScratch dd{nullptr, 0, nullptr, nullptr};   // de-duplication of a batch's ID list, and helios_dedup
    unsigned long long* hop_table[2] = {nullptr, nullptr};   // de-duplication of one hop's samples, hops alternate
    int32_t* hop_slot_of = nullptr;
    int32_t* list_pos[2] = {nullptr, nullptr};
    int32_t* list_slot[2] = {nullptr, nullptr};
    int32_t* cat = nullptr;
    unsigned long long* scan_status = nullptr;
    uint32_t scan_stride = 0;
    uint32_t* scan_ticket = nullptr;           // device, zero between launches
    uint32_t epoch = 0;

    // recorded batches (HIP graphs): per-batch values live in device memory (vars), fed from a ring
    // of pinned slots; while recording, scans get epoch offsets 1, 2, ... instead of fresh epochs
    helios::BatchVars* vars = nullptr;                 // device
    helios::BatchVars* vars_ring = nullptr;            // pinned [kVarsRing]
    uint32_t* batches_run = nullptr;           // device: recorded batches run so far (selects the ring slot)
    uint32_t vars_next = 0, vars_unsynced = 0;
    uint64_t launch_seq = 0;                   // recorded batches launched so far
    bool recording = false;
    uint32_t rec_scans = 0;
    uint64_t scratch_generation = 0;

    // what the last helios_prepare_batch left behind for helios_make_blocks
    bool blocks_ready = false;
    uint32_t last_slots = 0;
    int64_t last_n_seeds = 0;
    int32_t last_n_hops = 0;
    int64_t last_frontier_max[HELIOS_MAX_HOPS] = {0};
    int64_t last_flat_max[HELIOS_MAX_HOPS] = {0};
};

namespace helios {

inline int fail(helios_ctx* c, int code, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->errmsg, sizeof(c->errmsg), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define HIP_TRY(c, expr)                                                                       \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) return fail((c), HELIOS_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// keeps the caller's current device
struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && (prev == dev || hipSetDevice(dev) == hipSuccess)) ok = true;
        want = dev;
    }
    ~DeviceGuard() {
        if (ok && prev != want) (void)hipSetDevice(prev);
    }
    int want;
};

}  // namespace helios
