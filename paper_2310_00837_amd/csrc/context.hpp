// The context behind the C ABI and the helpers every file of the host runtime uses.
#pragma once
#include "../../include/helios.h"
#include "kernels.hpp"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

namespace helios {

// device counters (int64 each)
constexpr int kCntFrontier = 0;     // [HELIOS_MAX_HOPS + 1] frontier sizes
constexpr int kCntFlat = 16;        // [HELIOS_MAX_HOPS] sample-list sizes
constexpr int kCntCat = 32;         // length of [seeds | flat_0 | ...] compacted so far
constexpr int kCntUnique = 33;
constexpr int kCntHopTotal = 34;    // input length of a de-duplication between two hops (a copy of its flat size)
constexpr int kCntTier = 40;        // [3] list entries to copy from the HBM tier and the host tier, misses to serve
constexpr int kCntStage = 64;       // [HELIOS_MAX_HOPS][kStageWords] totals after every stage of a batch's compaction
constexpr int kNumCounters = kCntStage + HELIOS_MAX_HOPS * kStageWords;
constexpr uint32_t kVarsRing = 256;   // batch launches that may be queued on a context without a helios_sync

// rows of the scan status buffer: the two compactions that share a launch scan at the same time
constexpr int kScanRowsHop = 0;     // 2 rows: hop compaction, count pass
constexpr int kScanRowsLook = 2;    // 3 rows: batch compaction with lookup, stand-alone lookup, stand-alone de-duplication
constexpr int kScanRows = 5;

// A launch of the batch pipeline that has been prepared but not issued: the launches of the members of a
// gang are collected first and then issued together, step by step (see helios_gang_create).
enum StepKind { kStepSample = 0, kStepCompact = 1, kStepFinish = 2 };
struct PendingStep {
    StepKind kind;
    SampleJob sample;
    CompactJob compact;
    FinishJob finish;
};

// one timed role of the last batch (see helios_batch_ticks)
struct StampRole {
    int32_t kind, stage;
    uint32_t workgroups;
};

}  // namespace helios

struct helios_missq;
struct helios_plan;

struct helios_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    int timing = 0;                            // 0 off, 1 device clock per role, 2 (split copies only) HIP events on the copy kernels
    hipEvent_t t_hbm[2] = {nullptr, nullptr}, t_host[2] = {nullptr, nullptr};
    bool timed_events = false;                 // the last batch recorded the events above
    uint64_t* clock = nullptr;                 // device: workgroup ticks of the timed roles of a batch (allocated when timing is first asked for)
    uint64_t* clock_host = nullptr;            // pinned [kMaxStampRoles][2], written by the publish kernel
    helios::StampRole stamp_roles[helios::kMaxStampRoles];
    helios::StampTable stamp_table{};
    int n_stamps = 0;                          // timed roles of the last batch
    uint32_t stamp_words = 0;                  // words of `clock` taken by them
    double clock_khz = 100000.0;
    unsigned hbm_blocks = 0, host_blocks = 0;  // 0 = the launcher's default
    bool serve_misses = false;                 // the whole-path call also copies the rows of its miss list from the stand-in
    bool split_copies = false;                 // the whole-path call keeps its row copies in kernels of their own (see helios_set_param)
    char errmsg[256] = {0};

    helios::CsrView g{nullptr, nullptr, 0};
    int64_t n_edges = 0;
    bool has_graph = false;
    uint64_t graph_generation = 0;             // bumped by every helios_csr_load

    int32_t* rank = nullptr;
    int64_t rank_cap = 0;
    int64_t n_hbm = 0, n_host = 0;
    int32_t row_bytes = 0;
    const void *hbm_table = nullptr, *host_table = nullptr, *standin_table = nullptr;
    bool has_cache = false;
    uint64_t cache_generation = 0;             // bumped by every helios_cache_build

    int n_children = 0;                        // live plans and miss queues: they point back to the context
    std::vector<helios_plan*> plans;           // live plans (their error words are part of helios_sync)
    helios_missq* missq = nullptr;             // attached miss queue: batches submit their misses by themselves
    int64_t missq_timeout_us = 2000000;        // how long the completion kernel waits without progress
    unsigned missq_waves = 0;                  // 0 = default

    int32_t* err = nullptr;                    // pinned, GPU-mapped int32[2]: the context's device-side error word
    int32_t* err_now = nullptr;                // where kernels being launched report: err, or the word of the plan being recorded
    int64_t* cnt = nullptr;                    // device int64[kNumCounters]
    int64_t* learn = nullptr;                  // pinned int64[4]: {unique, HBM hits, host hits, misses} of the last finished lookup;
                                               // read without waiting, to size the copy grids of the calls that follow

    // scratch, sized for calls of up to cap_ids IDs
    int64_t cap_ids = 0;
    uint32_t table_slots = 0;                  // slots of every hash table below (power of two >= 2 * cap_ids)
    unsigned long long* batch_tables = nullptr;   // kBatchTables tables of the batch de-duplication, one after the other
    int32_t* batch_iof = nullptr;              // kBatchTables x cap_ids: index in `unique` of a first occurrence
    int32_t* batch_slot_of = nullptr;          // cap_ids
    uint32_t batch_dirty[helios::kBatchTables] = {0, 0, 0};   // slots of each batch table that may be non-empty
    uint64_t batch_seq = 0;                    // batches launched so far; batch b uses table b mod kBatchTables
    unsigned long long* hop_table[2] = {nullptr, nullptr};   // de-duplication of one hop's samples, hops alternate
    uint32_t hop_dirty[2] = {0, 0};
    int32_t* hop_slot_of = nullptr;
    int32_t* list_pos[2] = {nullptr, nullptr};
    int32_t* list_slot[2] = {nullptr, nullptr};
    int32_t* cat = nullptr;
    unsigned long long* scan_status = nullptr; // [kScanRows][scan_stride]
    uint32_t scan_stride = 0;
    uint32_t* scan_ticket = nullptr;           // device, two counters 64 bytes apart, zero between launches
    uint32_t epoch = 0;

    // recorded batches (HIP graphs): per-batch values live in device memory (vars), fed from a ring
    // of pinned slots; while recording, scans get epoch offsets 1, 2, ... instead of fresh epochs
    helios::BatchVars* vars = nullptr;         // device
    helios::BatchVars* vars_ring = nullptr;    // pinned [kVarsRing]
    uint32_t* batches_run = nullptr;           // device: recorded batches run so far (selects the ring slot)
    uint32_t vars_next = 0, vars_unsynced = 0;
    uint64_t launch_seq = 0;                   // recorded batches launched so far
    bool recording = false;
    uint32_t rec_scans = 0;
    uint32_t rec_clear_slots = 0;              // slots of the next batch's table that the recording empties
    uint64_t scratch_generation = 0;

    std::vector<helios::PendingStep>* defer = nullptr;   // set while a gang is recorded: where the pipeline's launches go
    int link_share = 1;                        // batches whose host-tier copies share the link in every launch (a gang's members)

    // what the last batch left behind for helios_make_blocks
    bool blocks_ready = false;
    uint32_t last_slots = 0;
    uint32_t last_table = 0;
    int64_t last_n_seeds = 0;
    int32_t last_n_hops = 0;
    int64_t last_frontier_max[HELIOS_MAX_HOPS] = {0};
    int64_t last_flat_max[HELIOS_MAX_HOPS] = {0};

    // scratch of helios_hotness_order, kept between calls
    void* hot_temp = nullptr;
    size_t hot_temp_bytes = 0;
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
