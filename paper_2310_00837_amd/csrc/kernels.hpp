// Host-side launchers of the Helios kernels.
// Every launcher enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include "common.hpp"
#include "compact_dev.hpp"
#include "gather_dev.hpp"
#include "hashtable.hpp"
#include "sample_dev.hpp"
#include "scan.hpp"

namespace helios {

struct CsrView {
    const int64_t* offsets;
    const int32_t* indices;
    int64_t n_nodes;
};

// ---- sample.hip
// Count pass of hop 0 as a kernel of its own, for seed lists too long for the folded count of the
// sampling pass: indptr[i] = start of frontier[i]'s samples in flat, indptr[n] = total (also to
// *n_flat_dev); size_out (nullable, device-accessible) gets {n, total}.  frontier_out (nullable, may
// equal frontier) receives a copy of the frontier; feed.ring (nullable): a recorded batch, whose
// variables this kernel takes from the host's ring (the frontier is their seeds).
hipError_t launch_frontier_count(hipStream_t stream, const CsrView& g, const int32_t* frontier, const BatchFeed& feed,
                                 int32_t* frontier_out, Count n, int64_t n_max, int32_t fanout, int64_t* indptr,
                                 int64_t flat_cap, int64_t* n_flat_dev, int64_t* size_out, const ScanState& scan, int32_t* err);

// ---- pipeline.hip: the launches of the sampling / whole-path pipeline; each carries one or more roles
// Every launch takes the jobs of n mini-batches (1 <= n <= kMaxGang), one per member of a gang; the
// members' roles share the launch.
constexpr int kMaxGang = 4;
// Sampling pass of one hop (see sample_dev.hpp), and beside it, if link_blocks > 0, a row copy from a
// source behind the host link (the cached rows that the stage before has just listed).  The fan-outs
// of all members select the same group width.
struct SampleJob {
    HopArgs hop;
    unsigned hop_blocks;
    GatherArgs link;
    unsigned link_blocks;
};
hipError_t launch_sample(hipStream_t stream, const SampleJob* jobs, int n);
// Compaction pass(es) after a hop: the hop's samples into the next frontier (hop_blocks > 0) and the
// stage of the batch's ID list that the hop has completed, with its cache lookup (look_blocks > 0).
struct CompactJob {
    CompactArgs hop;
    unsigned hop_blocks;
    CompactArgs look;
    unsigned look_blocks;
};
hipError_t launch_compact(hipStream_t stream, const CompactJob* jobs, int n);
// The end of a batch in one launch: host-tier copy of the last stage, the rows of the miss list from the
// storage stand-in (if the batch serves its own misses), HBM-tier copy of all stages, the inverse map,
// and the emptying of the table that the next batch of the context uses.  Any of the five may be absent
// (0 workgroups).  With vars (a recorded batch) the table to empty is the one after the batch's
// own among bt's, whatever clear.table says.  The rows of all members have one size.
struct FinishJob {
    GatherArgs hbm;
    unsigned hbm_blocks;
    GatherArgs link;
    unsigned link_blocks;
    GatherArgs miss;
    unsigned miss_blocks;
    InverseArgs inv;
    unsigned inv_blocks;
    ClearJob clear;
    unsigned clear_blocks;
    BatchTables bt;
    const BatchVars* vars;
};
hipError_t launch_finish(hipStream_t stream, const FinishJob* jobs, int n);
// what the kernels receive: the members' arguments and workgroup ranges side by side
struct SampleMember {
    HopArgs hop;
    GatherArgs link;
    Role r_hop, r_link;
};
struct SampleGang {
    SampleMember m[kMaxGang];
    int n;
};
struct CompactMember {
    CompactArgs hop, look;
    Role r_hop, r_look;
};
struct CompactGang {
    CompactMember m[kMaxGang];
    int n;
};
struct FinishMember {
    GatherArgs hbm, link, miss;
    InverseArgs inv;
    ClearJob clear;
    BatchTables bt;
    const BatchVars* vars;
    Role r_hbm, r_link, r_miss, r_inv, r_clear;
};
struct FinishGang {
    FinishMember m[kMaxGang];
    int n;
};
static_assert(sizeof(SampleGang) <= 4096 && sizeof(CompactGang) <= 4096 && sizeof(FinishGang) <= 4096,
              "kernel arguments are limited to 4 KB");
hipError_t launch_clear(hipStream_t stream, const ClearJob& job);
// reduces the stamps of n_roles roles (role q: workgroups[q] workgroups, stamps at clock + offset[q]) to
// {earliest start, latest end} pairs in pinned host memory
constexpr int kMaxStampRoles = 48;
struct StampTable {
    uint32_t offset[kMaxStampRoles];
    uint32_t workgroups[kMaxStampRoles];
};
hipError_t launch_clock_publish(hipStream_t stream, const uint64_t* clock, const StampTable& table, int n_roles,
                                uint64_t* host_out);

// ---- dedup.hip (the stand-alone de-duplication)
// First pass as a kernel of its own (for IDs that no kernel of this library produced): inserts ids[0, n)
// into s.table, which must be empty.
hipError_t launch_dedup_insert(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                               const DedupScratch& s, int32_t* err);
// Second pass over the whole list, and the optional third pass.
hipError_t launch_dedup_compact_plain(hipStream_t stream, const CompactArgs& a, int64_t n_max);
hipError_t launch_dedup_inverse(hipStream_t stream, const InverseArgs& a, int64_t n_max);

// ---- cache.hip
hipError_t launch_rank_build(hipStream_t stream, const int32_t* order, int64_t n_nodes, int32_t* rank, int32_t* err);

hipError_t launch_lookup_partition(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max,
                                   const int32_t* rank, int64_t n_nodes, int64_t n_hbm, int64_t n_host,
                                   const TierLists& lists, int32_t* miss_pos, int32_t* miss_id,
                                   int32_t* miss_slot, int64_t miss_cap, int64_t* stats_out, int64_t* learn,
                                   const ScanState& scan, int32_t* err);

// ---- gather.hip
// The row copy as a kernel of its own.  far_source selects the launch shape for a source behind the host
// link (few workgroups, one per CU).  With t_start / t_stop (nullable) the launch carries HIP events that
// take the kernel's own begin and end, as a kernel trace reports them.  expected: the probable length of the
// list (0 = unknown; see copy_role_blocks).  *blocks_out = workgroups launched.
hipError_t launch_gather_rows(hipStream_t stream, const GatherArgs& a, int64_t n_max, bool far_source, bool standin,
                              unsigned blocks_limit /* 0 = default */, int64_t expected, hipEvent_t t_start, hipEvent_t t_stop,
                              unsigned* blocks_out);

// ---- blocks.hip
// out[j] = index in a de-duplication's unique list of ids[j] (s = the scratch that de-duplication used,
// untouched since); an ID that is not in the list raises kErrData.
hipError_t launch_local_ids(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, const DedupScratch& s,
                            int32_t* out, int32_t* err);

// ---- hotness.hip
hipError_t launch_hotness_add(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                              int32_t* counts, int32_t* err);
size_t hotness_order_scratch_bytes(int64_t n_nodes);
// order = nodes by counts descending, ties by ascending ID; scratch: hotness_order_scratch_bytes(n_nodes) of device memory
hipError_t launch_hotness_order(hipStream_t stream, const int32_t* counts, int64_t n_nodes, int32_t* order, void* scratch,
                                int32_t* err);

// dst[0, bytes) = src[0, bytes) with the same 16-byte non-temporal accesses as the row copy
hipError_t launch_calibration_copy(hipStream_t stream, const void* src, void* dst, int64_t bytes);

}  // namespace helios
