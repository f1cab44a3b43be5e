// Host-side launchers of the Helios kernels (one per step of the path).
// Every launcher enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include "common.hpp"
#include "hashtable.hpp"
#include "scan.hpp"
#define HELIOS_KERNELS_MAX_SEG 9

namespace helios {

struct CsrView {
    const int64_t* offsets;
    const int32_t* indices;
    int64_t n_nodes;
};

// ---- sample.hip
// Count pass of hop 0: indptr[i] = start of frontier[i]'s samples in flat, indptr[n] = total
// (also to *n_flat_dev); size_out (nullable, device-accessible) gets {n, total}.  frontier_out
// (nullable, may equal frontier) receives a copy of the frontier; feed.ring (nullable): a recorded
// batch, whose variables this kernel takes from the host's ring (the frontier is their seeds).  The later hops get their indptr from launch_dedup_compact.  clear_a / clear_b: tables
// set to all ones on the way (those the sampling pass of hop 0 inserts into).
hipError_t launch_frontier_count(hipStream_t stream, const CsrView& g, const int32_t* frontier, const BatchFeed& feed,
                                 int32_t* frontier_out, Count n, int64_t n_max, int32_t fanout, int64_t* indptr,
                                 int64_t flat_cap, int64_t* n_flat_dev, int64_t* size_out, ClearJob clear_a, ClearJob clear_b,
                                 const ScanState& scan, int32_t* err);
// Sampling pass: flat[indptr[i] + k] = k-th sample of frontier[i].  vars (nullable) overrides
// rng_seed.  Every sample is also inserted into hop_table (position = its place in flat) and into
// batch_table (position = its place in [seeds | flat_0 | ...], which cat_out receives; with hop == 0
// the frontier itself is inserted as the seeds; prev_flat = sizes of flat_0 .. flat_{hop-1}); either
// table may be absent.  clear: a table set to all ones on the way (one that a later kernel fills).
hipError_t launch_sample_hop(hipStream_t stream, const CsrView& g, const int32_t* frontier, const int64_t* indptr,
                             Count n_frontier, int64_t n_frontier_max, int32_t fanout, int32_t hop, uint64_t rng_seed,
                             const BatchVars* vars, int32_t* flat, int64_t flat_cap, ClearJob clear, InsertInto hop_table,
                             InsertInto batch_table, int32_t* cat_out, int64_t n_seeds, const Count* prev_flat,
                             uint32_t* batches_run /* nullable: hop 0 of a recorded batch advances it */, int32_t* err);

// ---- dedup.hip
struct DedupScratch {
    unsigned long long* table;   // n_slots entries {id:32, first position:32}; all ones = empty
    uint32_t n_slots;            // power of two
    int32_t* slot_of;            // [n] table slot of every input position
    int32_t* index_of_first;     // [n] index in `unique` of a first occurrence
};
// The lengths of up to HELIOS_KERNELS_MAX_SEG segments whose concatenation is de-duplicated (each may be
// known only on the device).
struct SegLens {
    Count len[HELIOS_KERNELS_MAX_SEG];
    int n_seg;
};
// What the de-duplication between two hops also computes for the hop that follows: the sample
// counts min(deg, fanout) of the new frontier, scanned into indptr (indptr[n_unique] = total, also
// to *n_flat_dev); size_out (nullable, device-accessible) gets {n_unique, total}.
struct NextHopCount {
    const int64_t* offsets;
    int64_t n_nodes;
    int32_t fanout;
    int64_t* indptr;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;
};
struct TierLists {
    int32_t* pos[2];    // positions in the ID list, per cached tier (0 = HBM, 1 = host)
    int32_t* slot[2];   // row in the tier table
    int64_t* count;     // device int64[3]: tier 0, tier 1, misses
};
// What the batch's final de-duplication also computes: the cache lookup of the unique IDs (see
// launch_lookup_partition, whose outputs these are, with positions = indices into `unique`).
struct LookupOut {
    const int32_t* rank;
    int64_t n_hbm, n_host;
    TierLists lists;
    int32_t *miss_pos, *miss_id, *miss_slot;
    int64_t miss_cap;
    int64_t* stats_out;          // device-accessible int64[4], nullable
};
// First pass of a de-duplication as a kernel of its own (for IDs that no kernel of this library
// produced): clears s.table unless table_is_clear, then inserts ids[0, n).
hipError_t launch_dedup_insert(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                               const DedupScratch& s, bool table_is_clear, int32_t* err);
// Second pass: the IDs ids[0, n), n = the sum of lens (n_max bounds it; *n_total_dev receives it), have
// been inserted into s.table with their positions and s.slot_of is filled.  unique = the first
// occurrences in input order (*n_unique_dev, *n_unique_out (nullable) = their number),
// s.index_of_first[j] = index in unique of a first occurrence j.
hipError_t launch_dedup_compact(hipStream_t stream, const int32_t* ids, const SegLens& lens, int64_t n_max,
                                int64_t* n_total_dev, const DedupScratch& s, int32_t* unique, int64_t unique_cap,
                                int64_t* n_unique_dev, int64_t* n_unique_out, const NextHopCount* next /* nullable */,
                                const LookupOut* look /* nullable; not together with next */, const ScanState& scan,
                                int32_t* err);
// Third pass (optional): inverse[j] = index in unique of ids[j], for j < *n_total_dev.
hipError_t launch_dedup_inverse(hipStream_t stream, const int64_t* n_total_dev, int64_t n_max, const DedupScratch& s,
                                int32_t* inverse);

// ---- cache.hip
hipError_t launch_rank_build(hipStream_t stream, const int32_t* order, int64_t n_nodes, int32_t* rank, int32_t* err);

hipError_t launch_lookup_partition(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max,
                                   const int32_t* rank, int64_t n_nodes, int64_t n_hbm, int64_t n_host,
                                   const TierLists& lists, int32_t* miss_pos, int32_t* miss_id,
                                   int32_t* miss_slot, int64_t miss_cap, int64_t* stats_out,
                                   const ScanState& scan, int32_t* err);

// ---- gather.hip
// out[pos[k], :] = table[slot[k], :] for k < n; pos == nullptr means pos[k] = k.
// far_source selects the launch shape for a source behind the host link (few workgroups, one per CU).
// clock (nullable): device uint64[2 * kGatherMaxBlocks]; workgroup b stores its first and last tick of
// the constant-rate device clock at [b] and [blocks + b]; *blocks_out = workgroups launched.
// launch_clock_publish reduces them to {earliest start, latest end} in pinned host memory.
constexpr unsigned kGatherMaxBlocks = 8192;
hipError_t launch_gather_rows(hipStream_t stream, const void* table, const int32_t* pos, const int32_t* slot,
                              Count n, int64_t n_max, int32_t row_bytes, void* out, bool far_source,
                              uint64_t* clock, unsigned* blocks_out, unsigned blocks_limit /* 0 = default */);
hipError_t launch_clock_publish(hipStream_t stream, const uint64_t* clock, unsigned n_blocks, uint64_t* host_out);

// ---- blocks.hip
// out[j] = index in the last de-duplication's unique list of ids[j] (s = the scratch that
// de-duplication used, untouched since); an ID that is not in the list raises kErrData.
hipError_t launch_local_ids(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, const DedupScratch& s,
                            int32_t* out, int32_t* err);

// ---- hotness.hip
hipError_t launch_hotness_add(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                              int32_t* counts, int32_t* err);
size_t hotness_order_temp_bytes(int64_t n_nodes);
// order = nodes by counts descending, ties by ascending ID; ids_in / counts_sorted: int32[n_nodes] scratch
hipError_t launch_hotness_order(hipStream_t stream, const int32_t* counts, int64_t n_nodes, int32_t* ids_in,
                                int32_t* counts_sorted, int32_t* order, void* temp, size_t temp_bytes);

// dst[0, bytes) = src[0, bytes) with the same 16-byte non-temporal accesses as the row copy
hipError_t launch_calibration_copy(hipStream_t stream, const void* src, void* dst, int64_t bytes);

}  // namespace helios
