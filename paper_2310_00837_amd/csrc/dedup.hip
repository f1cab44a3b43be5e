// Order-preserving de-duplication of an ID list.
//
// unique = the distinct IDs in order of first occurrence.  The order is made
// independent of thread scheduling by keeping, per distinct ID, the smallest
// input position that holds it:
//   1. insert: an open-addressing hash table of 64-bit words {id:32 | pos:32}
//      (hashtable.hpp).  The slot of every input is remembered.  For IDs that
//      the sampling kernel produces, that kernel does the inserting as it writes
//      them (sample_dev.hpp); the insert kernel here serves helios_dedup.
//   2. compact (compact_dev.hpp): input j is a first occurrence iff its slot's
//      position is j; the flags are scanned in-workgroup and chained across
//      workgroups, so the unique list comes out in input order in the same pass.
//   3. inverse (optional): every input looks up the unique index of its ID's
//      first occurrence.
// The table has at least twice as many slots as inputs and is empty before the
// first insert; at the sizes of one mini-batch (at most 32 MB) it stays in L2 /
// MALL.  It is not staged through LDS.  Measured on the power-law workloads
// (dedup_probe.py): 15-21 % of a batch's list entries repeat an earlier entry,
// but only 0.5-4.4 % repeat one within the same 4096 entries (0.1-1.2 % within
// 1024), because the hubs that repeat are spread over the whole list.  A
// per-workgroup LDS table would take that little off the global table, while
// every entry paid an LDS probe and a barrier more.
#include "kernels.hpp"

namespace helios {

namespace {

__global__ __launch_bounds__(kBlock) void dedup_insert_kernel(const int32_t* __restrict__ ids, Count n_in, int64_t n_nodes,
                                                              DedupScratch s, int32_t* err) {
    // The first ID is fetched before the device-side count has arrived (the buffer holds n_in.host
    // entries, so the read is in bounds whatever the count turns out to be).
    const int64_t j0 = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    int32_t early = 0;
    if (j0 < n_in.host) early = ids[j0];
    const int64_t n = n_in.get();
    const uint32_t mask = s.n_slots - 1;
    for (int64_t j = j0; j < n; j += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int32_t id = j == j0 ? early : ids[j];
        if (id < 0 || static_cast<int64_t>(id) >= n_nodes) {
            raise(err, kErrData);
            s.slot_of[j] = -1;
            continue;
        }
        s.slot_of[j] = static_cast<int32_t>(table_insert(s.table, mask, static_cast<uint32_t>(id), static_cast<uint32_t>(j)));
    }
}

__global__ __launch_bounds__(kBlock) void dedup_compact_kernel(CompactArgs a) {
    compact_role<kCompactPlain>(a, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(kBlock) void dedup_inverse_kernel(InverseArgs a) { inverse_role(a, blockIdx.x, gridDim.x); }

unsigned grid_for(int64_t n_max, unsigned cap_blocks) {
    int64_t b = (n_max + kBlock - 1) / kBlock;
    if (b < 1) b = 1;
    if (b > cap_blocks) b = cap_blocks;
    return static_cast<unsigned>(b);
}

}  // namespace

hipError_t launch_dedup_insert(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, int64_t n_nodes,
                               const DedupScratch& s, int32_t* err) {
    hipLaunchKernelGGL(dedup_insert_kernel, dim3(grid_for(n_max, 4096)), dim3(kBlock), 0, stream, ids, n, n_nodes, s, err);
    return hipGetLastError();
}

hipError_t launch_dedup_compact_plain(hipStream_t stream, const CompactArgs& a, int64_t n_max) {
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    if (tiles < 1) tiles = 1;
    hipLaunchKernelGGL(dedup_compact_kernel, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_dedup_inverse(hipStream_t stream, const InverseArgs& a, int64_t n_max) {
    hipLaunchKernelGGL(dedup_inverse_kernel, dim3(grid_for(n_max, 4096)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
