// Batch generation: node IDs -> their index in the batch's unique list.
//
// The hash table of the batch's de-duplication still maps every ID of the batch
// to the input position of its first occurrence, and index_of_first maps that
// position to the index in `unique`; so relabelling an ID is one probe of a
// table that sits in L2, with no second table to build.
#include "kernels.hpp"

namespace helios {

namespace {

__global__ __launch_bounds__(kBlock) void local_ids_kernel(const int32_t* __restrict__ ids, Count n_in, DedupScratch s,
                                                           int32_t* out, int32_t* err) {
    const int64_t n = n_in.get();
    const uint32_t mask = s.n_slots - 1;
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; j < n;
         j += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int32_t id = ids[j];
        int32_t local = -1;
        if (id >= 0) {
            uint32_t slot = hash_id(static_cast<uint32_t>(id), mask);
            for (uint32_t probes = 0; probes <= mask; ++probes) {         // the table is at most half full
                const unsigned long long cur = s.table[slot];
                if (cur == ~0ull) break;                                   // not in the batch
                if (static_cast<uint32_t>(cur >> 32) == static_cast<uint32_t>(id)) {
                    local = s.index_of_first[static_cast<uint32_t>(cur)];
                    break;
                }
                slot = (slot + 1) & mask;
            }
        }
        if (local < 0) raise(err, kErrData);
        out[j] = local;
    }
}

}  // namespace

hipError_t launch_local_ids(hipStream_t stream, const int32_t* ids, Count n, int64_t n_max, const DedupScratch& s,
                            int32_t* out, int32_t* err) {
    int64_t b = (n_max + kBlock - 1) / kBlock;
    if (b < 1) b = 1;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL(local_ids_kernel, dim3(static_cast<unsigned>(b)), dim3(kBlock), 0, stream, ids, n, s, out, err);
    return hipGetLastError();
}

}  // namespace helios
