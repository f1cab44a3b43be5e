// Pre-sampling hotness: per-node counters and the hotness order.
//
// hotness_add: one batch's de-duplicated ID list adds one to each of its nodes'
// counters.  The IDs of a call are distinct, so the atomic adds of one call
// never meet on an address; calls on different streams may.
// hotness_order: nodes sorted by counter, descending, ties by ascending ID: a
// stable descending radix sort of (count, id) pairs whose ids start out
// ascending.  The sort is rocPRIM's device radix sort (a library primitive,
// used once per cache build, not on the per-batch path).
#include "kernels.hpp"

#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>

namespace helios {

namespace {

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

__global__ __launch_bounds__(kBlock) void iota_kernel(int32_t* v, int64_t n) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * kBlock)
        v[i] = static_cast<int32_t>(i);
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

size_t hotness_order_temp_bytes(int64_t n_nodes) {
    size_t bytes = 0;
    int32_t* nul = nullptr;
    (void)rocprim::radix_sort_pairs_desc(nullptr, bytes, nul, nul, nul, nul, static_cast<size_t>(n_nodes), 0, 32, nullptr);
    return bytes;
}

hipError_t launch_hotness_order(hipStream_t stream, const int32_t* counts, int64_t n_nodes, int32_t* ids_in,
                                int32_t* counts_sorted, int32_t* order, void* temp, size_t temp_bytes) {
    hipLaunchKernelGGL(iota_kernel, dim3(grid_for(n_nodes, 8192)), dim3(kBlock), 0, stream, ids_in, n_nodes);
    return rocprim::radix_sort_pairs_desc(temp, temp_bytes, counts, counts_sorted, ids_in, order,
                                          static_cast<size_t>(n_nodes), 0, 32, stream);
}

}  // namespace helios
