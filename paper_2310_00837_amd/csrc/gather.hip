// The row copy (gather_dev.hpp) as a kernel of its own: helios_gather, helios_gather_miss,
// helios_cache_fill, and the whole-path call when it keeps its copies apart for measurement.  The
// rows are 256 B - 2 KB, at random places of a table of tens of GB, so the kernel is bound by memory
// bandwidth (HBM for the GPU tier, the host link for the pinned-host tier and the storage stand-in).
// For an HBM source the grid is up to 8192 workgroups, four times what the chip holds at once, so
// the dispatcher balances the load; a far (host-link) source is limited per CU by the requests a CU
// keeps in flight, not by waves, so it takes one workgroup on each of 32-128 CUs, which fills the
// link and leaves the other CUs alone.
#include "kernels.hpp"

#include <hip/hip_ext.h>

namespace helios {

namespace {

// SRC only names the source in kernel traces: 0 = HBM tier (or any device table), 1 = host tier, 2 = storage stand-in
template <int L, int CPL, int R, int SRC>
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(GatherArgs a) {
    if constexpr (L == 0) copy_rows_long(a, blockIdx.x, gridDim.x);
    else copy_rows<L == 0 ? 64 : L, CPL == 0 ? 1 : CPL, R == 0 ? 1 : R>(a, blockIdx.x, gridDim.x);
}

// plain streaming copy of known size: the yardstick for hardware counters and for the
// bandwidth a copy can reach on this part
__global__ __launch_bounds__(kBlock) void calibration_copy_kernel(const chunk16* __restrict__ src, chunk16* __restrict__ dst,
                                                                  int64_t n_chunks) {
    const int64_t step = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n_chunks; i += step)
        store16(dst + i, load16(src + i));
}

template <int L, int CPL, int R, int SRC>
void launch_one(hipStream_t stream, const GatherArgs& a, unsigned blocks, hipEvent_t t_start, hipEvent_t t_stop) {
    if (t_start && t_stop)
        hipExtLaunchKernelGGL((gather_rows_kernel<L, CPL, R, SRC>), dim3(blocks), dim3(kBlock), 0, stream, t_start, t_stop, 0, a);
    else
        hipLaunchKernelGGL((gather_rows_kernel<L, CPL, R, SRC>), dim3(blocks), dim3(kBlock), 0, stream, a);
}

}  // namespace

hipError_t launch_calibration_copy(hipStream_t stream, const void* src, void* dst, int64_t bytes) {
    // one 16-byte piece per thread where the grid allows it: a plain copy, too, is quickest as many short-lived
    // workgroups that sweep the buffer once (measured: 6.1 against 5.5 TB/s for a grid of a few thousand)
    int64_t blocks = (bytes / 16 + kBlock - 1) / kBlock;
    blocks = blocks < 1 ? 1 : blocks > (1 << 18) ? (1 << 18) : blocks;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream,
                       static_cast<const chunk16*>(src), static_cast<chunk16*>(dst), bytes / 16);
    return hipGetLastError();
}

hipError_t launch_gather_rows(hipStream_t stream, const GatherArgs& a, int64_t n_max, bool far_source, bool standin,
                              unsigned blocks_limit, int64_t expected, hipEvent_t t_start, hipEvent_t t_stop, unsigned* blocks_out) {
    const unsigned nb = copy_role_blocks(a.chunks, far_source, n_max, blocks_limit, expected);
#define HELIOS_CALL_(L, CPL, R)                                                          \
    do {                                                                                 \
        if (!far_source) launch_one<L, CPL, R, 0>(stream, a, nb, t_start, t_stop);       \
        else if (!standin) launch_one<L, CPL, R, 1>(stream, a, nb, t_start, t_stop);     \
        else launch_one<L, CPL, R, 2>(stream, a, nb, t_start, t_stop);                   \
    } while (0)
    HELIOS_COPY_SHAPE_SWITCH(a.chunks, far_source, HELIOS_CALL_);
#undef HELIOS_CALL_
    if (blocks_out) *blocks_out = nb;
    return hipGetLastError();
}

}  // namespace helios
