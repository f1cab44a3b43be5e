// The launches of a mini-batch.
//
// A mini-batch is a chain of dependent steps (hop 0, its compaction, hop 1, ..., the row copies), and
// the step that takes longest, the copy of host-tier rows, needs only a few dozen workgroups, because
// the host link and not the GPU limits it.  The paper runs such steps as operators on separate
// streams (Sec. 3.3, intra-mini-batch pipeline: the requests for the vertices of one hop go out while
// the next hop is sampled).  Here the overlap is inside a launch instead: a launch carries several
// *roles*, each a range of its workgroups with a job of its own, so no second stream, event or
// hardware queue is involved (this part has four hardware queues per process, and a dependent launch
// beside a saturated link costs several microseconds).  For a two-hop batch:
//
//   sample     hop 0 (the count pass of the seeds folded in; inserts seeds and flat_0 into the tables)
//   compact    flat_0 -> frontier_1 + indptr_1   |  [seeds | flat_0] -> stage 0 of unique, tier lists, miss list
//   sample     hop 1                             |  host-tier copy of stage 0
//   compact    flat_1 -> stage 1 (the last) of unique, tier lists, miss list, stats
//   finish     host-tier copy of stage 1  |  HBM-tier copy of all stages  |  inverse  |  emptying of the next batch's table
//
// Five launches; the host link is busy from the second compaction of hop 0 on, except while a
// compaction runs.
#include "kernels.hpp"

namespace helios {

namespace {

template <int G>
__global__ __launch_bounds__(kBlock) void batch_sample_kernel(HopArgs hop, Role r_hop, GatherArgs link, Role r_link) {
    if (r_link.mine()) {                         // the link's workgroups come first: they start first
        copy_rows_any(link, r_link.rb(), r_link.blocks, true);
        return;
    }
    if (r_hop.mine()) sample_role<G>(hop, r_hop.rb(), r_hop.blocks);
}

__global__ __launch_bounds__(kBlock) void batch_compact_kernel(CompactArgs hop, Role r_hop, CompactArgs look, Role r_look) {
    if (r_look.mine()) {
        compact_role<kCompactLookup>(look, r_look.rb(), r_look.blocks);
        return;
    }
    if (r_hop.mine()) compact_role<kCompactNextHop>(hop, r_hop.rb(), r_hop.blocks);
}

// L, CPL, R: the shape of the HBM-tier copy loop for the row size; RF: rows per step of the host-tier copy
template <int L, int CPL, int R, int RF>
__global__ __launch_bounds__(kBlock) void batch_finish_kernel(GatherArgs hbm, Role r_hbm, GatherArgs link, Role r_link,
                                                              InverseArgs inv, Role r_inv, ClearJob clear, Role r_clear,
                                                              BatchTables bt, const BatchVars* vars) {
    if (r_link.mine()) {
        if constexpr (L == 0) copy_rows_long(link, r_link.rb(), r_link.blocks);
        else copy_rows<L == 0 ? 64 : L, CPL == 0 ? 1 : CPL, RF == 0 ? 1 : RF>(link, r_link.rb(), r_link.blocks);
        return;
    }
    if (r_hbm.mine()) {
        if constexpr (L == 0) copy_rows_long(hbm, r_hbm.rb(), r_hbm.blocks);
        else copy_rows<L == 0 ? 64 : L, CPL == 0 ? 1 : CPL, R == 0 ? 1 : R>(hbm, r_hbm.rb(), r_hbm.blocks);
        return;
    }
    if (r_inv.mine()) {
        inverse_role(inv, r_inv.rb(), r_inv.blocks);
        return;
    }
    if (r_clear.mine()) {
        // the table of the context's next batch; a recorded batch learns only on the device which one that is
        unsigned long long* table = vars ? bt.table((vars->table + 1) % kBatchTables) : clear.table;
        for (uint32_t w = r_clear.rb() * kBlock + threadIdx.x; table && w < clear.n_slots; w += r_clear.blocks * kBlock)
            table[w] = kEmptySlot;
    }
}

__global__ __launch_bounds__(kBlock) void clear_kernel(ClearJob c) { clear_slots(c); }

constexpr int kPublishThreads = 1024;

// one workgroup per role
__global__ __launch_bounds__(kPublishThreads) void clock_publish_kernel(const unsigned long long* clock, StampTable table,
                                                                        unsigned long long* host_out) {
    __shared__ unsigned long long s_lo[kPublishThreads / kWave], s_hi[kPublishThreads / kWave];
    const unsigned n_blocks = table.workgroups[blockIdx.x];
    const unsigned long long* mine = clock + table.offset[blockIdx.x];
    unsigned long long lo = ~0ull, hi = 0ull;
#pragma unroll 8
    for (unsigned b = threadIdx.x; b < n_blocks; b += kPublishThreads) {      // independent loads, issued together
        const unsigned long long a = mine[b], z = mine[n_blocks + b];
        lo = a < lo ? a : lo;
        hi = z > hi ? z : hi;
    }
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) {
        const unsigned long long lo2 = __shfl_xor(lo, d, kWave), hi2 = __shfl_xor(hi, d, kWave);
        lo = lo2 < lo ? lo2 : lo;
        hi = hi2 > hi ? hi2 : hi;
    }
    if ((threadIdx.x & (kWave - 1)) == 0) {
        s_lo[threadIdx.x / kWave] = lo;
        s_hi[threadIdx.x / kWave] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kPublishThreads / kWave; ++w) {
            lo = s_lo[w] < lo ? s_lo[w] : lo;
            hi = s_hi[w] > hi ? s_hi[w] : hi;
        }
        host_out[2 * blockIdx.x] = lo;
        host_out[2 * blockIdx.x + 1] = hi;
    }
}

}  // namespace

hipError_t launch_sample(hipStream_t stream, const HopArgs& hop, unsigned hop_blocks, const GatherArgs& link, unsigned link_blocks) {
    const Role r_link{0, link_blocks}, r_hop{link_blocks, hop_blocks};
    const dim3 grid(link_blocks + hop_blocks), block(kBlock);
    const int lanes = group_lanes(hop.fanout);
    if (lanes == 8) hipLaunchKernelGGL(batch_sample_kernel<8>, grid, block, 0, stream, hop, r_hop, link, r_link);
    else if (lanes == 16) hipLaunchKernelGGL(batch_sample_kernel<16>, grid, block, 0, stream, hop, r_hop, link, r_link);
    else if (lanes == 32) hipLaunchKernelGGL(batch_sample_kernel<32>, grid, block, 0, stream, hop, r_hop, link, r_link);
    else hipLaunchKernelGGL(batch_sample_kernel<64>, grid, block, 0, stream, hop, r_hop, link, r_link);
    return hipGetLastError();
}

hipError_t launch_compact(hipStream_t stream, const CompactArgs& hop, unsigned hop_blocks, const CompactArgs& look,
                          unsigned look_blocks) {
    const Role r_look{0, look_blocks}, r_hop{look_blocks, hop_blocks};
    hipLaunchKernelGGL(batch_compact_kernel, dim3(look_blocks + hop_blocks), dim3(kBlock), 0, stream, hop, r_hop, look, r_look);
    return hipGetLastError();
}

hipError_t launch_finish(hipStream_t stream, const GatherArgs& hbm, unsigned hbm_blocks, const GatherArgs& link,
                         unsigned link_blocks, const InverseArgs& inv, unsigned inv_blocks, const ClearJob& clear,
                         unsigned clear_blocks, const BatchTables& bt, const BatchVars* vars) {
    const Role r_link{0, link_blocks}, r_hbm{link_blocks, hbm_blocks}, r_inv{link_blocks + hbm_blocks, inv_blocks},
        r_clear{link_blocks + hbm_blocks + inv_blocks, clear_blocks};
    const unsigned total = link_blocks + hbm_blocks + inv_blocks + clear_blocks;
    if (total == 0) return hipSuccess;
    const dim3 grid(total), block(kBlock);
    const int chunks = hbm_blocks > 0 ? hbm.chunks : link_blocks > 0 ? link.chunks : 1;
    // the two copies move rows of the same size; their loops differ in the rows a group takes per step
#define HELIOS_CALL_(L, CPL, R)                                                                                            \
    hipLaunchKernelGGL((batch_finish_kernel<L, CPL, R, far_rows_per_step(L, CPL)>), grid, block, 0, stream, hbm, r_hbm, link, r_link, inv, \
                       r_inv, clear, r_clear, bt, vars)
    HELIOS_COPY_SHAPE_SWITCH(chunks, false, HELIOS_CALL_);
#undef HELIOS_CALL_
    return hipGetLastError();
}

hipError_t launch_clear(hipStream_t stream, const ClearJob& job) {
    if (!job.table || job.n_slots == 0) return hipSuccess;
    unsigned blocks = (job.n_slots + kBlock * 16 - 1) / (kBlock * 16);
    blocks = blocks < 1 ? 1 : blocks > 2048 ? 2048 : blocks;
    hipLaunchKernelGGL(clear_kernel, dim3(blocks), dim3(kBlock), 0, stream, job);
    return hipGetLastError();
}

hipError_t launch_clock_publish(hipStream_t stream, const uint64_t* clock, const StampTable& table, int n_roles,
                                uint64_t* host_out) {
    if (n_roles <= 0) return hipSuccess;
    hipLaunchKernelGGL(clock_publish_kernel, dim3(static_cast<unsigned>(n_roles)), dim3(kPublishThreads), 0, stream,
                       reinterpret_cast<const unsigned long long*>(clock), table, reinterpret_cast<unsigned long long*>(host_out));
    return hipGetLastError();
}

}  // namespace helios
