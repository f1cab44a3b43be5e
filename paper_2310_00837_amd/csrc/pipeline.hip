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
//              (|  the rows of the miss list from the storage stand-in, if the batch serves its own misses)
//
// Five launches; the host link is busy from the end of the first compaction on, except while a
// compaction runs.
#include "kernels.hpp"

namespace helios {

namespace {

// Every launch below takes the roles of up to kMaxGang mini-batches (a "gang": batches of different
// contexts that share a stream and go through their steps together), so that the chain of short,
// latency-bound launches is paid once per gang and not once per batch.  A workgroup looks up which
// member's role it belongs to; the members' arguments sit side by side in the kernel arguments.
// The link roles of all members come first in every launch: they start first.
template <int G>
__global__ __launch_bounds__(kBlock) void batch_sample_kernel(SampleGang g) {
#pragma unroll 1
    for (int m = 0; m < g.n; ++m) {
        const SampleMember& a = g.m[m];
        if (a.r_link.mine()) {
            copy_rows_any(a.link, a.r_link.rb(), a.r_link.blocks, true);
            return;
        }
        if (a.r_hop.mine()) {
            sample_role<G>(a.hop, a.r_hop.rb(), a.r_hop.blocks);
            return;
        }
    }
}

__global__ __launch_bounds__(kBlock) void batch_compact_kernel(CompactGang g) {
#pragma unroll 1
    for (int m = 0; m < g.n; ++m) {
        const CompactMember& a = g.m[m];
        if (a.r_look.mine()) {
            compact_role<kCompactLookup>(a.look, a.r_look.rb(), a.r_look.blocks);
            return;
        }
        if (a.r_hop.mine()) {
            compact_role<kCompactNextHop>(a.hop, a.r_hop.rb(), a.r_hop.blocks);
            return;
        }
    }
}

// L, CPL, R: the shape of the HBM-tier copy loop for the row size; RF: rows per step of the host-tier copy
template <int L, int CPL, int R, int RF>
__global__ __launch_bounds__(kBlock) void batch_finish_kernel(FinishGang g) {
#pragma unroll 1
    for (int m = 0; m < g.n; ++m) {
        const FinishMember& a = g.m[m];
        if (a.r_link.mine()) {
            if constexpr (L == 0) copy_rows_long(a.link, a.r_link.rb(), a.r_link.blocks);
            else copy_rows<L == 0 ? 64 : L, CPL == 0 ? 1 : CPL, RF == 0 ? 1 : RF>(a.link, a.r_link.rb(), a.r_link.blocks);
            return;
        }
        if (a.r_miss.mine()) {
            if constexpr (L == 0) copy_rows_long(a.miss, a.r_miss.rb(), a.r_miss.blocks);
            else copy_rows<L == 0 ? 64 : L, CPL == 0 ? 1 : CPL, RF == 0 ? 1 : RF>(a.miss, a.r_miss.rb(), a.r_miss.blocks);
            return;
        }
        if (a.r_hbm.mine()) {
            if constexpr (L == 0) copy_rows_long(a.hbm, a.r_hbm.rb(), a.r_hbm.blocks);
            else copy_rows<L == 0 ? 64 : L, CPL == 0 ? 1 : CPL, R == 0 ? 1 : R>(a.hbm, a.r_hbm.rb(), a.r_hbm.blocks);
            return;
        }
        if (a.r_inv.mine()) {
            inverse_role(a.inv, a.r_inv.rb(), a.r_inv.blocks);
            return;
        }
        if (a.r_clear.mine()) {
            // the table of the context's next batch; a recorded batch learns only on the device which one that is
            unsigned long long* table = a.vars ? a.bt.table((a.vars->table + 1) % kBatchTables) : a.clear.table;
            for (uint32_t w = a.r_clear.rb() * kBlock + threadIdx.x; table && w < a.clear.n_slots; w += a.r_clear.blocks * kBlock)
                table[w] = kEmptySlot;
            return;
        }
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

// Workgroup ranges: the link roles of all members first, then the members' other roles.
hipError_t launch_sample(hipStream_t stream, const SampleJob* jobs, int n) {
    if (n < 1 || n > kMaxGang) return hipErrorInvalidValue;
    SampleGang g{};
    g.n = n;
    unsigned at = 0;
    for (int m = 0; m < n; ++m) {
        g.m[m].hop = jobs[m].hop;
        g.m[m].link = jobs[m].link;
        g.m[m].r_link = Role{at, jobs[m].link_blocks};
        at += jobs[m].link_blocks;
    }
    for (int m = 0; m < n; ++m) {
        g.m[m].r_hop = Role{at, jobs[m].hop_blocks};
        at += jobs[m].hop_blocks;
        if (group_lanes(jobs[m].hop.fanout) != group_lanes(jobs[0].hop.fanout)) return hipErrorInvalidValue;
    }
    if (at == 0) return hipSuccess;
    const dim3 grid(at), block(kBlock);
    const int lanes = group_lanes(jobs[0].hop.fanout);
    if (lanes == 8) hipLaunchKernelGGL(batch_sample_kernel<8>, grid, block, 0, stream, g);
    else if (lanes == 16) hipLaunchKernelGGL(batch_sample_kernel<16>, grid, block, 0, stream, g);
    else if (lanes == 32) hipLaunchKernelGGL(batch_sample_kernel<32>, grid, block, 0, stream, g);
    else hipLaunchKernelGGL(batch_sample_kernel<64>, grid, block, 0, stream, g);
    return hipGetLastError();
}

hipError_t launch_compact(hipStream_t stream, const CompactJob* jobs, int n) {
    if (n < 1 || n > kMaxGang) return hipErrorInvalidValue;
    CompactGang g{};
    g.n = n;
    unsigned at = 0;
    for (int m = 0; m < n; ++m) {
        g.m[m].hop = jobs[m].hop;
        g.m[m].look = jobs[m].look;
        g.m[m].r_look = Role{at, jobs[m].look_blocks};
        at += jobs[m].look_blocks;
    }
    for (int m = 0; m < n; ++m) {
        g.m[m].r_hop = Role{at, jobs[m].hop_blocks};
        at += jobs[m].hop_blocks;
    }
    if (at == 0) return hipSuccess;
    hipLaunchKernelGGL(batch_compact_kernel, dim3(at), dim3(kBlock), 0, stream, g);
    return hipGetLastError();
}

hipError_t launch_finish(hipStream_t stream, const FinishJob* jobs, int n) {
    if (n < 1 || n > kMaxGang) return hipErrorInvalidValue;
    FinishGang g{};
    g.n = n;
    unsigned at = 0;
    int chunks = 0;
    for (int m = 0; m < n; ++m) {
        FinishMember& a = g.m[m];
        a.hbm = jobs[m].hbm;
        a.link = jobs[m].link;
        a.inv = jobs[m].inv;
        a.clear = jobs[m].clear;
        a.bt = jobs[m].bt;
        a.vars = jobs[m].vars;
        a.miss = jobs[m].miss;
        a.r_link = Role{at, jobs[m].link_blocks};
        at += jobs[m].link_blocks;
        a.r_miss = Role{at, jobs[m].miss_blocks};
        at += jobs[m].miss_blocks;
        // the copies of all members move rows of one size (the loops are compiled for it)
        const int mine = jobs[m].hbm_blocks > 0 ? jobs[m].hbm.chunks : jobs[m].link_blocks > 0 ? jobs[m].link.chunks
                         : jobs[m].miss_blocks > 0 ? jobs[m].miss.chunks : 0;
        if (mine > 0 && chunks > 0 && mine != chunks) return hipErrorInvalidValue;
        if (mine > 0) chunks = mine;
    }
    for (int m = 0; m < n; ++m) {
        FinishMember& a = g.m[m];
        a.r_hbm = Role{at, jobs[m].hbm_blocks};
        at += jobs[m].hbm_blocks;
    }
    for (int m = 0; m < n; ++m) {
        FinishMember& a = g.m[m];
        a.r_inv = Role{at, jobs[m].inv_blocks};
        at += jobs[m].inv_blocks;
        a.r_clear = Role{at, jobs[m].clear_blocks};
        at += jobs[m].clear_blocks;
    }
    if (at == 0) return hipSuccess;
    if (chunks == 0) chunks = 1;
    const dim3 grid(at), block(kBlock);
    // the two copies move rows of the same size; their loops differ in the rows a group takes per step
#define HELIOS_CALL_(L, CPL, R) \
    hipLaunchKernelGGL((batch_finish_kernel<L, CPL, R, far_rows_per_step(L, CPL)>), grid, block, 0, stream, g)
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
