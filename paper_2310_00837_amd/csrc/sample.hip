// One hop of uniform neighbour sampling without replacement over a CSR graph.
//
// The work per node is two dependent random reads (the row bounds, then up to
// `fanout` entries of the row), so a hop is bound by memory latency, not
// bandwidth.  It is split in two so that the kernel that does the sampling has
// no dependence between workgroups at all:
//
//   count   one thread per four frontier nodes: row bounds -> sample count
//           min(deg, fanout); the counts are scanned in the workgroup and
//           chained across workgroups (scan.hpp) into indptr, each node's place
//           in `flat`.  For hop 0 this is frontier_count_kernel below; for the
//           later hops the de-duplication that produces the frontier does it in
//           the same pass (dedup.hip), so those hops need no kernel for it.
//   sample  a group of G lanes owns one node (G = the smallest of 8, 16, 32, 64
//           that covers the fan-out): lane k computes the k-th Philox draw and
//           Floyd candidate, the group settles collisions with shuffles, and
//           lane k reads the k-th chosen neighbour and writes it to
//           flat[indptr[i] + k].  All reads of a node are issued together; any
//           number of workgroups can run, in any order.
// Fan-outs above 64 use one wave per node, loop over the picks in chunks of 64
// and keep the chosen positions in LDS.
#include "kernels.hpp"
#include "philox.hpp"

namespace helios {

namespace {

constexpr int kMaxFanout = 1024;

struct CountArgs {
    const int64_t* offsets;
    int64_t n_nodes;
    const int32_t* frontier;
    const BatchVars* vars;        // nullable: the frontier is vars->seeds (recorded batch)
    int32_t* frontier_out;        // nullable: receives a copy of the frontier
    Count n;
    int32_t fanout;
    int64_t* indptr;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;            // nullable: [0] = frontier size, [1] = sample-list size
    ScanState scan;
    int32_t* err;
};

__global__ __launch_bounds__(kBlock) void frontier_count_kernel(CountArgs a) {
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[1], s_excl[1];
    __shared__ ScanLookbackLds<1> s_look;
    const int64_t n = a.n.get();
    const int64_t n_tiles = (n + kTileItems - 1) / kTileItems;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (a.size_out) a.size_out[0] = n;
        if (n == 0) {                            // empty frontier: empty hop
            a.indptr[0] = 0;
            *a.n_flat_dev = 0;
            if (a.size_out) a.size_out[1] = 0;
        }
    }
    if (static_cast<int64_t>(blockIdx.x) >= n_tiles) return;
    const uint32_t tile = scan_take_ticket(a.scan, static_cast<uint32_t>(n_tiles), &s_ticket);
    const int32_t* frontier = a.vars ? a.vars->seeds : a.frontier;
    const int64_t j0 = static_cast<int64_t>(tile) * kTileItems + static_cast<int64_t>(threadIdx.x) * kItemsPerThread;
    int32_t v[kItemsPerThread];
    uint32_t cnt[kItemsPerThread];
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) v[k] = j0 + k < n ? frontier[j0 + k] : -1;
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        cnt[k] = 0;
        if (j0 + k < n) {
            if (a.frontier_out && a.frontier_out != frontier) a.frontier_out[j0 + k] = v[k];
            cnt[k] = sample_count(a.offsets, a.n_nodes, v[k], a.fanout, a.err);
        }
        sum += cnt[k];
    }
    uint32_t tile_total;
    const uint32_t local = block_exclusive_scan(sum, s_wave, tile_total);
    if (threadIdx.x == 0) s_agg[0] = tile_total;
    scan_chained_prefix<1>(a.scan, tile, s_agg, s_excl, &s_look, a.err);
    int64_t at = static_cast<int64_t>(s_excl[0]) + local;
#pragma unroll
    for (int k = 0; k < kItemsPerThread; ++k) {
        if (j0 + k < n) a.indptr[j0 + k] = at;
        at += cnt[k];
    }
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = static_cast<int64_t>(s_excl[0]) + tile_total;
        a.indptr[n] = total;
        *a.n_flat_dev = total;
        if (a.size_out) a.size_out[1] = total;
        if (total > a.flat_cap) raise(a.err, kErrCapacity);
    }
}

struct HopArgs {
    const int64_t* offsets;
    const int32_t* indices;
    int64_t n_nodes;
    const int32_t* frontier;
    const int64_t* indptr;
    Count n_frontier;
    int32_t fanout;
    int32_t hop;
    uint64_t rng_seed;
    const BatchVars* vars;        // nullable: rng_seed comes from here (recorded batch)
    int32_t* flat;
    int64_t flat_cap;
    unsigned long long* clear_table;
    uint32_t clear_slots;
};

template <int G>
__global__ __launch_bounds__(kBlock) void sample_hop_kernel(HopArgs a) {
    constexpr int kGroups = kBlock / G;          // nodes per workgroup and step
    __shared__ int32_t s_chosen[(G == kWave) ? kWavesPerBlock * kMaxFanout : 1];

    // side job: empty the hash table of the de-duplication that follows this hop
    for (uint32_t w = blockIdx.x * kBlock + threadIdx.x; w < a.clear_slots; w += gridDim.x * kBlock) a.clear_table[w] = ~0ull;

    const int group = threadIdx.x / G;
    const int l = threadIdx.x % G;
    const int f = a.fanout;
    if (f <= 0) return;
    const int64_t n = a.n_frontier.get();
    const uint64_t rng_seed = a.vars ? a.vars->rng_seed : a.rng_seed;
    const int64_t step = static_cast<int64_t>(gridDim.x) * kGroups;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kGroups + group; i < n; i += step) {
        // the lanes of a group read the same words
        const int32_t v = a.frontier[i];
        const int64_t out = a.indptr[i];
        if (v < 0 || static_cast<int64_t>(v) >= a.n_nodes) continue;      // reported by the count pass
        const int64_t base = a.offsets[v];
        const int64_t d64 = a.offsets[v + 1] - base;
        if (d64 <= 0 || d64 > 0x7fffffffLL) continue;
        const int32_t deg = static_cast<int32_t>(d64);
        const int cnt = deg < f ? deg : f;
        // `out` can only be off if an earlier output overflowed its capacity; never write outside flat
        const bool out_ok = out >= 0 && out + cnt <= a.flat_cap;

        if (f <= G) {
            int32_t pos = l;                                  // deg <= f: the whole row, CSR order
            const bool floyd = deg > f && l < f;
            const int32_t j = deg - f + l;                    // position looked at in step l
            if (floyd)
                pos = static_cast<int32_t>(bounded(node_draw(rng_seed, v, a.hop, static_cast<uint32_t>(l)),
                                                   static_cast<uint64_t>(j) + 1u));
            // Floyd: step k takes t_k unless an earlier step already holds it, then it takes j_k.
            // Step i2's pick is final once steps < i2 have been applied to it.
            const int32_t t = pos;
            int32_t s = pos;
            if (deg > f) {                                    // uniform over the group
                for (int i2 = 0; i2 + 1 < f; ++i2) {
                    const int32_t si = __shfl(s, i2, G);
                    if (floyd && l > i2 && si == t) s = j;
                }
            }
            if (l < cnt && out_ok) a.flat[out + l] = a.indices[base + s];
            continue;
        }
        if constexpr (G == kWave) {                           // fan-out above 64: one wave per node
            if (deg <= f) {
                for (int k = l; k < deg; k += kWave)
                    if (out_ok) a.flat[out + k] = a.indices[base + k];
                continue;
            }
            int32_t* chosen = s_chosen + wave_id() * kMaxFanout;
            for (int c0 = 0; c0 < f; c0 += kWave) {
                const int k = c0 + l;
                const bool active = k < f;
                const int32_t j = deg - f + k;
                int32_t t = -1, s = -1;
                if (active) {
                    t = static_cast<int32_t>(bounded(node_draw(rng_seed, v, a.hop, static_cast<uint32_t>(k)),
                                                     static_cast<uint64_t>(j) + 1u));
                    s = t;
                    for (int p = 0; p < c0; ++p)
                        if (chosen[p] == t) s = j;            // taken in an earlier chunk
                }
                const int in_chunk = f - c0 < kWave ? f - c0 : kWave;
                for (int i2 = 0; i2 + 1 < in_chunk; ++i2) {
                    const int32_t si = __shfl(s, i2, kWave);
                    if (active && l > i2 && si == t) s = j;
                }
                if (active) {
                    chosen[k] = s;
                    if (out_ok) a.flat[out + k] = a.indices[base + s];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
    }
}

int group_lanes(int32_t fanout) { return fanout <= 8 ? 8 : fanout <= 16 ? 16 : fanout <= 32 ? 32 : 64; }

}  // namespace

hipError_t launch_frontier_count(hipStream_t stream, const CsrView& g, const int32_t* frontier, const BatchVars* vars,
                                 int32_t* frontier_out, Count n, int64_t n_max, int32_t fanout, int64_t* indptr,
                                 int64_t flat_cap, int64_t* n_flat_dev, int64_t* size_out, const ScanState& scan,
                                 int32_t* err) {
    CountArgs a{g.offsets, g.n_nodes, frontier, vars, frontier_out, n, fanout, indptr, flat_cap, n_flat_dev, size_out,
                scan, err};
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    if (tiles < 1) tiles = 1;                  // the first workgroup also writes the sizes of an empty hop
    hipLaunchKernelGGL(frontier_count_kernel, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sample_hop(hipStream_t stream, const CsrView& g, const int32_t* frontier, const int64_t* indptr,
                             Count n_frontier, int64_t n_frontier_max, int32_t fanout, int32_t hop, uint64_t rng_seed,
                             const BatchVars* vars, int32_t* flat, int64_t flat_cap, unsigned long long* clear_table,
                             uint32_t clear_slots) {
    HopArgs a{g.offsets, g.indices, g.n_nodes, frontier, indptr, n_frontier, fanout, hop, rng_seed, vars,
              flat, flat_cap, clear_table, clear_table ? clear_slots : 0u};
    const int lanes = group_lanes(fanout);
    const int64_t per_block = kBlock / lanes;
    int64_t blocks = (n_frontier_max + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kBlock);
    if (lanes == 8) hipLaunchKernelGGL(sample_hop_kernel<8>, grid, block, 0, stream, a);
    else if (lanes == 16) hipLaunchKernelGGL(sample_hop_kernel<16>, grid, block, 0, stream, a);
    else if (lanes == 32) hipLaunchKernelGGL(sample_hop_kernel<32>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(sample_hop_kernel<64>, grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
