// One hop of uniform neighbour sampling without replacement over a CSR graph.
//
// One kernel per hop.  The work per node is two dependent random reads (the row
// bounds, then up to `fanout` entries of the row), so the kernel is bound by
// memory latency, not bandwidth: it is laid out to keep as many nodes in flight
// as possible and to put nothing between the two reads that does not have to be
// there.
//   - A group of G lanes owns one node (G = the smallest of 8, 16, 32, 64 that
//     covers the fan-out); a workgroup of 256 threads owns a tile of 256/G
//     consecutive frontier nodes.
//   - The group reads the node's row bounds; lane k computes the k-th Philox
//     draw and Floyd candidate, the group settles collisions with shuffles, and
//     lane k reads the k-th chosen neighbour.  All reads of a node are issued
//     together.
//   - While those reads are in flight the sample counts min(deg, fanout) are
//     scanned inside the workgroup and chained across workgroups (scan.hpp),
//     which gives every node its place in `flat` without a second kernel or a
//     host round trip.  Then lane k writes its neighbour.
// Fan-outs above 64 use one wave per node, loop over the picks in chunks of 64
// and keep the chosen positions in LDS.
#include "kernels.hpp"
#include "philox.hpp"

namespace helios {

namespace {

constexpr int kMaxFanout = 1024;

struct HopArgs {
    const int64_t* offsets;
    const int32_t* indices;
    int64_t n_nodes;
    const int32_t* frontier;
    int32_t* frontier_out;
    Count n_frontier;
    int32_t fanout;
    int32_t hop;
    uint64_t rng_seed;
    const BatchVars* vars;        // nullable: rng_seed (and, at hop 0, the frontier) come from here
    int64_t* indptr;
    int32_t* flat;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;
    unsigned long long* clear_table;
    uint32_t clear_slots;
    ScanState scan;
    int32_t* err;
};

template <int G>
__global__ __launch_bounds__(kBlock) void sample_hop_kernel(HopArgs a) {
    constexpr int kGroups = kBlock / G;          // nodes per tile
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_agg[1], s_excl[1];
    __shared__ ScanLookbackLds<1> s_look;
    __shared__ int32_t s_chosen[(G == kWave) ? kWavesPerBlock * kMaxFanout : 1];

    const uint32_t tile = blockIdx.x;
    const int group = threadIdx.x / G;
    const int l = threadIdx.x % G;
    const int64_t i = static_cast<int64_t>(tile) * kGroups + group;     // this group's frontier entry
    const uint64_t rng_seed = a.vars ? a.vars->rng_seed : a.rng_seed;
    const int32_t* frontier = (a.vars && a.hop == 0) ? a.vars->seeds : a.frontier;
    // fetched before the device-side frontier size has arrived; the buffer holds n_frontier.host entries
    const int32_t v_early = i < a.n_frontier.host ? frontier[i] : -1;
    const int64_t n = a.n_frontier.get();
    const int64_t n_tiles = (n + kGroups - 1) / kGroups;
    // side job: empty the hash table of the de-duplication that follows this hop
    for (uint32_t w = blockIdx.x * kBlock + threadIdx.x; w < a.clear_slots; w += gridDim.x * kBlock) a.clear_table[w] = ~0ull;
    if (tile == 0 && threadIdx.x == 0) {
        if (a.size_out) a.size_out[0] = n;
        if (n == 0) {                            // empty frontier: empty hop
            a.indptr[0] = 0;
            *a.n_flat_dev = 0;
            if (a.size_out) a.size_out[1] = 0;
        }
    }
    if (static_cast<int64_t>(tile) >= n_tiles) return;

    const int f = a.fanout;

    // ---- row bounds and sample count (the lanes of a group read the same words)
    int32_t v = 0, deg = 0;
    int64_t base = 0;
    if (i < n) {
        v = v_early;
        if (l == 0 && a.frontier_out && a.frontier_out != frontier) a.frontier_out[i] = v;
        if (v < 0 || static_cast<int64_t>(v) >= a.n_nodes) {
            raise(a.err, kErrData);
        } else {
            base = a.offsets[v];
            const int64_t d = a.offsets[v + 1] - base;
            if (d < 0 || d > 0x7fffffffLL) raise(a.err, kErrData);
            else deg = static_cast<int32_t>(d);
        }
    }
    const int cnt = deg < f ? deg : f;

    // ---- picks and neighbour reads for fan-outs that fit the group
    int32_t nbr = 0;
    if (f <= G && l < cnt) {
        int32_t pos = l;                                  // deg <= f: the whole row, CSR order
        if (deg > f) {
            const int32_t j = deg - f + l;                // position looked at in step l
            const int32_t t = static_cast<int32_t>(
                bounded(node_draw(rng_seed, v, a.hop, static_cast<uint32_t>(l)), static_cast<uint64_t>(j) + 1u));
            pos = t;
        }
        nbr = pos;                                        // settled below
    }
    if (f <= G) {
        // Floyd: step k takes t_k unless an earlier step already holds it, then it takes j_k.
        // Step i2's pick is final once steps < i2 have been applied to it.
        const bool floyd = deg > f && l < f;
        const int32_t j = deg - f + l;
        const int32_t t = nbr;
        int32_t s = nbr;
        for (int i2 = 0; i2 + 1 < f; ++i2) {
            const int32_t si = __shfl(s, i2, G);
            if (floyd && l > i2 && si == t) s = j;
        }
        if (l < cnt) nbr = a.indices[base + s];
    }

    // ---- place of every node's samples in `flat` (overlaps the reads above)
    uint32_t tile_total;
    const uint32_t local = block_exclusive_scan(l == 0 ? static_cast<uint32_t>(cnt) : 0u, s_wave, tile_total);
    if (threadIdx.x == 0) s_agg[0] = tile_total;
    scan_chained_prefix<1>(a.scan, tile, s_agg, s_excl, &s_look, a.err);
    const int64_t tile_base = s_excl[0];
    const int64_t out = tile_base + __shfl(local, 0, G);
    if (l == 0 && i < n) a.indptr[i] = out;
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = tile_base + tile_total;
        a.indptr[n] = total;
        *a.n_flat_dev = total;
        if (a.size_out) a.size_out[1] = total;
        if (total > a.flat_cap) raise(a.err, kErrCapacity);
    }

    if (f <= G) {
        if (l < cnt && out + l < a.flat_cap) a.flat[out + l] = nbr;
        return;
    }
    if constexpr (G == kWave) {                           // fan-out above 64: one wave per node
        if (deg <= f) {
            for (int k = l; k < deg; k += kWave)
                if (out + k < a.flat_cap) a.flat[out + k] = a.indices[base + k];
            return;
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
                if (out + k < a.flat_cap) a.flat[out + k] = a.indices[base + s];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

}  // namespace

int sample_group_lanes(int32_t fanout) { return fanout <= 8 ? 8 : fanout <= 16 ? 16 : fanout <= 32 ? 32 : 64; }

int64_t sample_hop_tiles(int64_t n_frontier_max, int32_t fanout) {
    const int64_t per_tile = kBlock / sample_group_lanes(fanout);
    const int64_t tiles = (n_frontier_max + per_tile - 1) / per_tile;
    return tiles < 1 ? 1 : tiles;              // the first tile also writes the sizes of an empty hop
}

hipError_t launch_sample_hop(hipStream_t stream, const CsrView& g, const int32_t* frontier_in, int32_t* frontier_out,
                             Count n_frontier, int64_t n_frontier_max, int32_t fanout, int32_t hop, uint64_t rng_seed,
                             const BatchVars* vars, int64_t* indptr, int32_t* flat, int64_t flat_cap, int64_t* n_flat_dev,
                             int64_t* size_out, unsigned long long* clear_table, uint32_t clear_slots,
                             const ScanState& scan, int32_t* err) {
    HopArgs a{g.offsets, g.indices, g.n_nodes, frontier_in, frontier_out, n_frontier, fanout, hop, rng_seed, vars,
              indptr, flat, flat_cap, n_flat_dev, size_out, clear_table, clear_table ? clear_slots : 0u, scan, err};
    const int lanes = sample_group_lanes(fanout);
    int64_t tiles = sample_hop_tiles(n_frontier_max, fanout);
    const dim3 grid(static_cast<unsigned>(tiles)), block(kBlock);
    if (lanes == 8) hipLaunchKernelGGL(sample_hop_kernel<8>, grid, block, 0, stream, a);
    else if (lanes == 16) hipLaunchKernelGGL(sample_hop_kernel<16>, grid, block, 0, stream, a);
    else if (lanes == 32) hipLaunchKernelGGL(sample_hop_kernel<32>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(sample_hop_kernel<64>, grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
