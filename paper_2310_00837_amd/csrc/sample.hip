// One hop of uniform neighbour sampling without replacement over a CSR graph.
//
// One kernel per hop.  A workgroup owns a tile of 256 frontier nodes:
//   1. one thread per node reads the node's row bounds (two random 8-byte
//      reads) and derives its sample count min(deg, fanout);
//   2. the counts are scanned inside the workgroup and chained across
//      workgroups (scan.hpp), which gives every node its place in `flat`
//      without a second kernel or a host round trip;
//   3. groups of G lanes (G = the smallest of 8, 16, 32, 64 that covers the
//      fan-out) take the tile's nodes in turn: lane k computes the k-th
//      Philox draw and Floyd candidate, the group settles collisions with
//      shuffles, and lane k reads and writes the k-th neighbour.  The f index
//      reads of a node are issued together, so their latency overlaps.
// Fan-outs above 64 use one wave per node and keep the chosen positions in LDS.
#include "kernels.hpp"
#include "philox.hpp"

namespace helios {

namespace {

constexpr int kTile = kBlock;                 // frontier nodes per workgroup
constexpr int kMaxFanout = 1024;

struct HopArgs {
    const int64_t* offsets;
    const int32_t* indices;
    int64_t n_nodes;
    const int32_t* frontier;
    Count n_frontier;
    int32_t fanout;
    int32_t hop;
    uint64_t rng_seed;
    int64_t* indptr;
    int32_t* flat;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;
    ScanState scan;
    int32_t* err;
};

template <int G>
__global__ __launch_bounds__(kBlock) void sample_hop_kernel(HopArgs a) {
    __shared__ int64_t s_base[kTile];
    __shared__ int32_t s_deg[kTile];
    __shared__ int32_t s_node[kTile];
    __shared__ uint32_t s_off[kTile];
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[1], s_excl[1];
    __shared__ int32_t s_chosen[(G == kWave) ? kWavesPerBlock * kMaxFanout : 1];

    const uint32_t tile = scan_take_ticket(a.scan, &s_ticket);
    const int64_t n = a.n_frontier.get();
    const int64_t n_tiles = (n + kTile - 1) / kTile;
    if (tile == 0 && threadIdx.x == 0) {
        if (a.size_out) a.size_out[0] = n;
        if (n == 0) {                         // empty frontier: empty hop
            a.indptr[0] = 0;
            *a.n_flat_dev = 0;
            if (a.size_out) a.size_out[1] = 0;
        }
    }
    if (static_cast<int64_t>(tile) >= n_tiles) return;

    // ---- 1. row bounds and sample count of this thread's node
    const int64_t first = static_cast<int64_t>(tile) * kTile;
    const int tile_count = static_cast<int>(n - first < kTile ? n - first : kTile);
    const int f = a.fanout;
    uint32_t cnt = 0;
    if (static_cast<int>(threadIdx.x) < tile_count) {
        const int32_t v = a.frontier[first + threadIdx.x];
        int64_t base = 0, deg = 0;
        if (v < 0 || static_cast<int64_t>(v) >= a.n_nodes) {
            raise(a.err, kErrData);
        } else {
            base = a.offsets[v];
            deg = a.offsets[v + 1] - base;
            if (deg < 0 || deg > 0x7fffffffLL) { raise(a.err, kErrData); deg = 0; }
        }
        s_node[threadIdx.x] = v;
        s_base[threadIdx.x] = base;
        s_deg[threadIdx.x] = static_cast<int32_t>(deg);
        cnt = static_cast<uint32_t>(deg < f ? deg : f);
    }

    // ---- 2. place of every node's samples in `flat`
    uint32_t tile_total;
    const uint32_t local = block_exclusive_scan(cnt, s_wave, tile_total);
    s_off[threadIdx.x] = local;
    if (threadIdx.x == 0) s_agg[0] = tile_total;
    scan_chained_prefix<1>(a.scan, tile, s_agg, s_excl);
    const int64_t tile_base = s_excl[0];
    if (static_cast<int>(threadIdx.x) < tile_count) a.indptr[first + threadIdx.x] = tile_base + local;
    if (static_cast<int64_t>(tile) == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = tile_base + tile_total;
        a.indptr[n] = total;
        *a.n_flat_dev = total;
        if (a.size_out) a.size_out[1] = total;
        if (total > a.flat_cap) raise(a.err, kErrCapacity);
    }
    if (f <= 0) return;

    // ---- 3. G lanes per node
    constexpr int kGroups = kBlock / G;
    const int group = threadIdx.x / G;
    const int l = threadIdx.x % G;
    for (int i = group; i < tile_count; i += kGroups) {
        const int64_t base = s_base[i];
        const int32_t deg = s_deg[i];
        const int64_t out = tile_base + s_off[i];
        if (deg <= f) {                                   // whole row, CSR order
            for (int k = l; k < deg; k += G)
                if (out + k < a.flat_cap) a.flat[out + k] = a.indices[base + k];
        } else if (f <= G) {
            const int32_t v = s_node[i];
            const int32_t j = deg - f + l;                // position looked at in step l
            int32_t t = j, s = j;
            if (l < f) {
                t = static_cast<int32_t>(bounded(node_draw(a.rng_seed, v, a.hop, static_cast<uint32_t>(l)),
                                                 static_cast<uint64_t>(j) + 1u));
                s = t;
            }
            // step i2's pick is final once steps < i2 have been applied to it
            for (int i2 = 0; i2 + 1 < f; ++i2) {
                const int32_t si = __shfl(s, i2, G);
                if (l > i2 && l < f && si == t) s = j;
            }
            if (l < f && out + l < a.flat_cap) a.flat[out + l] = a.indices[base + s];
        } else if constexpr (G == kWave) {                // fan-out above 64: one wave per node
            const int32_t v = s_node[i];
            int32_t* chosen = s_chosen + wave_id() * kMaxFanout;
            for (int c0 = 0; c0 < f; c0 += kWave) {
                const int k = c0 + l;
                const bool active = k < f;
                const int32_t j = deg - f + k;
                int32_t t = -1, s = -1;
                if (active) {
                    t = static_cast<int32_t>(bounded(node_draw(a.rng_seed, v, a.hop, static_cast<uint32_t>(k)),
                                                     static_cast<uint64_t>(j) + 1u));
                    s = t;
                    for (int p = 0; p < c0; ++p)
                        if (chosen[p] == t) s = j;        // taken in an earlier chunk
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
}

}  // namespace

hipError_t launch_sample_hop(hipStream_t stream, const CsrView& g, const int32_t* frontier, Count n_frontier,
                             int64_t n_frontier_max, int32_t fanout, int32_t hop, uint64_t rng_seed,
                             int64_t* indptr, int32_t* flat, int64_t flat_cap, int64_t* n_flat_dev,
                             int64_t* size_out, const ScanState& scan, int32_t* err) {
    HopArgs a{g.offsets, g.indices, g.n_nodes, frontier, n_frontier, fanout, hop, rng_seed,
              indptr, flat, flat_cap, n_flat_dev, size_out, scan, err};
    int64_t tiles = (n_frontier_max + kTile - 1) / kTile;
    if (tiles < 1) tiles = 1;                  // the first tile also writes the sizes of an empty hop
    const dim3 grid(static_cast<unsigned>(tiles)), block(kBlock);
    if (fanout <= 8) hipLaunchKernelGGL(sample_hop_kernel<8>, grid, block, 0, stream, a);
    else if (fanout <= 16) hipLaunchKernelGGL(sample_hop_kernel<16>, grid, block, 0, stream, a);
    else if (fanout <= 32) hipLaunchKernelGGL(sample_hop_kernel<32>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(sample_hop_kernel<64>, grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace helios
