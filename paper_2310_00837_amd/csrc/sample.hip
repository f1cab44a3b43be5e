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
//
// The sampled IDs are de-duplicated right afterwards (into the next hop's
// frontier, and, in the whole-path call, into the batch's ID list), so the lane
// that writes a sample also inserts it into the hash tables of those
// de-duplications: they then start at their second pass, and a mini-batch has
// one kernel launch fewer per hop.  The tables must be empty before the first
// insert: each kernel here clears, on the way, the tables that the kernels
// after it fill.
#include "kernels.hpp"
#include "philox.hpp"

namespace helios {

namespace {

constexpr int kMaxFanout = 1024;

struct CountArgs {
    const int64_t* offsets;
    int64_t n_nodes;
    const int32_t* frontier;
    BatchFeed feed;               // recorded batch: the batch's variables come from the host's ring, and the frontier is their seeds
    int32_t* frontier_out;        // nullable: receives a copy of the frontier
    Count n;
    int32_t fanout;
    int64_t* indptr;
    int64_t flat_cap;
    int64_t* n_flat_dev;
    int64_t* size_out;            // nullable: [0] = frontier size, [1] = sample-list size
    ClearJob clear[2];            // tables that the sampling pass of this hop inserts into
    ScanState scan;
    int32_t* err;
};

__global__ __launch_bounds__(kBlock) void frontier_count_kernel(CountArgs a) {
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];
    __shared__ uint32_t s_ticket, s_agg[1], s_excl[1];
    __shared__ ScanLookbackLds<1> s_look;
    // A recorded batch starts here: every workgroup that counts reads the batch's variables from the slot of the host's
    // ring that the count of batches run so far selects (the read travels while the tables are cleared), and
    // the first workgroup leaves them in device memory for the kernels that follow.
    BatchVars bv{};
    const bool counts = static_cast<int64_t>(blockIdx.x) * kTileItems < a.n.host || blockIdx.x == 0;   // else: clears only
    if (a.feed.ring && counts) bv = a.feed.ring[*a.feed.batches_run % a.feed.ring_slots];
    clear_slots(a.clear[0]);                     // side job of the whole grid
    clear_slots(a.clear[1]);
    ScanState scan = a.scan;
    if (a.feed.ring) {
        scan.vars = nullptr;
        scan.epoch += bv.epoch_base;
        if (blockIdx.x == 0 && threadIdx.x == 0) *a.feed.vars_out = bv;
    }
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
    const uint32_t tile = scan_take_ticket(scan, static_cast<uint32_t>(n_tiles), &s_ticket);
    const int32_t* frontier = a.feed.ring ? bv.seeds : a.frontier;
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
    scan_chained_prefix<1>(scan, tile, s_agg, s_excl, &s_look, a.err);
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
    ClearJob clear;               // the table the next hop's sampling pass inserts into
    InsertInto hop_table;         // de-duplication of this hop's samples; position = place in flat
    InsertInto batch_table;       // de-duplication of [seeds | flat_0 | ...]; position = place in that list
    int32_t* cat_out;             // with batch_table: receives [seeds | flat_0 | ...]
    int64_t n_seeds;
    Count prev_flat[HELIOS_KERNELS_MAX_SEG - 1];   // sizes of flat_0 .. flat_{hop-1}
    uint32_t* batches_run;        // nullable: hop 0 of a recorded batch counts the batch (see frontier_count_kernel)
    int32_t* err;
};

// flat[at] = id has just been written: the same lane inserts id into the tables of the de-duplications
// that follow.  cat_at is the place of the sample in [seeds | flat_0 | ...].
__device__ __forceinline__ void insert_sample(const HopArgs& a, int32_t id, int64_t at, int64_t cat_at) {
    const bool node = id >= 0 && static_cast<int64_t>(id) < a.n_nodes;
    if (!node) raise(a.err, kErrData);
    if (a.hop_table.table)
        a.hop_table.slot_of[at] = node ? static_cast<int32_t>(table_insert(a.hop_table.table, a.hop_table.n_slots - 1,
                                                                           static_cast<uint32_t>(id), static_cast<uint32_t>(at)))
                                       : -1;
    if (a.batch_table.table) {
        a.cat_out[cat_at] = id;
        a.batch_table.slot_of[cat_at] =
            node ? static_cast<int32_t>(table_insert(a.batch_table.table, a.batch_table.n_slots - 1, static_cast<uint32_t>(id),
                                                     static_cast<uint32_t>(cat_at)))
                 : -1;
    }
}

template <int G>
__global__ __launch_bounds__(kBlock) void sample_hop_kernel(HopArgs a) {
    constexpr int kGroups = kBlock / G;          // nodes per workgroup and step
    __shared__ int32_t s_chosen[(G == kWave) ? kWavesPerBlock * kMaxFanout : 1];

    clear_slots(a.clear);                        // side job of the whole grid
    // the count pass has taken this batch's slot of the ring: the next batch takes the next one
    if (a.batches_run && blockIdx.x == 0 && threadIdx.x == 0) *a.batches_run += 1;

    const int group = threadIdx.x / G;
    const int l = threadIdx.x % G;
    const int f = a.fanout;
    const int64_t n = a.n_frontier.get();
    const bool seeds_too = a.batch_table.table && a.hop == 0;   // the frontier of hop 0 is the head of the batch's list
    int64_t cat_base = a.n_seeds;                // where flat_hop starts in [seeds | flat_0 | ...]
    for (int h = 0; h < a.hop; ++h) cat_base += a.prev_flat[h].get();
    if (f <= 0 && !seeds_too) return;
    const uint64_t rng_seed = a.vars ? a.vars->rng_seed : a.rng_seed;
    const int64_t step = static_cast<int64_t>(gridDim.x) * kGroups;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kGroups + group; i < n; i += step) {
        // the lanes of a group read the same words
        const int32_t v = a.frontier[i];
        const int64_t out = a.indptr[i];
        if (seeds_too && l == 0) {               // seed i is element i of the batch's list
            a.cat_out[i] = v;
            a.batch_table.slot_of[i] = v >= 0 && static_cast<int64_t>(v) < a.n_nodes
                                           ? static_cast<int32_t>(table_insert(a.batch_table.table, a.batch_table.n_slots - 1,
                                                                               static_cast<uint32_t>(v), static_cast<uint32_t>(i)))
                                           : -1;
        }
        if (f <= 0) continue;
        if (v < 0 || static_cast<int64_t>(v) >= a.n_nodes) continue;      // reported by the count pass
        const int64_t base = a.offsets[v];
        const int64_t d64 = a.offsets[v + 1] - base;
        if (d64 <= 0 || d64 > 0x7fffffffLL) continue;
        const int32_t deg = static_cast<int32_t>(d64);
        const int cnt = deg < f ? deg : f;
        // `out` can only be off if an earlier output overflowed its capacity; never write outside flat, but
        // write every place below the capacity: the de-duplications read all of them
        const bool out_ok = out >= 0;
        const int64_t room = a.flat_cap - out;   // samples of this node that fit

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
            if (l < cnt && out_ok && l < room) {
                const int32_t id = a.indices[base + s];
                a.flat[out + l] = id;
                insert_sample(a, id, out + l, cat_base + out + l);
            }
            continue;
        }
        if constexpr (G == kWave) {                           // fan-out above 64: one wave per node
            if (deg <= f) {
                for (int k = l; k < deg; k += kWave)
                    if (out_ok && k < room) {
                        const int32_t id = a.indices[base + k];
                        a.flat[out + k] = id;
                        insert_sample(a, id, out + k, cat_base + out + k);
                    }
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
                    if (out_ok && k < room) {
                        const int32_t id = a.indices[base + s];
                        a.flat[out + k] = id;
                        insert_sample(a, id, out + k, cat_base + out + k);
                    }
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

hipError_t launch_frontier_count(hipStream_t stream, const CsrView& g, const int32_t* frontier, const BatchFeed& feed,
                                 int32_t* frontier_out, Count n, int64_t n_max, int32_t fanout, int64_t* indptr,
                                 int64_t flat_cap, int64_t* n_flat_dev, int64_t* size_out, ClearJob clear_a, ClearJob clear_b,
                                 const ScanState& scan, int32_t* err) {
    CountArgs a{g.offsets, g.n_nodes, frontier, feed, frontier_out, n, fanout, indptr, flat_cap, n_flat_dev, size_out,
                {clear_a, clear_b}, scan, err};
    int64_t tiles = (n_max + kTileItems - 1) / kTileItems;
    if (tiles < 1) tiles = 1;                  // the first workgroup also writes the sizes of an empty hop
    // enough workgroups for the clearing (16 words a thread), all resident at once
    const int64_t words = static_cast<int64_t>(clear_a.table ? clear_a.n_slots : 0) + (clear_b.table ? clear_b.n_slots : 0);
    int64_t blocks = (words + kBlock * 16 - 1) / (kBlock * 16);
    if (blocks > 2048) blocks = 2048;
    if (blocks < tiles) blocks = tiles;
    hipLaunchKernelGGL(frontier_count_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sample_hop(hipStream_t stream, const CsrView& g, const int32_t* frontier, const int64_t* indptr,
                             Count n_frontier, int64_t n_frontier_max, int32_t fanout, int32_t hop, uint64_t rng_seed,
                             const BatchVars* vars, int32_t* flat, int64_t flat_cap, ClearJob clear, InsertInto hop_table,
                             InsertInto batch_table, int32_t* cat_out, int64_t n_seeds, const Count* prev_flat,
                             uint32_t* batches_run, int32_t* err) {
    HopArgs a{g.offsets, g.indices, g.n_nodes, frontier, indptr, n_frontier, fanout, hop, rng_seed, vars,
              flat, flat_cap, clear, hop_table, batch_table, cat_out, n_seeds, {}, hop == 0 ? batches_run : nullptr, err};
    for (int h = 0; h < hop && h < HELIOS_KERNELS_MAX_SEG - 1; ++h) a.prev_flat[h] = prev_flat[h];
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
