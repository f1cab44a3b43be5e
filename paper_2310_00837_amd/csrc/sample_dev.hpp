// Device code of one hop of uniform neighbour sampling without replacement over a CSR graph.
//
// The work per node is two dependent random reads (the row bounds, then up to `fanout` entries of
// the row), so a hop is bound by memory latency, not bandwidth.  It has two parts:
//
//   count   row bounds -> sample count min(deg, fanout) per frontier node, scanned into indptr, each
//           node's place in `flat`.  For hop 0 of a batch of at most kFoldMaxSeeds seeds every
//           workgroup of the sampling pass redoes this scan for the whole seed list in LDS (a
//           thousand cached 16-byte reads cost less than a kernel launch); larger seed lists get
//           frontier_count_kernel (sample.hip) first; for the later hops the de-duplication that
//           produces the frontier does it in the same pass (compact_dev.hpp).
//   sample  a group of G lanes owns one node (G = the smallest of 8, 16, 32, 64 that covers the
//           fan-out): lane k computes the k-th Philox draw and Floyd candidate, the group settles
//           collisions with shuffles, and lane k reads the k-th chosen neighbour and writes it to
//           flat[indptr[i] + k].  All reads of a node are issued together; any number of
//           workgroups can run, in any order.
// Fan-outs above 64 use one wave per node, loop over the picks in chunks of 64 and keep the chosen
// positions in LDS.
//
// The sampled IDs are de-duplicated right afterwards (into the next hop's frontier, and, in the
// whole-path call, into the batch's ID list), so the lane that writes a sample also inserts it into
// the hash tables of those de-duplications: they then start at their second pass.  The tables must
// be empty before the first insert; who empties which table when is the host runtime's business.
#pragma once
#include "compact_dev.hpp"
#include "philox.hpp"

namespace helios {

constexpr int kMaxFanout = 1024;
constexpr int kFoldItems = 8;                          // seeds per thread in the folded count pass
constexpr int kFoldMaxSeeds = kBlock * kFoldItems;     // 2048

struct HopArgs {
    const int64_t* offsets;
    const int32_t* indices;
    int64_t n_nodes;
    const int32_t* frontier;      // with fold and a recorded batch: unused, the frontier is the batch's seeds
    const int64_t* indptr;        // without fold: [n + 1], read
    Count n_frontier;
    int32_t fanout;
    int32_t hop;
    uint64_t rng_seed;
    const BatchVars* vars;        // nullable: rng_seed and the batch table come from here (recorded batch, not folded)
    int32_t* flat;
    int64_t flat_cap;
    ClearJob clear;               // a table emptied on the way (one that no kernel of this launch touches)
    InsertInto hop_table;         // de-duplication of this hop's samples; position = place in flat
    BatchTables batch;            // de-duplication of [seeds | flat_0 | ...]; position = place in that list
    int32_t* cat_out;             // with batch: receives [seeds | flat_0 | ...]
    int64_t n_seeds;
    Count prev_flat[HELIOS_KERNELS_MAX_SEG - 1];   // sizes of flat_0 .. flat_{hop-1}
    int32_t* err;
    // folded count pass (hop 0): the outputs that frontier_count_kernel would write
    bool fold;
    BatchFeed feed;               // feed.ring set: a recorded batch starts here
    int32_t* frontier_out;        // nullable: receives a copy of the frontier
    int64_t* indptr_out;          // [n + 1]
    int64_t* n_flat_dev;
    int64_t* size_out;            // nullable: [0] = frontier size, [1] = sample-list size
    Stamps stamps;
};

struct SampleTables {
    InsertInto hop;
    unsigned long long* batch_table;   // nullable
    uint32_t batch_mask;
    int32_t* batch_slot_of;
    int32_t* cat_out;
};

// flat[at] = id has just been written: the same lane inserts id into the tables of the de-duplications
// that follow.  cat_at is the place of the sample in [seeds | flat_0 | ...].
__device__ __forceinline__ void insert_sample(const SampleTables& t, int64_t n_nodes, int32_t* err, int32_t id, int64_t at,
                                              int64_t cat_at) {
    const bool node = id >= 0 && static_cast<int64_t>(id) < n_nodes;
    if (!node) raise(err, kErrData);
    if (t.hop.table)
        t.hop.slot_of[at] = node ? static_cast<int32_t>(table_insert(t.hop.table, t.hop.n_slots - 1, static_cast<uint32_t>(id),
                                                                     static_cast<uint32_t>(at)))
                                 : -1;
    if (t.batch_table) {
        t.cat_out[cat_at] = id;
        t.batch_slot_of[cat_at] = node ? static_cast<int32_t>(table_insert(t.batch_table, t.batch_mask, static_cast<uint32_t>(id),
                                                                           static_cast<uint32_t>(cat_at)))
                                       : -1;
    }
}

template <int G>
__device__ __forceinline__ void sample_role(const HopArgs& a, uint32_t rb, uint32_t nrb) {
    constexpr int kGroups = kBlock / G;          // nodes per workgroup and step
    __shared__ int32_t s_chosen[(G == kWave) ? kWavesPerBlock * kMaxFanout : 1];
    __shared__ uint32_t s_indptr[kFoldMaxSeeds + 1];
    __shared__ uint32_t s_wave[kWavesPerBlock + 1];

    stamp_start(a.stamps, rb);
    // A recorded batch starts at its folded hop 0: every workgroup reads the batch's variables from the slot of
    // the host's ring that the count of batches run so far selects, and the first leaves them in device memory
    // for the kernels that follow (the next kernel advances the count).
    const int32_t* frontier = a.frontier;
    uint64_t rng_seed = a.rng_seed;
    uint32_t which = a.batch.which;
    if (a.fold && a.feed.ring) {
        const BatchVars bv = a.feed.ring[*a.feed.batches_run % a.feed.ring_slots];
        if (rb == 0 && threadIdx.x == 0) *a.feed.vars_out = bv;
        frontier = bv.seeds;
        rng_seed = bv.rng_seed;
        which = bv.table % kBatchTables;
    } else if (a.vars) {
        rng_seed = a.vars->rng_seed;
        which = a.vars->table % kBatchTables;
    }
    for (uint32_t w = rb * kBlock + threadIdx.x; a.clear.table && w < a.clear.n_slots; w += nrb * kBlock)
        a.clear.table[w] = kEmptySlot;                    // side job of the role

    const int f = a.fanout;
    const int64_t n = a.n_frontier.get();
    if (a.fold) {
        // the count pass of the whole (short) frontier, in every workgroup
        const int64_t j0 = static_cast<int64_t>(threadIdx.x) * kFoldItems;
        int32_t v[kFoldItems];
        uint32_t cnt[kFoldItems];
#pragma unroll
        for (int k = 0; k < kFoldItems; ++k) v[k] = j0 + k < n ? frontier[j0 + k] : -1;
        uint32_t sum = 0;
#pragma unroll
        for (int k = 0; k < kFoldItems; ++k) {
            cnt[k] = j0 + k < n ? sample_count(a.offsets, a.n_nodes, v[k], f, a.err) : 0u;
            sum += cnt[k];
        }
        uint32_t total;
        uint32_t at = block_exclusive_scan(sum, s_wave, total);
#pragma unroll
        for (int k = 0; k < kFoldItems; ++k) {
            if (j0 + k < n) {
                s_indptr[j0 + k] = at;
                if (rb == 0) {
                    a.indptr_out[j0 + k] = at;
                    if (a.frontier_out && a.frontier_out != frontier) a.frontier_out[j0 + k] = v[k];
                }
            }
            at += cnt[k];
        }
        if (rb == 0 && threadIdx.x == 0) {
            a.indptr_out[n] = total;
            *a.n_flat_dev = total;
            if (a.size_out) { a.size_out[0] = n; a.size_out[1] = total; }
            if (static_cast<int64_t>(total) > a.flat_cap) raise(a.err, kErrCapacity);
        }
        __syncthreads();
    }

    const int group = threadIdx.x / G;
    const int l = threadIdx.x % G;
    SampleTables tabs{a.hop_table, nullptr, 0, nullptr, a.cat_out};
    if (a.batch.table0) {
        tabs.batch_table = a.batch.table(which);
        tabs.batch_mask = a.batch.n_slots - 1;
        tabs.batch_slot_of = a.batch.slot_of;
    }
    const bool seeds_too = tabs.batch_table && a.hop == 0;   // the frontier of hop 0 is the head of the batch's list
    int64_t cat_base = a.n_seeds;                // where flat_hop starts in [seeds | flat_0 | ...]
    for (int h = 0; h < a.hop; ++h) cat_base += a.prev_flat[h].get();
    if (f > 0 || seeds_too) {
        const int64_t step = static_cast<int64_t>(nrb) * kGroups;
        for (int64_t i = static_cast<int64_t>(rb) * kGroups + group; i < n; i += step) {
            // the lanes of a group read the same words
            const int32_t v = frontier[i];
            const int64_t out = a.fold ? static_cast<int64_t>(s_indptr[i]) : a.indptr[i];
            if (seeds_too && l == 0) {               // seed i is element i of the batch's list
                tabs.cat_out[i] = v;
                tabs.batch_slot_of[i] = v >= 0 && static_cast<int64_t>(v) < a.n_nodes
                                            ? static_cast<int32_t>(table_insert(tabs.batch_table, tabs.batch_mask,
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
                    insert_sample(tabs, a.n_nodes, a.err, id, out + l, cat_base + out + l);
                }
                continue;
            }
            if constexpr (G == kWave) {                           // fan-out above 64: one wave per node
                if (deg <= f) {
                    for (int k = l; k < deg; k += kWave)
                        if (out_ok && k < room) {
                            const int32_t id = a.indices[base + k];
                            a.flat[out + k] = id;
                            insert_sample(tabs, a.n_nodes, a.err, id, out + k, cat_base + out + k);
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
                            insert_sample(tabs, a.n_nodes, a.err, id, out + k, cat_base + out + k);
                        }
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            }
        }
    }
    stamp_end(a.stamps, rb, nrb);
}

inline int group_lanes(int32_t fanout) { return fanout <= 8 ? 8 : fanout <= 16 ? 16 : fanout <= 32 ? 32 : 64; }

// workgroups of a sampling role over a frontier of at most n_max nodes
inline unsigned sample_role_blocks(int32_t fanout, int64_t n_max) {
    const int64_t per_block = kBlock / group_lanes(fanout);
    int64_t blocks = (n_max + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxRoleBlocks) blocks = kMaxRoleBlocks;
    return static_cast<unsigned>(blocks);
}

}  // namespace helios
