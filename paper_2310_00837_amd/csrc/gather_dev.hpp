// Device code of the row copy: out[pos[k], :] = table[slot[k], :].
//
// A copy is a *role*: a range of the workgroups of some kernel launch.  The same loop is a kernel of
// its own (helios_gather, helios_gather_miss, helios_cache_fill, and the whole-path call in its
// split form) or shares a launch with other roles (the whole-path call: the host-tier copy of one
// stage rides on the sampling kernel of the next hop, and the last stage's rides beside the
// HBM-tier copy and the inverse pass), so that work that is bound by the host link runs beside
// work that is bound by latency or HBM bandwidth without a second stream.
//
// A group of L lanes owns one row and moves it as 16-byte pieces, so a row is read and written as
// whole contiguous lines; L is the smallest power of two that covers the row (at most a wave).
// Each group takes R consecutive list entries per step and issues all their loads before the first
// store.  A workgroup takes a run of consecutive entries per step and the workgroups take the runs
// in turn, so the rows being written at any moment are one dense window of the output that moves
// forward as workgroups are dispatched (list positions ascend): measured on this part, many
// short-lived workgroups on consecutive runs copy 8-10 % faster than a few thousand long-lived
// ones that stride over the whole list (6.0 against 5.5 TB/s for 2 KB rows; a plain copy behaves
// the same way).  The bounds of the list are read on the device.  Source and destination are
// touched once: non-temporal accesses keep them from displacing the graph and the cache map in L2.
#pragma once
#include "common.hpp"

namespace helios {

typedef uint32_t chunk16 __attribute__((ext_vector_type(4)));   // one 16-byte piece of a row

struct GatherArgs {
    const chunk16* table;
    const int32_t* pos;      // nullable: identity
    const int32_t* slot;
    const int64_t* begin;    // nullable (0): device-side first entry of the list to copy
    Count n;                 // one past the last entry
    int32_t chunks;          // 16-byte pieces per row
    chunk16* out;
    // Lists that a caller supplies are checked: a slot outside [0, table_rows) or a position outside
    // [0, out_rows) is reported (kErrData) and skipped.  table_rows < 0: the list is the library's own.
    int64_t table_rows, out_rows;
    int32_t* err;
    Stamps stamps;
};

__device__ __forceinline__ chunk16 load16(const chunk16* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store16(chunk16* p, const chunk16& v) { __builtin_nontemporal_store(v, p); }

// entry k of the list -> (source row, destination row); false if it must be skipped
__device__ __forceinline__ bool gather_entry(const GatherArgs& a, int64_t k, int64_t& s, int64_t& d) {
    s = a.slot[k];
    d = a.pos ? static_cast<int64_t>(a.pos[k]) : k;
    if (a.table_rows >= 0 && (s < 0 || s >= a.table_rows || d < 0 || d >= a.out_rows)) {
        raise(a.err, kErrData);
        return false;
    }
    return true;
}

// L lanes per row, CPL pieces per lane (L * CPL >= chunks), R rows per step; workgroup rb of nrb.
template <int L, int CPL, int R>
__device__ __forceinline__ void copy_rows(const GatherArgs& a, uint32_t rb, uint32_t nrb) {
    constexpr int kGroups = kBlock / L;
    stamp_start(a.stamps, rb);
    const int l = threadIdx.x % L;
    const int g = threadIdx.x / L;
    // Workgroup rb takes the runs rb, rb + nrb, ... of kGroups * R consecutive list entries: every workgroup gets
    // the same number of runs to within one, so all of them (for a far source: all the CUs whose requests fill
    // the link) stay busy until the list ends.
    const int64_t first = a.begin ? *a.begin : 0;
    const int64_t n = a.n.get();
    for (int64_t k0 = first + (static_cast<int64_t>(rb) * kGroups + g) * R; k0 < n; k0 += static_cast<int64_t>(nrb) * kGroups * R) {
        chunk16 v[R][CPL];
        int64_t dst[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t k = k0 + r;
            dst[r] = -1;
            int64_t s, d;
            if (k < n && gather_entry(a, k, s, d)) {
                dst[r] = d;
                const chunk16* src = a.table + s * a.chunks;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int idx = l + c * L;
                    if (idx < a.chunks) v[r][c] = load16(src + idx);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (dst[r] >= 0) {
                chunk16* o = a.out + dst[r] * a.chunks;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int idx = l + c * L;
                    if (idx < a.chunks) store16(o + idx, v[r][c]);
                }
            }
        }
    }
    stamp_end(a.stamps, rb, nrb);
}

// any row length: a wave per row, looping over the pieces
__device__ __forceinline__ void copy_rows_long(const GatherArgs& a, uint32_t rb, uint32_t nrb) {
    stamp_start(a.stamps, rb);
    const int64_t first = a.begin ? *a.begin : 0;
    const int64_t n = a.n.get();
    const int l = lane_id();
    const int64_t step = static_cast<int64_t>(nrb) * kWavesPerBlock;
    for (int64_t k = first + static_cast<int64_t>(rb) * kWavesPerBlock + wave_id(); k < n; k += step) {
        int64_t s, d;
        if (!gather_entry(a, k, s, d)) continue;
        const chunk16* src = a.table + s * a.chunks;
        chunk16* o = a.out + d * a.chunks;
        for (int idx = l; idx < a.chunks; idx += kWave) store16(o + idx, load16(src + idx));
    }
    stamp_end(a.stamps, rb, nrb);
}

// The shape of the copy loop for a row of `chunks` pieces.  far: the source is behind the host link (more
// rows in flight per group, because each takes microseconds); an HBM source is quickest with one row per group
// and step (measured: 2 KB rows 166 / 170 us with one / two rows, 512 B rows 181 / 186 / 193 us with 1 / 2 / 4).
#define HELIOS_COPY_SHAPE_SWITCH(chunks, far, CALL)                     \
    do {                                                                \
        const int c_ = (chunks);                                        \
        if (far) {                                                      \
            if (c_ <= 4) { CALL(4, 1, 2); }                             \
            else if (c_ <= 8) { CALL(8, 1, 2); }                        \
            else if (c_ <= 16) { CALL(16, 1, 2); }                      \
            else if (c_ <= 32) { CALL(32, 1, 4); }                      \
            else if (c_ <= 64) { CALL(64, 1, 2); }                      \
            else if (c_ <= 128) { CALL(64, 2, 2); }                     \
            else if (c_ <= 256) { CALL(64, 4, 1); }                     \
            else { CALL(0, 0, 0); }                                     \
        } else {                                                        \
            if (c_ <= 4) { CALL(4, 1, 1); }                             \
            else if (c_ <= 8) { CALL(8, 1, 1); }                        \
            else if (c_ <= 16) { CALL(16, 1, 1); }                      \
            else if (c_ <= 32) { CALL(32, 1, 1); }                      \
            else if (c_ <= 64) { CALL(64, 1, 1); }                      \
            else if (c_ <= 128) { CALL(64, 2, 1); }                     \
            else if (c_ <= 256) { CALL(64, 4, 1); }                     \
            else { CALL(0, 0, 0); }                                     \
        }                                                               \
    } while (0)

// rows per step of the far shape for a row that the near shape copies with L lanes and CPL pieces per lane
constexpr int far_rows_per_step(int L, int CPL) { return L == 0 ? 0 : L <= 16 ? 2 : L == 32 ? 4 : CPL >= 4 ? 1 : 2; }

// The copy with the shape chosen on the device: for roles that ride on another kernel (a host-link
// copy beside a sampling pass), where one instantiation has to serve every row size.  The loop is
// bound by the link, not by its instruction count.
__device__ __forceinline__ void copy_rows_any(const GatherArgs& a, uint32_t rb, uint32_t nrb, bool far) {
#define HELIOS_CALL_(L, CPL, R)                                         \
    if constexpr ((L) == 0) copy_rows_long(a, rb, nrb);                 \
    else copy_rows<(L) == 0 ? 64 : (L), (CPL) == 0 ? 1 : (CPL), (R) == 0 ? 1 : (R)>(a, rb, nrb)
    HELIOS_COPY_SHAPE_SWITCH(a.chunks, far, HELIOS_CALL_);
#undef HELIOS_CALL_
}

// Workgroups of a copy role over a list of at most n_max rows.  expected (0 = unknown): how many rows the
// list will probably hold (the count of the context's previous batch).
inline unsigned copy_role_blocks(int32_t chunks, bool far, int64_t n_max, unsigned limit /* 0 = default */, int64_t expected) {
    int rows_per_step = 1;
#define HELIOS_CALL_(L, CPL, R) rows_per_step = (L) == 0 ? kWavesPerBlock : (kBlock / ((L) == 0 ? 64 : (L))) * (R)
    HELIOS_COPY_SHAPE_SWITCH(chunks, far, HELIOS_CALL_);
#undef HELIOS_CALL_
    // far source: limited per CU by the requests a CU keeps in flight, not by waves, so one workgroup on each
    // of as many CUs as fill the link (more for short rows) and no more: every kernel launched on the GPU while
    // the link is saturated starts some microseconds late, the later the more link waves are in flight.
    // HBM source: best is one step per workgroup (see the head of this file), i.e. as many workgroups as the
    // list has runs, if the length of the list can be guessed (a workgroup that finds nothing to do costs
    // 0.2 ns, so a grid for the worst case would cost more than it gains); else a fixed few thousand.
    int64_t max_blocks = far ? (chunks <= 16 ? 128 : chunks <= 32 ? 44 : 32) : (n_max >= 500000 ? 8192 : 2048);
    if (!far && expected > 0) {
        max_blocks = (expected + expected / 16 + rows_per_step - 1) / rows_per_step;
        if (max_blocks < 256) max_blocks = 256;
    }
    if (limit > 0) max_blocks = limit;
    if (max_blocks > kMaxRoleBlocks) max_blocks = kMaxRoleBlocks;
    int64_t blocks = (n_max + rows_per_step - 1) / rows_per_step;
    if (blocks < 1) blocks = 1;
    if (blocks > max_blocks) blocks = max_blocks;
    return static_cast<unsigned>(blocks);
}

}  // namespace helios
