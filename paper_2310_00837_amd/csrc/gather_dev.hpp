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
// Each group takes R list entries per step and issues all their loads before the first store.  The
// groups of the role share the list evenly (entry k belongs to group k mod groups) and the bounds
// of the list are read on the device.  Source and destination are touched once: non-temporal
// accesses keep them from displacing the graph and the cache map in L2.
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
    // Group j of the role takes the list entries j, j + groups, j + 2 * groups, ..., R of them per step: every
    // group gets the same number of rows to within one, so all workgroups (for a far source: all the CUs
    // whose requests fill the link) stay busy until the list ends.
    const int64_t groups = static_cast<int64_t>(nrb) * kGroups;
    const int64_t first = a.begin ? *a.begin : 0;
    const int64_t n = a.n.get();
    for (int64_t k0 = first + static_cast<int64_t>(rb) * kGroups + g; k0 < n; k0 += groups * R) {
        chunk16 v[R][CPL];
        int64_t dst[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t k = k0 + r * groups;
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
// rows in flight per group, because each takes microseconds).
#define HELIOS_COPY_SHAPE_SWITCH(chunks, far, CALL)                     \
    do {                                                                \
        const int c_ = (chunks);                                        \
        if (c_ <= 4) { CALL(4, 1, 2); }                                 \
        else if (c_ <= 8) { CALL(8, 1, 2); }                            \
        else if (c_ <= 16) { CALL(16, 1, 2); }                          \
        else if (c_ <= 32 && (far)) { CALL(32, 1, 4); }                 \
        else if (c_ <= 32) { CALL(32, 1, 1); }                          \
        else if (c_ <= 64) { CALL(64, 1, 2); }                          \
        else if (c_ <= 128) { CALL(64, 2, 2); }                         \
        else if (c_ <= 256) { CALL(64, 4, 1); }                         \
        else { CALL(0, 0, 0); }                                         \
    } while (0)

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

// workgroups of a copy role over a list of at most n_max rows
inline unsigned copy_role_blocks(int32_t chunks, bool far, int64_t n_max, unsigned limit /* 0 = default */) {
    // far source: limited per CU by the requests a CU keeps in flight, not by waves, so one workgroup on each
    // of as many CUs as fill the link (more for short rows) and no more: every kernel launched on the GPU while
    // the link is saturated starts some microseconds late, the later the more link waves are in flight.
    // HBM source: 8192 workgroups (four rounds of what the chip holds) balance long lists best; lists that can
    // hold at most a few hundred thousand rows are quicker with the 2048 that are resident at once.
    unsigned max_blocks = far ? (chunks <= 16 ? 128u : chunks <= 32 ? 44u : 32u) : (n_max >= 500000 ? kMaxRoleBlocks : 2048u);
    if (limit > 0) max_blocks = limit < kMaxRoleBlocks ? limit : kMaxRoleBlocks;
    int rows_per_step = 1;
#define HELIOS_CALL_(L, CPL, R) rows_per_step = (L) == 0 ? kWavesPerBlock : (kBlock / ((L) == 0 ? 64 : (L))) * (R)
    HELIOS_COPY_SHAPE_SWITCH(chunks, far, HELIOS_CALL_);
#undef HELIOS_CALL_
    int64_t blocks = (n_max + rows_per_step - 1) / rows_per_step;
    if (blocks < 1) blocks = 1;
    if (blocks > max_blocks) blocks = max_blocks;
    return static_cast<unsigned>(blocks);
}

}  // namespace helios
