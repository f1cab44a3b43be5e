// helios_dedup_noalloc: the de-duplication of helios_dedup for callers that cannot allocate
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// helios_dedup takes its scratch (hash table, slot of every input, unique index of every first
// occurrence, scan status words, counters) from memory the context allocates and grows.  Here all
// of it lives in one file-scope device array of fixed size, so the call enqueues kernels and
// nothing else.  The array exists once per GPU the library runs on and keeps the contents of the
// last call: every call starts with a fill kernel that empties the table and zeroes the scan
// status, ticket and counters (a kernel, not a memset: a memset node in a captured graph is not
// reliable on this platform).  All calls on one GPU share the array, so calls that overlap on one
// GPU (two streams, two contexts, two host threads) race; callers serialise them.
#include "context.hpp"
#include "noalloc.hpp"

#include <mutex>

using namespace helios;

namespace {

constexpr int64_t kMaxIds = HELIOS_DEDUP_NOALLOC_MAX_IDS;
constexpr uint32_t kSlots = 2u * static_cast<uint32_t>(kMaxIds);              // power of two, twice the inputs
constexpr uint32_t kStride = static_cast<uint32_t>(kMaxIds / kTileItems + 2);   // tiles the status rows hold
static_assert((kSlots & (kSlots - 1)) == 0, "the table size must be a power of two");

// layout of the scratch array, in bytes (every part 256-byte aligned)
constexpr size_t kOffTable = 0;
constexpr size_t kOffSlotOf = kOffTable + sizeof(unsigned long long) * kSlots;
constexpr size_t kOffIndexOfFirst = kOffSlotOf + sizeof(int32_t) * kMaxIds;
constexpr size_t kOffStatus = kOffIndexOfFirst + sizeof(int32_t) * kMaxIds;
constexpr size_t kStatusBytes = (sizeof(unsigned long long) * 3 * kStride + 255) / 256 * 256;
constexpr size_t kOffSmall = kOffStatus + kStatusBytes;     // ticket (uint32) at +0, counters (int64[2]) at +64
constexpr size_t kSmallBytes = 256;
constexpr size_t kScratchBytes = kOffSmall + kSmallBytes;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_ptr[kMaxDevices] = {nullptr};     // device address of `scratch` on every GPU seen so far

// empties the table, zeroes the scan status words and the small block
__global__ __launch_bounds__(kBlock) void noalloc_reset_kernel(unsigned long long* table, uint32_t n_slots,
                                                               unsigned long long* zero_from, uint32_t n_zero_words) {
    const uint32_t step = gridDim.x * kBlock;
    for (uint32_t w = blockIdx.x * kBlock + threadIdx.x; w < n_slots; w += step) table[w] = kEmptySlot;
    for (uint32_t w = blockIdx.x * kBlock + threadIdx.x; w < n_zero_words; w += step) zero_from[w] = 0ull;
}

}  // namespace

namespace helios {

int noalloc_init(int device) {
    if (device < 0 || device >= kMaxDevices) return HELIOS_EINVAL;
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_ptr[device]) return HELIOS_OK;
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {     // the current device's copy of the array
        (void)hipGetLastError();
        return HELIOS_EHIP;
    }
    g_ptr[device] = static_cast<unsigned char*>(p);
    return HELIOS_OK;
}

}  // namespace helios

extern "C" int helios_dedup_noalloc(helios_ctx* c, const int32_t* ids, int64_t n_ids, int32_t* unique, int64_t unique_cap,
                                    int32_t* inverse, int64_t* n_unique) {
    if (!c) return HELIOS_EINVAL;
    if (!c->has_graph) return fail(c, HELIOS_ESTATE, "helios_dedup_noalloc before helios_csr_load");
    if (n_ids < 0 || unique_cap < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (n_ids > kMaxIds)
        return fail(c, HELIOS_EINVAL, "helios_dedup_noalloc handles at most %lld IDs per call (got %lld); use helios_dedup",
                    (long long)kMaxIds, (long long)n_ids);
    if ((n_ids > 0 && !ids) || (unique_cap > 0 && !unique)) return fail(c, HELIOS_EINVAL, "NULL pointer");
    unsigned char* base = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        base = c->device >= 0 && c->device < kMaxDevices ? g_ptr[c->device] : nullptr;
    }
    if (!base) return fail(c, HELIOS_ESTATE, "the static scratch of device %d was not set up by helios_create", c->device);
    DeviceGuard guard(c->device);
    unsigned long long* table = reinterpret_cast<unsigned long long*>(base + kOffTable);
    unsigned long long* status = reinterpret_cast<unsigned long long*>(base + kOffStatus);
    uint32_t* ticket = reinterpret_cast<uint32_t*>(base + kOffSmall);
    int64_t* counters = reinterpret_cast<int64_t*>(base + kOffSmall + 64);
    // a table no larger than this call needs: cheaper to empty, and it stays in cache
    uint32_t slots = 1024;
    while (static_cast<int64_t>(slots) < 2 * n_ids) slots <<= 1;
    const DedupScratch s{table, slots, reinterpret_cast<int32_t*>(base + kOffSlotOf),
                         reinterpret_cast<int32_t*>(base + kOffIndexOfFirst)};
    const uint32_t zero_words = static_cast<uint32_t>((kStatusBytes + kSmallBytes) / sizeof(unsigned long long));
    unsigned reset_blocks = (slots + kBlock * 16 - 1) / (kBlock * 16);
    reset_blocks = reset_blocks < 1 ? 1 : reset_blocks > 1024 ? 1024 : reset_blocks;
    hipLaunchKernelGGL(noalloc_reset_kernel, dim3(reset_blocks), dim3(kBlock), 0, c->stream, table, slots, status, zero_words);
    HIP_TRY(c, hipGetLastError());
    // the status words are zero, so any epoch but zero reads them as unpublished; the same value every
    // call keeps a captured call replayable
    const ScanState scan{status, ticket, kStride, 1u, nullptr};
    const Count n{nullptr, n_ids};
    HIP_TRY(c, launch_dedup_insert(c->stream, ids, n, n_ids, c->g.n_nodes, s, c->err));
    CompactArgs a{};
    a.ids = ids;
    a.lens.n_seg = 1;
    a.lens.first_here = 0;
    a.lens.len[0] = n;
    a.n_max = n_ids;
    a.n_total_dev = counters + 0;
    a.s = s;
    a.unique = unique;
    a.unique_cap = unique_cap;
    a.last = true;
    a.n_unique_dev = counters + 1;
    a.n_unique_out = n_unique;
    a.scan = scan;
    a.err = c->err;
    HIP_TRY(c, launch_dedup_compact_plain(c->stream, a, n_ids));
    if (inverse) {
        const InverseArgs inv{Count{counters + 0, n_ids}, s, BatchTables{nullptr, 0, nullptr, 0, 0, nullptr, 0}, nullptr, inverse,
                              Stamps{nullptr}};
        HIP_TRY(c, launch_dedup_inverse(c->stream, inv, n_ids));
    }
    return HELIOS_OK;
}
