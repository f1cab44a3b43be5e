// Asynchronous miss service in the shape of the paper's GPU-initiated IO stack
// (Sec. 3.1): two decoupled kernels, command submission (Sec. 3.1.1) and
// completion handling (Sec. 3.1.2), with the device in between played by host
// threads that serve the storage stand-in.
//
//   submit    one thread per miss (several misses per thread): builds the
//             command {storage row, staging row} and writes it to one of
//             n_queues submission queues in pinned host memory; when all
//             commands are written, the last workgroup rings every queue's
//             doorbell once (doorbell batching): {round, number of commands}.
//   service   (host threads, the stand-in for the SSDs' controllers) a thread
//             owns the queues t, t + T, ...; it waits for a queue's doorbell,
//             copies every command's row from the stand-in table to the staging
//             buffer (pinned host memory, the temporary IO buffer) and posts a
//             completion entry {round, command index} to the queue's completion
//             queue.  Commands of a queue complete in either direction, so the
//             order of completions differs from the order of submission.
//   complete  a wave owns several completion queues.  It polls up to 64
//             entries of a queue with one load, takes the leading ones that
//             carry this round's number, and all its lanes move those rows from
//             the staging buffer to their rows of the feature buffer.  A wave
//             that sees no progress for the time limit reports an error and
//             ends: no wave waits for ever.
// Nothing on the GPU waits between submit and complete: the kernels of the
// cached tiers run there, and by the time the completion kernel starts most
// entries are posted.
//
// A round is one submit/complete pair; the queues are reused from their first
// entry in every round, and the round number in doorbells and completion
// entries tells new entries from old ones (as the phase bit of an NVMe queue
// does).  Stream order keeps a round's submission behind the completion kernel
// of the round before it.
#include "missq.hpp"

#include <atomic>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

using namespace helios;

namespace helios {

struct MissqView {
    unsigned long long* sq;         // pinned [n_queues][depth]: {staging row : 32 | storage row : 32}
    unsigned long long* doorbell;   // pinned [n_queues]: {round : 32 | commands : 32}
    unsigned long long* cq;         // pinned [n_queues][depth]: {round : 32 | command index : 32}
    unsigned char* staging;         // pinned [n_queues * depth][row_bytes]
    int32_t* cmd_pos;               // device [n_queues * depth]: the row of `out` a command's data goes to
    uint32_t* arrivals;             // device: workgroups of the submission kernel that have finished
    int64_t* n_cmds;                // device: commands of the current round
    int32_t n_queues, depth;
};

}  // namespace helios

struct helios_missq {
    helios_ctx* ctx = nullptr;
    MissqView v{};
    int32_t n_threads = 0;
    int32_t row_bytes = 0;
    const unsigned char* standin = nullptr;
    int64_t standin_rows = 0;
    uint64_t cache_generation = 0;

    // host API thread only
    uint32_t round = 0;             // the last round opened
    bool open = false;              // that round's completion kernel has not been enqueued yet

    std::mutex mu;
    std::condition_variable cv;
    uint32_t announced = 0;         // guarded by mu: rounds the service threads may wait for
    std::atomic<bool> stop{false};
    std::atomic<bool> faulted{false};
    std::atomic<int64_t> commands_served{0}, rounds_served{0};     // rounds: summed over the threads
    std::vector<std::thread> threads;
};

namespace {

typedef uint32_t chunk16 __attribute__((ext_vector_type(4)));

constexpr int kCommandsPerThread = 4;
constexpr int kCopyUnroll = 4;           // 16-byte loads a lane has in flight while it moves completed rows

__device__ __forceinline__ int64_t commands_of_queue(int64_t n, int64_t per_q, int q) {
    const int64_t rest = n - static_cast<int64_t>(q) * per_q;
    return rest <= 0 ? 0 : rest < per_q ? rest : per_q;
}

struct SubmitArgs {
    MissqView q;
    const int32_t* miss_pos;
    const int32_t* miss_slot;
    int64_t standin_rows, out_rows;   // a command outside either is reported and served into nowhere
    Count n;
    uint32_t round;
    const BatchVars* vars;          // nullable: the round is vars->io_round (recorded batch)
    int32_t* err;
};

// Queue q takes the commands [q * per_q, (q + 1) * per_q) of the miss list, so a wave writes 64
// consecutive 8-byte commands of one queue.
__global__ __launch_bounds__(kBlock) void missq_submit_kernel(SubmitArgs a) {
    __shared__ uint32_t s_last;
    const int64_t cap = static_cast<int64_t>(a.q.n_queues) * a.q.depth;
    int64_t n = a.n.get();
    if (n > cap) {
        if (blockIdx.x == 0 && threadIdx.x == 0) raise(a.err, kErrCapacity);
        n = cap;
    }
    if (n > 0 && a.standin_rows <= 0) {          // every node is cached: nothing can miss, the list is wrong
        if (blockIdx.x == 0 && threadIdx.x == 0) raise(a.err, kErrData);
        n = 0;
    }
    const uint32_t round = a.vars ? a.vars->io_round : a.round;
    const int64_t per_q = (n + a.q.n_queues - 1) / a.q.n_queues;
    const int64_t step = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; j < n; j += step) {
        const int64_t q = j / per_q;
        const int64_t at = q * a.q.depth + (j - q * per_q);
        int32_t pos = a.miss_pos[j], slot = a.miss_slot[j];
        if (pos < 0 || pos >= a.out_rows || slot < 0 || slot >= a.standin_rows) {
            // the caller's list is wrong here: the command still takes its place in the queue (the counts per queue
            // are fixed), but it reads row 0 and its data goes nowhere
            raise(a.err, kErrData);
            pos = -1;
            slot = 0;
        }
        a.q.cmd_pos[at] = pos;
        a.q.sq[at] = (static_cast<unsigned long long>(at) << 32) | static_cast<uint32_t>(slot);
    }
    __threadfence_system();                    // the commands are in host memory before this workgroup counts as done
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t arrived = atomicAdd(a.q.arrivals, 1u);
        s_last = arrived == gridDim.x - 1;
        if (s_last) atomicExch(a.q.arrivals, 0u);          // ready for the next launch
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence_system();
    if (threadIdx.x == 0) *a.q.n_cmds = n;
    for (int q = threadIdx.x; q < a.q.n_queues; q += kBlock) {
        const unsigned long long bell =
            (static_cast<unsigned long long>(round) << 32) | static_cast<uint32_t>(commands_of_queue(n, per_q, q));
        __hip_atomic_store(a.q.doorbell + q, bell, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

struct CompleteArgs {
    MissqView q;
    chunk16* out;
    int32_t chunks;                 // 16-byte pieces per row
    uint32_t round;
    unsigned long long timeout_ticks;
    int n_waves;
    int32_t* err;
};

__global__ __launch_bounds__(kBlock) void missq_complete_kernel(CompleteArgs a) {
    const int l = lane_id();
    const int w = blockIdx.x * kWavesPerBlock + wave_id();
    const int W = a.n_waves;
    if (w >= W) return;
    const int64_t cap = static_cast<int64_t>(a.q.n_queues) * a.q.depth;
    int64_t n = *a.q.n_cmds;
    n = n < 0 ? 0 : n > cap ? cap : n;
    if (n == 0) return;
    const int64_t per_q = (n + a.q.n_queues - 1) / a.q.n_queues;

    // lane k keeps the state of this wave's k-th queue, w + k * W (the launcher keeps k below 64)
    const int my_q = w + l * W;
    const int my_count = my_q < a.q.n_queues ? static_cast<int>(commands_of_queue(n, per_q, my_q)) : 0;
    int my_head = 0;
    int remaining = static_cast<int>(wave_sum(static_cast<uint32_t>(my_count)));
    const chunk16* staging = reinterpret_cast<const chunk16*>(a.q.staging);
    unsigned long long last_progress = wall_clock64();
    int idle_sleeps = 1;            // polls over the link get rarer while nothing arrives

    while (remaining > 0) {
        bool progress = false;
        for (int k = 0; w + k * W < a.q.n_queues; ++k) {
            const int q = w + k * W;
            const int count = __shfl(my_count, k, kWave), head = __shfl(my_head, k, kWave);
            if (head >= count) continue;                                   // uniform over the wave
            const int64_t base = static_cast<int64_t>(q) * a.q.depth;
            // the leader polls the entry the queue is waiting for; only when that one is posted does the wave
            // read the 64 entries from there on (an idle poll costs the host one cache line, not eight)
            unsigned long long first = 0;
            if (l == 0) first = __hip_atomic_load(a.q.cq + base + head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            first = __shfl(first, 0, kWave);
            if (static_cast<uint32_t>(first >> 32) != a.round) continue;
            const int idx = head + l;
            unsigned long long e = 0;
            if (idx < count) e = __hip_atomic_load(a.q.cq + base + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            const bool posted = idx < count && static_cast<uint32_t>(e >> 32) == a.round;
            const unsigned long long mask = __ballot(posted);
            const int lead = mask == ~0ull ? kWave : __builtin_ctzll(~mask);   // entries are posted in order
            if (lead == 0) continue;
            __threadfence_system();                // the staging rows are read after their completion entries
            const uint32_t cid = static_cast<uint32_t>(e);                 // lane r: command of the r-th new entry
            if (l < lead && cid >= static_cast<uint32_t>(count)) raise(a.err, kErrInternal);
            const int total = lead * a.chunks;
            for (int t0 = 0; t0 < total; t0 += kWave * kCopyUnroll) {
                chunk16 v[kCopyUnroll];
                int64_t dst[kCopyUnroll];
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u) {
                    const int t = t0 + u * kWave + l;
                    const bool valid = t < total;
                    const int r = valid ? t / a.chunks : 0;
                    const int piece = t - r * a.chunks;
                    const uint32_t c_r = __shfl(cid, r, kWave);
                    dst[u] = -1;
                    if (valid && c_r < static_cast<uint32_t>(count)) {
                        const int64_t row = base + c_r;
                        const int64_t to = a.q.cmd_pos[row];       // negative: a command the submission refused
                        if (to >= 0) {
                            v[u] = __builtin_nontemporal_load(staging + row * a.chunks + piece);
                            dst[u] = to * a.chunks + piece;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kCopyUnroll; ++u)
                    if (dst[u] >= 0) __builtin_nontemporal_store(v[u], a.out + dst[u]);
            }
            if (l == k) my_head += lead;
            remaining -= lead;
            progress = true;
        }
        if (progress) {
            last_progress = wall_clock64();
            idle_sleeps = 1;
        } else {
            if (wall_clock64() - last_progress > a.timeout_ticks) {        // the device has stopped answering
                if (l == 0) raise(a.err, kErrInternal);
                return;
            }
            for (int z = 0; z < idle_sleeps; ++z) __builtin_amdgcn_s_sleep(127);     // ~3 us each
            if (idle_sleeps < 4) idle_sleeps += 1;
        }
    }
}

inline void cpu_relax() {
#if !defined(__HIP_DEVICE_COMPILE__)
    __asm__ __volatile__("pause" ::: "memory");
#endif
}

// One queue's commands of one round: stand-in row -> staging row, then the completion entry.
void serve_queue(helios_missq* m, int q, uint32_t round, uint32_t count) {
    const MissqView& v = m->v;
    if (count > static_cast<uint32_t>(v.depth)) {
        m->faulted.store(true);
        return;
    }
    const size_t rb = static_cast<size_t>(m->row_bytes);
    const int64_t base = static_cast<int64_t>(q) * v.depth;
    const int64_t n_staging = static_cast<int64_t>(v.n_queues) * v.depth;
    const bool forward = ((round + static_cast<uint32_t>(q)) & 1u) == 0;
    constexpr uint32_t kAhead = 6;
    constexpr uint32_t kPostBatch = 8;         // completion entries of one cache line are posted together
    unsigned long long entry[kPostBatch];
    uint32_t held = 0;                         // copied, not yet posted; their entries go to cq[p - held, p)
    auto post = [&](uint32_t p_end) {
        for (uint32_t b = 0; b < held; ++b) __atomic_store_n(v.cq + base + (p_end - held + b), entry[b], __ATOMIC_RELEASE);
        held = 0;
    };
    for (uint32_t p = 0; p < count; ++p) {
        if (p + kAhead < count) {              // the rows are at random places of a large table
            const uint32_t i2 = forward ? p + kAhead : count - 1 - (p + kAhead);
            const uint32_t s2 = static_cast<uint32_t>(__atomic_load_n(v.sq + base + i2, __ATOMIC_RELAXED));
            if (static_cast<int64_t>(s2) < m->standin_rows) {
                const unsigned char* r2 = m->standin + static_cast<size_t>(s2) * rb;
                for (size_t b = 0; b < rb && b < 512; b += 64) __builtin_prefetch(r2 + b, 0, 0);
            }
        }
        const uint32_t i = forward ? p : count - 1 - p;
        const unsigned long long cmd = __atomic_load_n(v.sq + base + i, __ATOMIC_RELAXED);
        const int64_t slot = static_cast<uint32_t>(cmd), row = static_cast<int64_t>(cmd >> 32);
        if (slot >= m->standin_rows || row >= n_staging) {      // no completion entry: the completion kernel reports it
            m->faulted.store(true);
            post(p);
            return;
        }
        memcpy(v.staging + static_cast<size_t>(row) * rb, m->standin + static_cast<size_t>(slot) * rb, rb);
        entry[held++] = (static_cast<unsigned long long>(round) << 32) | i;
        if (held == kPostBatch || ((p + 1) & (kPostBatch - 1)) == 0) post(p + 1);
    }
    post(count);
    m->commands_served.fetch_add(count, std::memory_order_relaxed);
}

void service_thread(helios_missq* m, int t) {
    std::vector<int> mine;
    for (int q = t; q < m->v.n_queues; q += m->n_threads) mine.push_back(q);
    std::vector<char> done(mine.size());
    uint32_t served = 0;
    for (;;) {
        {
            std::unique_lock<std::mutex> lk(m->mu);
            m->cv.wait(lk, [&] { return m->stop.load() || m->announced != served; });
            if (m->stop.load()) return;
        }
        const uint32_t round = served + 1;
        std::fill(done.begin(), done.end(), 0);
        size_t left = mine.size();
        unsigned idle = 0;
        while (left > 0) {
            bool progress = false;
            for (size_t k = 0; k < mine.size(); ++k) {
                if (done[k]) continue;
                const unsigned long long bell = __atomic_load_n(m->v.doorbell + mine[k], __ATOMIC_ACQUIRE);
                const int32_t ahead = static_cast<int32_t>(static_cast<uint32_t>(bell >> 32) - round);
                if (ahead < 0) continue;                       // not rung yet
                // A doorbell of a later round: this round's ring has been overwritten, which the GPU only
                // does once the round is complete, so the round had no commands on this queue.
                if (ahead == 0) serve_queue(m, mine[k], round, static_cast<uint32_t>(bell));
                done[k] = 1;
                left -= 1;
                progress = true;
            }
            if (!progress) {
                if (m->stop.load()) return;
                if (++idle < 2048) {
                    cpu_relax();
                } else {
                    idle = 0;
                    std::this_thread::yield();
                }
            }
        }
        served = round;
        m->rounds_served.fetch_add(1, std::memory_order_relaxed);
    }
}

// Reads one byte of every page of the stand-in table from the host.  Pinned memory that only the GPU
// has written so far is resident but not yet in this process's page table; without this pass every
// first read of a page by a service thread would take a page fault (microseconds, against the tenth
// of a microsecond the row copy itself takes).
void touch_pages(const unsigned char* p, size_t bytes) {
    constexpr size_t kPage = 4096;
    const unsigned n_threads = 8;
    const size_t pages = (bytes + kPage - 1) / kPage;
    std::vector<std::thread> ts;
    std::atomic<unsigned> sink{0};
    for (unsigned t = 0; t < n_threads; ++t)
        ts.emplace_back([=, &sink] {
            unsigned acc = 0;
            for (size_t pg = pages * t / n_threads; pg < pages * (t + 1) / n_threads; ++pg)
                acc += *reinterpret_cast<const volatile unsigned char*>(p + pg * kPage);
            sink.fetch_add(acc, std::memory_order_relaxed);
        });
    for (std::thread& th : ts) th.join();
}

void stop_threads(helios_missq* m) {
    {
        std::lock_guard<std::mutex> lk(m->mu);
        m->stop.store(true);
    }
    m->cv.notify_all();
    for (std::thread& th : m->threads)
        if (th.joinable()) th.join();
    m->threads.clear();
}

void free_buffers(helios_missq* m) {
    if (m->v.sq) (void)hipHostFree(m->v.sq);
    if (m->v.doorbell) (void)hipHostFree(m->v.doorbell);
    if (m->v.cq) (void)hipHostFree(m->v.cq);
    if (m->v.staging) (void)hipHostFree(m->v.staging);
    (void)hipFree(m->v.cmd_pos);
    (void)hipFree(m->v.n_cmds);
    m->v = MissqView{};
}

void announce(helios_missq* m) {
    {
        std::lock_guard<std::mutex> lk(m->mu);
        m->announced = m->round;
    }
    m->cv.notify_all();
}

int launch_submit(helios_ctx* c, helios_missq* m, const int32_t* miss_pos, const int32_t* miss_slot, Count n,
                  int64_t n_max, int64_t out_rows, uint32_t round, const BatchVars* vars) {
    SubmitArgs a{m->v, miss_pos, miss_slot, m->standin_rows, out_rows, n, round, vars, c->err_now};
    int64_t blocks = (n_max + kBlock * kCommandsPerThread - 1) / (kBlock * kCommandsPerThread);
    blocks = blocks < 1 ? 1 : blocks > 16 ? 16 : blocks;     // every workgroup ends with a system-scope fence and a ticket: few of them
    hipLaunchKernelGGL(missq_submit_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, c->stream, a);
    HIP_TRY(c, hipGetLastError());
    return HELIOS_OK;
}

}  // namespace

namespace helios {

bool missq_matches_cache(const helios_ctx* c, const helios_missq* q) {
    return q && q->ctx == c && c->has_cache && q->cache_generation == c->cache_generation;
}


int missq_next_round(helios_ctx* c, helios_missq* q, uint32_t* round_out) {
    if (!missq_matches_cache(c, q)) return fail(c, HELIOS_ESTATE, "the miss queue was made for another cache; create it again");
    if (q->open) return fail(c, HELIOS_ESTATE, "the previous round of the miss queue has not been completed (helios_missq_complete)");
    *round_out = q->round + 1;
    return HELIOS_OK;
}

void missq_commit_round(helios_missq* q, uint32_t round) {
    q->round = round;
    q->open = true;
    announce(q);
}

int missq_submit_from_batch(helios_ctx* c, const int32_t* miss_pos, const int32_t* miss_slot, Count n_miss,
                            int64_t n_miss_max, int64_t out_rows) {
    helios_missq* q = c->missq;
    if (c->recording) {             // the round is opened at every launch of the recording
        if (!missq_matches_cache(c, q)) return fail(c, HELIOS_ESTATE, "the miss queue was made for another cache; create it again");
        return launch_submit(c, q, miss_pos, miss_slot, n_miss, n_miss_max, out_rows, 0, c->vars);
    }
    uint32_t round = 0;
    int rc = missq_next_round(c, q, &round);
    if (rc) return rc;
    rc = launch_submit(c, q, miss_pos, miss_slot, n_miss, n_miss_max, out_rows, round, nullptr);
    if (rc == HELIOS_OK) missq_commit_round(q, round);
    return rc;
}

}  // namespace helios

extern "C" {

int helios_missq_create(helios_ctx* c, int32_t n_queues, int32_t queue_depth, int32_t n_service_threads,
                        helios_missq** out) {
    if (!c || !out) return HELIOS_EINVAL;
    *out = nullptr;
    if (!c->has_cache) return fail(c, HELIOS_ESTATE, "helios_missq_create before helios_cache_build");
    if (n_queues < 1 || n_queues > 4096 || queue_depth < 1 || queue_depth > (1 << 20) || n_service_threads < 0 ||
        n_service_threads > 64)
        return fail(c, HELIOS_EINVAL, "helios_missq_create: 1..4096 queues of 1..2^20 entries, 0..64 threads");
    const int64_t entries = static_cast<int64_t>(n_queues) * queue_depth;
    if (entries > (1ll << 26) || entries * c->row_bytes > (8ll << 30))
        return fail(c, HELIOS_EINVAL, "helios_missq_create: the staging buffer would exceed 8 GiB");
    const int64_t standin_rows = c->g.n_nodes - c->n_hbm - c->n_host;
    if (standin_rows > 0 && !c->standin_table) return fail(c, HELIOS_ESTATE, "no stand-in table was given to helios_cache_build");
    DeviceGuard guard(c->device);
    helios_missq* m = new helios_missq();
    m->ctx = c;
    m->n_threads = n_service_threads;
    m->row_bytes = c->row_bytes;
    m->standin = static_cast<const unsigned char*>(c->standin_table);
    m->standin_rows = standin_rows;
    m->cache_generation = c->cache_generation;
    m->v.n_queues = n_queues;
    m->v.depth = queue_depth;
    const unsigned flags = hipHostMallocMapped | hipHostMallocPortable | hipHostMallocCoherent;
    const size_t q_bytes = sizeof(unsigned long long) * static_cast<size_t>(entries);
    bool ok = hipHostMalloc(reinterpret_cast<void**>(&m->v.sq), q_bytes, flags) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&m->v.cq), q_bytes, flags) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&m->v.doorbell), sizeof(unsigned long long) * n_queues, flags) == hipSuccess &&
              hipHostMalloc(reinterpret_cast<void**>(&m->v.staging), static_cast<size_t>(entries) * c->row_bytes, flags) == hipSuccess &&
              hipMalloc(&m->v.cmd_pos, sizeof(int32_t) * static_cast<size_t>(entries)) == hipSuccess &&
              hipMalloc(&m->v.n_cmds, 64) == hipSuccess;
    if (ok) {
        memset(m->v.sq, 0, q_bytes);
        memset(m->v.cq, 0, q_bytes);
        memset(m->v.doorbell, 0, sizeof(unsigned long long) * n_queues);
        m->v.arrivals = reinterpret_cast<uint32_t*>(m->v.n_cmds + 1);
        ok = hipMemsetAsync(m->v.n_cmds, 0, 64, c->stream) == hipSuccess && hipStreamSynchronize(c->stream) == hipSuccess;
    }
    if (!ok) {
        const hipError_t e = hipGetLastError();
        free_buffers(m);
        delete m;
        return fail(c, HELIOS_EHIP, "helios_missq_create: %s", hipGetErrorString(e));
    }
    if (n_service_threads > 0 && standin_rows > 0) touch_pages(m->standin, static_cast<size_t>(standin_rows) * c->row_bytes);
    for (int t = 0; t < n_service_threads; ++t) m->threads.emplace_back(service_thread, m, t);
    c->n_children += 1;
    *out = m;
    return HELIOS_OK;
}

int helios_missq_destroy(helios_missq* m) {
    if (!m) return HELIOS_EINVAL;
    helios_ctx* c = m->ctx;
    DeviceGuard guard(c->device);
    (void)hipStreamSynchronize(c->stream);
    if (c->missq == m) c->missq = nullptr;
    c->n_children -= 1;
    stop_threads(m);
    free_buffers(m);
    delete m;
    return HELIOS_OK;
}

int helios_missq_attach(helios_ctx* c, helios_missq* m) {
    if (!c) return HELIOS_EINVAL;
    if (c->recording) return fail(c, HELIOS_ESTATE, "a batch is being recorded");
    if (m && m->ctx != c) return fail(c, HELIOS_EINVAL, "the miss queue belongs to another context");
    if (m && !missq_matches_cache(c, m)) return fail(c, HELIOS_ESTATE, "the miss queue was made for another cache; create it again");
    c->missq = m;
    return HELIOS_OK;
}

int helios_missq_submit(helios_missq* m, const int32_t* miss_pos, const int32_t* miss_slot, int64_t n_miss_max,
                        const int64_t* n_miss_dev, int64_t out_rows) {
    if (!m) return HELIOS_EINVAL;
    helios_ctx* c = m->ctx;
    if (n_miss_max < 0 || out_rows < 0) return fail(c, HELIOS_EINVAL, "negative size");
    if (n_miss_max > 0 && (!miss_pos || !miss_slot)) return fail(c, HELIOS_EINVAL, "NULL pointer");
    DeviceGuard guard(c->device);
    uint32_t round = 0;
    int rc = missq_next_round(c, m, &round);
    if (rc) return rc;
    rc = launch_submit(c, m, miss_pos, miss_slot, Count{n_miss_dev, n_miss_max}, n_miss_max, out_rows, round, nullptr);
    if (rc == HELIOS_OK) missq_commit_round(m, round);
    return rc;
}

int helios_missq_complete(helios_missq* m, void* out) {
    if (!m) return HELIOS_EINVAL;
    helios_ctx* c = m->ctx;
    if (!m->open) return fail(c, HELIOS_ESTATE, "helios_missq_complete without a submitted round");
    if (!out) return fail(c, HELIOS_EINVAL, "NULL pointer");
    DeviceGuard guard(c->device);
    int waves = c->missq_waves ? static_cast<int>(c->missq_waves) : 256;
    const int least = (m->v.n_queues + kWave - 1) / kWave;         // a wave keeps at most 64 queues
    waves = waves < least ? least : waves;
    waves = waves > m->v.n_queues ? m->v.n_queues : waves;
    CompleteArgs a{m->v, static_cast<chunk16*>(out), m->row_bytes / 16, m->round,
                   static_cast<unsigned long long>(static_cast<double>(c->missq_timeout_us) * c->clock_khz / 1000.0),
                   waves, c->err};
    hipLaunchKernelGGL(missq_complete_kernel, dim3(static_cast<unsigned>((waves + kWavesPerBlock - 1) / kWavesPerBlock)),
                       dim3(kBlock), 0, c->stream, a);
    HIP_TRY(c, hipGetLastError());
    m->open = false;
    return HELIOS_OK;
}

int helios_missq_faulted(const helios_missq* m) { return m && m->faulted.load() ? 1 : 0; }

int helios_missq_counters(const helios_missq* m, int64_t* out) {
    if (!m || !out) return HELIOS_EINVAL;
    out[0] = m->round;
    out[1] = m->n_threads > 0 ? m->rounds_served.load() / m->n_threads : 0;
    out[2] = m->commands_served.load();
    return HELIOS_OK;
}

}  // extern "C"
