/*
 * helios.h -- C ABI of the MI355X (gfx950) library for the mini-batch
 * preparation path of Helios (arXiv 2310.00837): k-hop uniform neighbour
 * sampling over a CSR graph, de-duplication of the sampled IDs, lookup in a
 * GPU-managed two-tier feature cache, gather of feature rows and the miss
 * list for the storage tier.
 *
 * General rules
 * -------------
 *  - Every function returns a helios_status.  Errors that the host can see
 *    (null pointer, negative size, call order) are returned at once and
 *    nothing is launched.  helios_last_error() gives a text for the last one.
 *  - All work is asynchronous on the context's HIP stream.  Errors that only
 *    the device can see (a node ID outside [0, N), an output that does not
 *    fit its capacity) are recorded on the device and returned by the next
 *    helios_sync(); nothing is written beyond a capacity.
 *  - "device" pointers are HIP device memory.  "device-accessible" pointers
 *    may be device memory or pinned, GPU-mapped host memory (hipHostMalloc);
 *    their contents are valid after helios_sync().
 *  - "host" pointers are ordinary host memory, read during the call only.
 *  - All caller buffers are BORROWED: the library never frees or reallocates
 *    them.  Graph and cache tables must outlive the context (or the next
 *    helios_csr_load / helios_cache_build).
 *  - Node IDs, positions and slots are int32; edge offsets and counts int64.
 *    A single call handles fewer than 2^31 IDs; a CSR row holds fewer than
 *    2^31 entries.
 *  - The library allocates its own scratch (hash tables, scan state, position
 *    lists) and grows it when a call needs more than any call before;
 *    helios_reserve() does that ahead of time, after which calls of that size
 *    allocate nothing.
 *  - One context serves one stream; calls on one context must not overlap
 *    from several host threads.
 */
#ifndef HELIOS_H
#define HELIOS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct helios_ctx helios_ctx;

typedef enum {
    HELIOS_OK = 0,
    HELIOS_EINVAL = -1,    /* bad argument seen by the host                         */
    HELIOS_ECAPACITY = -2, /* an output did not fit its capacity (from helios_sync)  */
    HELIOS_EHIP = -3,      /* a HIP runtime call failed                              */
    HELIOS_ESTATE = -4,    /* call order: graph or cache not loaded yet              */
    HELIOS_EDATA = -5,     /* a node ID outside [0, N), or an order that is not a
                              permutation (from helios_sync)                         */
    HELIOS_EINTERNAL = -6  /* a bounded device-side wait ran out (from helios_sync);
                              the results of that call are invalid                   */
} helios_status;

#define HELIOS_MAX_HOPS 8
#define HELIOS_MAX_FANOUT 1024

/* Context on `device`, working on `hip_stream` (a hipStream_t, borrowed;
 * NULL = the default stream).  helios_destroy waits for the stream and frees
 * the library's own memory only; while plans, gangs or miss queues of the
 * context are alive it returns HELIOS_ESTATE and destroys nothing. */
int helios_create(helios_ctx **out, int device, void *hip_stream);
int helios_destroy(helios_ctx *ctx);
const char *helios_last_error(const helios_ctx *ctx);

/* Grow the scratch so that calls with up to max_ids IDs allocate nothing. */
int helios_reserve(helios_ctx *ctx, int64_t max_ids);

/* Wait for the stream; return the first device-side error since the last
 * helios_sync (and clear it), else HELIOS_OK. */
int helios_sync(helios_ctx *ctx);

/* Graph topology (Sec. 3.2.1: the whole topology is kept where GPU threads
 * read it directly).  offsets: int64[n_nodes+1], indices: int32[n_edges];
 * row v = indices[offsets[v] .. offsets[v+1]) = the IDs that can be sampled
 * as neighbours of v.  Both are device-accessible, borrowed. */
int helios_csr_load(helios_ctx *ctx, int64_t n_nodes, int64_t n_edges,
                    const int64_t *offsets, const int32_t *indices);

/* Cache placement (Sec. 3.2.2 "Cache Initialization": vertices sorted by
 * hotness, the hottest rows fill GPU memory, the next-hottest fill CPU
 * memory).  hotness_order: device int32[n_nodes], a permutation;
 * hotness_order[r] is the node of rank r.  The library builds and owns
 * rank[] (rank[hotness_order[r]] = r).  hbm_rows / host_rows are clamped to
 * what is left of n_nodes.  The three tables are borrowed, laid out in rank
 * order, row_bytes per row (a multiple of 16):
 *   hbm_table     device memory,       row r <-> rank r
 *   host_table    pinned mapped host,  row s <-> rank hbm_rows + s
 *   standin_table pinned mapped host,  row t <-> rank hbm_rows + host_rows + t
 * (the stand-in replaces the SSD array of Sec. 3.1; it may be NULL if
 * helios_gather_miss is never called).  A table with zero rows may be NULL.
 * Requires helios_csr_load first (for n_nodes). */
int helios_cache_build(helios_ctx *ctx, const int32_t *hotness_order,
                       int64_t hbm_rows, int64_t host_rows, int32_t row_bytes,
                       const void *hbm_table, const void *host_table, const void *standin_table);

/* Helper for filling a tier table from a full feature table:
 * dst[i, :] = src[order[first_rank + i], :] for i in [0, n_rows).
 * src and dst are device-accessible; order is device int32. */
int helios_cache_fill(helios_ctx *ctx, const void *src_table, const int32_t *order,
                      int64_t first_rank, int64_t n_rows, int32_t row_bytes, void *dst);

/* k-hop uniform neighbour sampling without replacement (Sec. 3.2.2 "Cache
 * Lookup": a GPU kernel for neighbour sampling; Sec. 4.1: 2-hop, fan-outs 25
 * and 10).  The frontier of hop 0 is `seeds` as given; the frontier of hop
 * h+1 is the de-duplicated sample list of hop h in first-occurrence order.
 * Node v at hop h yields min(deg(v), fanouts[h]) neighbours: the whole row in
 * CSR order if it is no longer than the fan-out, else positions chosen by
 * Floyd's subset algorithm from Philox4x32-10 draws keyed by
 * (rng_seed, hop, v), so a node's sample does not depend on its place in the
 * frontier.
 *   seeds    device int32[n_seeds]
 *   fanouts  host int32[n_hops], 0 <= fanout <= HELIOS_MAX_FANOUT
 *   hops     host array of n_hops descriptors of device output buffers:
 *            frontier[frontier_cap], indptr[frontier_cap + 1], flat[flat_cap];
 *            the worst case is frontier_cap(0) = n_seeds,
 *            flat_cap(h) = frontier_cap(h) * fanouts[h], frontier_cap(h+1) = flat_cap(h)
 *   sizes    device-accessible int64[2 * n_hops]: sizes[2h] = |frontier h|,
 *            sizes[2h+1] = |flat h| (the required sizes, also on ECAPACITY)
 * flat[indptr[i] .. indptr[i+1]) are the samples of frontier[i]. */
typedef struct {
    int32_t *frontier;
    int64_t frontier_cap;
    int64_t *indptr;
    int32_t *flat;
    int64_t flat_cap;
} helios_hop_out;

int helios_sample(helios_ctx *ctx, const int32_t *seeds, int64_t n_seeds,
                  const int32_t *fanouts, int32_t n_hops, uint64_t rng_seed,
                  const helios_hop_out *hops, int64_t *sizes);

/* De-duplication of the sampled ID list (the "sampled vertices' ID list" of
 * Sec. 3.1.1).  unique = the distinct values of ids in order of first
 * occurrence; inverse[j] (nullable) = index in unique of ids[j].
 *   ids device int32[n_ids]; unique device int32[unique_cap];
 *   inverse device int32[n_ids]; n_unique device-accessible int64[1]. */
int helios_dedup(helios_ctx *ctx, const int32_t *ids, int64_t n_ids,
                 int32_t *unique, int64_t unique_cap, int32_t *inverse, int64_t *n_unique);

/* helios_dedup for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * results and same errors as helios_dedup, but the call allocates and frees
 * nothing: all its scratch (hash table, per-input slots, scan state, counters)
 * is a fixed array of about 6 MiB in the library's device image, which every
 * GPU the library runs on holds until the process ends.  At most
 * HELIOS_DEDUP_NOALLOC_MAX_IDS IDs per call, more is HELIOS_EINVAL.  All
 * contexts of a GPU share that array and each call starts by resetting it, so
 * calls that overlap on one GPU (different streams or host threads) race: the
 * caller serialises them.  It does not touch the scratch of helios_dedup or of
 * the batch calls. */
#define HELIOS_DEDUP_NOALLOC_MAX_IDS 262144
int helios_dedup_noalloc(helios_ctx *ctx, const int32_t *ids, int64_t n_ids,
                         int32_t *unique, int64_t unique_cap, int32_t *inverse, int64_t *n_unique);

/* Cache lookup + feature gather + miss list (Sec. 3.2.2 "Cache Lookup": GPU
 * threads read cached rows directly from GPU memory or, through the mapped
 * address, from CPU memory; Sec. 3.1.1: the IDs found in neither cache are
 * the request list of the storage tier).  For j in [0, n_ids): r =
 * rank[ids[j]]; r < hbm_rows: out[j,:] = hbm_table[r,:]; r < hbm_rows +
 * host_rows: out[j,:] = host_table[r - hbm_rows,:]; else out[j,:] is left
 * untouched and (j, ids[j], r - hbm_rows - host_rows) is appended to the
 * miss list, which is dense and ascending in j.
 *   ids device int32[n_ids] (duplicates allowed);  out device [n_ids x row_bytes]
 *   miss_pos / miss_id / miss_slot device int32[miss_cap]
 *   stats device-accessible; n_hit_hbm + n_hit_host + n_miss = n_ids */
typedef struct {
    int64_t n_ids;
    int64_t n_hit_hbm;
    int64_t n_hit_host;
    int64_t n_miss;
} helios_gather_stats;

int helios_gather(helios_ctx *ctx, const int32_t *ids, int64_t n_ids, void *out,
                  int32_t *miss_pos, int32_t *miss_id, int32_t *miss_slot, int64_t miss_cap,
                  helios_gather_stats *stats);

/* Service of the miss list from the storage stand-in (in place of the IO
 * stack of Sec. 3.1): out[miss_pos[k],:] = standin_table[miss_slot[k],:].
 * n_miss_max bounds the list; if n_miss_dev (device-accessible int64, e.g.
 * &stats->n_miss) is not NULL the count is read from it on the device,
 * otherwise exactly n_miss_max entries are served.  out has out_rows rows.
 * The list is the caller's, so every entry is checked on the device: one whose
 * slot is no row of the stand-in, or whose position is no row of out, is
 * skipped and reported as HELIOS_EDATA by the next helios_sync. */
int helios_gather_miss(helios_ctx *ctx, const int32_t *miss_pos, const int32_t *miss_slot,
                       int64_t n_miss_max, const int64_t *n_miss_dev, void *out, int64_t out_rows);

/* The whole path for one mini-batch with no host round trip between the
 * steps: helios_sample, then helios_dedup of [seeds | flat_0 | ... |
 * flat_{K-1}], then helios_gather of the unique IDs (Sec. 3.3 decomposes an
 * iteration into these operators).  Arguments as in the three calls;
 * inverse (nullable) has room for n_seeds + sum_h flat_cap(h) entries; out has
 * room for unique_cap rows.  Results equal those of the three calls made one
 * after the other. */
int helios_prepare_batch(helios_ctx *ctx, const int32_t *seeds, int64_t n_seeds,
                         const int32_t *fanouts, int32_t n_hops, uint64_t rng_seed,
                         const helios_hop_out *hops, int64_t *sizes,
                         int32_t *unique, int64_t unique_cap, int32_t *inverse, int64_t *n_unique,
                         void *out, int32_t *miss_pos, int32_t *miss_id, int32_t *miss_slot,
                         int64_t miss_cap, helios_gather_stats *stats);

/* Pinned, GPU-mapped host memory of exactly `bytes` bytes for the host tier
 * and the storage stand-in (Sec. 3.2.1 "CPU Cache": CPU memory that GPU
 * threads read directly).  The pointer is valid on the host and on every GPU.
 * Returns NULL on failure.  Free with helios_host_free, after every context
 * that uses the memory is destroyed or has been given other tables. */
void *helios_host_alloc(int64_t bytes);
int helios_host_free(void *ptr);

/* Batch generation (Sec. 3.3 names it as the operator between cache lookup
 * and training): the hops of the last helios_prepare_batch on this context in
 * local numbering.  For hop h, row_local[i] = index in `unique` of
 * frontier_h[i] and col_local[e] = index in `unique` of flat_h[e]; together
 * with indptr_h this is the hop's block in CSR form over the rows of `out`.
 * hops: the descriptors given to helios_prepare_batch; blocks: host array of
 * n_hops descriptors of device buffers, row_local[frontier_cap(h)],
 * col_local[flat_cap(h)].  It reuses the hash table of that batch's
 * de-duplication, which the context keeps until the second batch after it is
 * launched; helios_make_blocks serves the context's last batch (HELIOS_ESTATE
 * if there is none), helios_plan_make_blocks (below) the last batch of a
 * recorded plan, also when one more batch has been queued behind it. */
typedef struct {
    int32_t *row_local;
    int32_t *col_local;
} helios_block_out;

int helios_make_blocks(helios_ctx *ctx, const helios_hop_out *hops, int32_t n_hops,
                       const helios_block_out *blocks);

/* Pre-sampling hotness (Sec. 3.2.2 "Cache Initialization": an epoch of
 * pre-sampling collects every vertex's hotness, then the GPU sorts the
 * vertices by hotness, descending).  helios_hotness_add adds one to the
 * counter of every ID of one batch's de-duplicated list (ids device int32,
 * distinct; n_max bounds the list; n_dev, nullable, is a device-accessible
 * count as in helios_gather_miss; counts device int32[n_nodes], zeroed by the
 * caller before the epoch).  helios_hotness_order writes the nodes by counter
 * descending, ties by ascending ID, to order (device int32[n_nodes]): the
 * hotness_order argument of helios_cache_build.  Its scratch (about 13 bytes
 * per node) is allocated on the first call and kept by the context. */
int helios_hotness_add(helios_ctx *ctx, const int32_t *ids, int64_t n_max, const int64_t *n_dev,
                       int32_t *counts);
int helios_hotness_order(helios_ctx *ctx, const int32_t *counts, int32_t *order);

/* A plain streaming copy dst[0, bytes) = src[0, bytes) (bytes a multiple of
 * 16; device-accessible pointers) with the row copy's 16-byte accesses.  It
 * is the yardstick of the measurements: hardware byte counters are scaled by
 * what they read for this kernel, whose traffic is known, and its rate is the
 * copy bandwidth the part reaches. */
int helios_calibration_copy(helios_ctx *ctx, const void *src, void *dst, int64_t bytes);

/* Launch-shape parameters (tuning; results do not depend on them).
 * *_GATHER_BLOCKS: workgroups that copy the HBM tier / the host tier and
 * stand-in (0 = built-in default; the host-link copies need few workgroups to
 * fill the link, and fewer of them leave more of the GPU to the work that runs
 * beside them, cf. Sec. 3.3 "Operator Resources Allocation"; by default the
 * members of a gang share what one batch alone would take).  SPLIT_COPIES:
 * zero (the default): helios_prepare_batch overlaps its steps inside its
 * launches (Sec. 3.3, intra-mini-batch pipeline): the host-tier rows that one
 * hop has brought in are copied while the next hop is sampled, and the last
 * ones beside the HBM-tier copy.  Non-zero: the two tier copies run after the
 * last hop as kernels of their own, one after the other (for measuring each
 * copy by itself).
 * SERVE_MISSES: non-zero: helios_prepare_batch (and recordings and gangs made
 * while it is set) also serves the batch's miss list from the storage
 * stand-in, out[miss_pos[k],:] = standin_table[miss_slot[k],:], as
 * helios_gather_miss would right after it (S6 by zero-copy reads, beside the
 * last host-tier copy); the miss list is still written.  Needs the stand-in
 * table; not together with an attached miss queue (HELIOS_ESTATE).
 * MISSQ_TIMEOUT_US: how long a wave of helios_missq_complete's kernel waits
 * without seeing a new completion before it gives up (default 2 000 000);
 * MISSQ_WAVES: waves of that kernel (0 = default 256; at least one per 64
 * queues, at most one per queue). */
typedef enum {
    HELIOS_PARAM_HBM_GATHER_BLOCKS = 1,
    HELIOS_PARAM_HOST_GATHER_BLOCKS = 2,
    HELIOS_PARAM_SPLIT_COPIES = 3,
    HELIOS_PARAM_MISSQ_TIMEOUT_US = 4,
    HELIOS_PARAM_MISSQ_WAVES = 5,
    HELIOS_PARAM_SERVE_MISSES = 6
} helios_param;
int helios_set_param(helios_ctx *ctx, int param, int64_t value);

/* A recorded batch: the kernel sequence of helios_prepare_batch for one fixed
 * set of buffers, captured once into a HIP graph and replayed with one launch
 * per mini-batch (the per-batch path is a handful of short kernels, so the
 * host's launch cost matters).  helios_plan_create takes the arguments of
 * helios_prepare_batch except seeds and rng_seed; all buffers, capacities,
 * n_seeds and fan-outs are fixed by it.  helios_plan_launch(plan, seeds,
 * rng_seed) enqueues one batch on the context's stream: seeds (device
 * int32[n_seeds]) may be a different buffer every time.  Results, errors and
 * helios_make_blocks behave as after helios_prepare_batch.  The context's
 * stream must not be the NULL stream; the timing level in force at creation
 * (0 or 1; level 2 cannot be recorded) is part of the recording.  A
 * plan is bound to its context and becomes invalid (HELIOS_ESTATE) if the
 * context's scratch grows afterwards; call helios_reserve first.  At most 255
 * launches may be queued without a helios_sync (one more waits for the stream
 * by itself).  Destroy the plan before the context. */
typedef struct helios_plan helios_plan;
int helios_plan_create(helios_ctx *ctx, int64_t n_seeds, const int32_t *fanouts, int32_t n_hops,
                       const helios_hop_out *hops, int64_t *sizes,
                       int32_t *unique, int64_t unique_cap, int32_t *inverse, int64_t *n_unique,
                       void *out, int32_t *miss_pos, int32_t *miss_id, int32_t *miss_slot,
                       int64_t miss_cap, helios_gather_stats *stats, helios_plan **plan_out);
int helios_plan_launch(helios_plan *plan, const int32_t *seeds, uint64_t rng_seed);
/* Waits until the plan's last launch has finished (not for launches of other
 * plans queued behind it on the same context) and reports the device-side
 * errors of this plan's batches (every plan has an error word of its own;
 * helios_sync reports and clears those of all plans of the context).  With two plans over two buffer sets on one context the
 * host can queue a batch behind the one that is running and still take each
 * batch's results as soon as it is done. */
int helios_plan_wait(helios_plan *plan);
/* helios_make_blocks for the plan's last launch, from the plan's own buffers
 * (the hops and sizes given to helios_plan_create; without a sizes array only
 * right after the launch).  Valid while at most one more batch has been
 * launched on the context since (e.g. two plans over two buffer sets used in
 * turn: launch A, launch B, wait A, blocks of A, launch A, ...); else
 * HELIOS_ESTATE.  Its device-side errors are reported by the plan's wait. */
int helios_plan_make_blocks(helios_plan *plan, const helios_block_out *blocks);
int helios_plan_destroy(helios_plan *plan);

/* A gang: the mini-batches of several contexts recorded into the same
 * launches.  One mini-batch is a chain of short launches that latency, not
 * throughput, bounds; the chains of independent mini-batches overlap best
 * when they are the same launches (Sec. 3.3 pipelines independent
 * mini-batches on streams; here up to HELIOS_MAX_GANG of them share every
 * launch, each with workgroups of its own, and gangs in turn may run on
 * different streams).  The members are contexts created on one and the same
 * (non-NULL) stream, each with its graph, its cache (rows of one size) and
 * its scratch; member m's batch goes to buffers[m] (the buffer arguments of
 * helios_prepare_batch; hops points to n_hops entries) and its results and
 * errors are those of helios_prepare_batch on that context, bit for bit.
 * n_seeds (at most 2048), the fan-outs and n_hops are the same for all
 * members.  Event timing (level 2), split copies and an attached miss queue do
 * not go with a gang (HELIOS_ESTATE); timing level 1 at creation is part of the
 * recording, and helios_batch_ticks then gives a member's roles.  Argument errors are reported through ctxs[0]
 * (helios_last_error).
 *
 * helios_gang_launch: seeds[m] (device int32[n_seeds]) and rng_seeds[m] are
 * member m's; one launch sequence on the shared stream prepares all batches.
 * helios_gang_wait: waits for the gang's last launch; member_status
 * (nullable, n_members entries) receives every member's own device-side
 * error code, the return value is the first that is not HELIOS_OK.
 * helios_gang_make_blocks: helios_plan_make_blocks for one member's batch.
 * A call on a gang counts as a call on each of its contexts (one host thread
 * at a time).  Between launches of a gang its contexts may be used for other calls; the
 * rules of a recorded batch apply to every member (scratch, cache and graph
 * unchanged since the recording; at most 255 launches without a wait).
 * Destroy the gang before its contexts. */
#define HELIOS_MAX_GANG 4
typedef struct {
    const helios_hop_out *hops;
    int64_t *sizes;
    int32_t *unique;
    int64_t unique_cap;
    int32_t *inverse;
    int64_t *n_unique;
    void *out;
    int32_t *miss_pos, *miss_id, *miss_slot;
    int64_t miss_cap;
    helios_gather_stats *stats;
} helios_batch_buffers;
typedef struct helios_gang helios_gang;
int helios_gang_create(helios_ctx *const *ctxs, int32_t n_members, int64_t n_seeds,
                       const int32_t *fanouts, int32_t n_hops,
                       const helios_batch_buffers *buffers, helios_gang **gang_out);
int helios_gang_launch(helios_gang *gang, const int32_t *const *seeds, const uint64_t *rng_seeds);
int helios_gang_wait(helios_gang *gang, int32_t *member_status);
int helios_gang_make_blocks(helios_gang *gang, int32_t member, const helios_block_out *blocks);
int helios_gang_destroy(helios_gang *gang);

/* Asynchronous service of the miss list in the shape of the GPU-initiated IO
 * stack of Sec. 3.1, with host threads over the storage stand-in in the place
 * of the SSDs: a submission kernel (Sec. 3.1.1: one thread per miss builds a
 * command {storage row, staging row} and writes it to one of n_queues
 * submission queues; each queue's doorbell is rung once, after all commands
 * are written), service threads (a thread owns every n_service_threads-th
 * queue, copies each command's row from the stand-in table into a pinned
 * staging buffer and posts a completion entry, not in submission order), and
 * a completion kernel (Sec. 3.1.2: a wave owns several completion queues,
 * polls their entries and moves completed rows from the staging buffer to
 * out[miss_pos]).  Nothing on the GPU waits between the two kernels.  The
 * result equals helios_gather_miss's.
 *
 * helios_missq_create: queue memory for up to n_queues * queue_depth misses
 * per round (1..4096 queues of 1..2^20 entries; the staging buffer of that
 * many rows must stay below 8 GiB) on the context's current cache; starts the
 * service threads (0..64; with 0 nothing is ever served: for tests of the
 * time limit).  The queue is bound to the context and to that cache: after
 * another helios_cache_build its calls return HELIOS_ESTATE.
 * helios_missq_submit enqueues the submission kernel on the context's stream
 * (arguments as helios_gather_miss: out_rows = rows of the buffer that
 * helios_missq_complete will be given; an entry outside the stand-in or
 * outside out is reported as HELIOS_EDATA and its data is dropped);
 * helios_missq_complete enqueues the completion kernel.  The two alternate (else HELIOS_ESTATE): one round at a
 * time per queue; to keep several batches in flight give each context a queue.
 * A round with more misses than the queues hold reports HELIOS_ECAPACITY at
 * helios_sync and serves the first n_queues * queue_depth.  If the service
 * stops answering (or met a command it had to refuse: helios_missq_faulted
 * returns 1), the completion kernel ends after the time limit and
 * helios_sync returns HELIOS_EINTERNAL; the queue must then be destroyed.
 * helios_missq_attach(ctx, q): from now on every helios_prepare_batch and
 * every batch recorded by helios_plan_create on ctx submits its own miss list
 * right after the cache lookup, before the cached tiers are copied, so the
 * service runs beside those copies; the caller follows each batch with
 * helios_missq_complete.  q = NULL detaches.  A recorded batch can only be
 * launched while the queue it was recorded with is attached.
 * helios_missq_destroy waits for the stream, detaches the queue and stops the
 * threads; destroy a queue before its context. */
typedef struct helios_missq helios_missq;
int helios_missq_create(helios_ctx *ctx, int32_t n_queues, int32_t queue_depth,
                        int32_t n_service_threads, helios_missq **out);
int helios_missq_submit(helios_missq *q, const int32_t *miss_pos, const int32_t *miss_slot,
                        int64_t n_miss_max, const int64_t *n_miss_dev, int64_t out_rows);
int helios_missq_complete(helios_missq *q, void *out);
int helios_missq_attach(helios_ctx *ctx, helios_missq *q);
int helios_missq_faulted(const helios_missq *q);
/* out[0] = rounds opened, out[1] = rounds every service thread has finished,
 * out[2] = commands served since the queue was created */
int helios_missq_counters(const helios_missq *q, int64_t *out3);
int helios_missq_destroy(helios_missq *q);

/* Timing.  Level 1: every workgroup of every step ("role": a launch of the
 * whole-path call carries several, see SPLIT_COPIES) of the next
 * helios_prepare_batch / helios_gather / recorded batch stores its first and
 * last tick of the GPU's constant-rate clock; helios_batch_ticks waits for the
 * stream and returns, per role of the last batch, earliest start and latest
 * end (ticks of a clock that all contexts of a device share, so batches in
 * flight on several contexts can be placed on one time axis; *ticks_per_us,
 * nullable, receives its rate).  kind is a helios_role, stage the hop (for
 * copies: the stage of the batch's ID list, i.e. the hop that completed it).
 * helios_gather_times returns the HBM-tier copy's span and the sum of the
 * host-tier copies' spans in milliseconds.  Level 2 (directly launched calls
 * with split copies, and helios_gather): the two copy kernels are launched
 * with HIP events that take each kernel's own begin and end, as a kernel
 * trace reports them; helios_gather_times returns them in hbm_event_ms /
 * host_event_ms (nullable; 0 at level 1).  Level 0 turns timing off.  The
 * level in force when a batch is recorded (0 or 1) is part of the recording. */
typedef enum {
    HELIOS_ROLE_SAMPLE = 1,          /* sampling pass of a hop                       */
    HELIOS_ROLE_COMPACT_HOP = 2,     /* a hop's samples -> next frontier             */
    HELIOS_ROLE_COMPACT_LOOKUP = 3,  /* a stage of the batch's ID list, cache lookup */
    HELIOS_ROLE_COPY_HOST = 4,       /* host-tier rows of a stage                    */
    HELIOS_ROLE_COPY_HBM = 5,        /* HBM-tier rows                                */
    HELIOS_ROLE_INVERSE = 6,
    HELIOS_ROLE_COPY_STANDIN = 7     /* rows of the miss list, from the stand-in     */
} helios_role;
typedef struct {
    int32_t kind, stage;
    int64_t workgroups;
    uint64_t start, end;             /* 0, 0 if the role did not run */
} helios_role_ticks;
int helios_set_timing(helios_ctx *ctx, int level);
int helios_batch_ticks(helios_ctx *ctx, helios_role_ticks *out, int32_t cap, int32_t *n_out,
                       double *ticks_per_us);
int helios_gather_times(helios_ctx *ctx, float *hbm_ms, float *host_ms,
                        float *hbm_event_ms, float *host_event_ms);

#ifdef __cplusplus
}
#endif
#endif /* HELIOS_H */
