/*
 * CPU oracle for the mini-batch preparation path of Helios (arXiv 2310.00837):
 * k-hop uniform neighbour sampling over a CSR graph, de-duplication of the
 * sampled IDs, two-tier cache lookup, feature-row gather and the miss list.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-purpose CPU
 * program that defines what the GPU library must reproduce bit for bit.  It
 * shares no code, header, table or constant generator with the HIP path and
 * is never called by it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * What the paper fixes and what it leaves open
 * --------------------------------------------
 * The paper (Sec. 3.2.2 "Cache Lookup", Sec. 3.3, Sec. 4.1 "GNN Models")
 * says only: 2-hop random neighbour sampling with fan-outs 25 and 10, a cache
 * lookup that finds each sampled vertex's feature row in GPU memory, CPU
 * memory or neither, and a list of sampled vertex IDs handed to the IO stack
 * (Sec. 3.1.1).  It gives no RNG, no replacement rule and no output order.
 * Every choice below marked [reading] is this build's reading; the GPU path
 * reproduces the same reading.
 *
 * Parity status of each function (what pins it besides itself):
 *   orc_philox4x32_10   pinned: published known-answer vectors of the
 *                       Philox4x32-10 generator (Salmon et al., SC'11).
 *   orc_bounded         pinned: closed form floor(x*n / 2^64) with big ints.
 *   orc_floyd_positions pinned: exhaustive enumeration (every f-subset of d
 *                       positions is reached by exactly f! of the draw
 *                       tuples) and chi-square uniformity.
 *   orc_sample_*        pinned by invariants only (true neighbours, distinct
 *                       positions, min(deg, fanout) per node, whole row when
 *                       deg <= fanout); the counter layout of the draw
 *                       stream and the frontier rule are readings:
 *                       "parity unpinned" against the paper.
 *   orc_dedup           pinned: order-preserving set (library routine).
 *   orc_rank_build / orc_lookup / orc_gather / orc_gather_miss
 *                       pinned: permutation inverse, closed-form tier ranges,
 *                       array indexing features[ids] (library routine).
 *   orc_hotness_add / orc_hotness_order
 *                       pinned: bincount and lexicographic sort (library
 *                       routines); what counts as hotness is a reading.
 *   orc_local_ids       pinned: dictionary lookup (library routine).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11).  Counter of four 32-bit words, key of two.
 * One round: two 32x32->64 products; the high halves are xored with the
 * other counter words and the round key, the low halves pass through; then
 * the key is bumped by the two Weyl constants.                          */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* [reading] The k-th 64-bit draw of (rng_seed, hop, node).  The stream is
 * keyed by the node and the hop, not by where the node sits in the frontier,
 * so a node's sample does not depend on frontier order or on duplicates.
 * Key = the two halves of rng_seed.  Philox block m has the counter
 * (node, m, hop, tag); it yields draws 2m (words 0,1) and 2m+1 (words 2,3),
 * low word first.  The tag 0x48454C49 separates this use of the generator
 * from any other.                                                        */
uint64_t orc_draw(uint64_t rng_seed, int32_t node, int32_t hop, uint32_t k)
{
    uint32_t ctr[4] = { (uint32_t)node, k >> 1, (uint32_t)hop, 0x48454C49u };
    uint32_t key[2] = { (uint32_t)rng_seed, (uint32_t)(rng_seed >> 32) };
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    if ((k & 1u) == 0) return (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    return (uint64_t)w[2] | ((uint64_t)w[3] << 32);
}

/* [reading] Map a 64-bit draw to [0, n) by the high half of the 128-bit
 * product.  No rejection step: the bias is below n / 2^64.               */
uint64_t orc_bounded(uint64_t x, uint64_t n)
{
    return (uint64_t)(((unsigned __int128)x * (unsigned __int128)n) >> 64);
}

/* [reading] Floyd's subset algorithm (Bentley & Floyd, CACM 30(9), 1987):
 * f distinct positions out of d, d > f, every f-subset equally likely when
 * the draws are uniform.  Step k (k = 0..f-1) looks at j = d - f + k, draws
 * t uniformly from [0, j], and takes t unless t was taken already, in which
 * case it takes j (which cannot have been taken: every earlier pick is
 * below j).  Picks are reported in step order.                           */
void orc_floyd_positions(int64_t d, int32_t f, const uint64_t *draws, int64_t *s)
{
    for (int32_t k = 0; k < f; ++k) {
        int64_t j = d - f + k;
        int64_t t = (int64_t)orc_bounded(draws[k], (uint64_t)(j + 1));
        int taken = 0;
        for (int32_t i = 0; i < k; ++i)
            if (s[i] == t) taken = 1;
        s[k] = taken ? j : t;
    }
}

/* Sample of one node at one hop: min(deg, f) neighbours.  A row no longer
 * than the fan-out is returned whole, in CSR order, and uses no random
 * numbers; otherwise the Floyd positions index the row.  Returns the count,
 * or -1 if the node ID is outside [0, n_nodes).                          */
int64_t orc_sample_node(int64_t n_nodes, const int64_t *offsets, const int32_t *indices,
                        int32_t v, int32_t hop, int32_t f, uint64_t rng_seed, int32_t *out)
{
    if (v < 0 || (int64_t)v >= n_nodes) return -1;
    int64_t base = offsets[v];
    int64_t d = offsets[v + 1] - base;
    if (f <= 0) return 0;
    if (d <= (int64_t)f) {
        for (int64_t k = 0; k < d; ++k) out[k] = indices[base + k];
        return d;
    }
    uint64_t *draws = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)f);
    int64_t *s = (int64_t *)malloc(sizeof(int64_t) * (size_t)f);
    for (int32_t k = 0; k < f; ++k) draws[k] = orc_draw(rng_seed, v, hop, (uint32_t)k);
    orc_floyd_positions(d, f, draws, s);
    for (int32_t k = 0; k < f; ++k) out[k] = indices[base + s[k]];
    free(draws);
    free(s);
    return f;
}

/* One hop over a frontier: indptr[i] = start of node i's samples in flat,
 * indptr[n_frontier] = total.  flat must hold n_frontier * f entries.
 * Returns 0, or -1 if a frontier entry is not a node ID.  The loop over
 * frontier nodes is independent per node (OpenMP when compiled with it). */
int orc_sample_hop(int64_t n_nodes, const int64_t *offsets, const int32_t *indices,
                   const int32_t *frontier, int64_t n_frontier, int32_t hop, int32_t f,
                   uint64_t rng_seed, int64_t *indptr, int32_t *flat)
{
    int bad = 0;
    indptr[0] = 0;
    for (int64_t i = 0; i < n_frontier; ++i) {
        int32_t v = frontier[i];
        if (v < 0 || (int64_t)v >= n_nodes) { bad = 1; indptr[i + 1] = indptr[i]; continue; }
        int64_t d = offsets[v + 1] - offsets[v];
        int64_t c = d < (int64_t)f ? d : (int64_t)f;
        if (c < 0) c = 0;
        indptr[i + 1] = indptr[i] + c;
    }
    if (bad) return -1;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_frontier; ++i)
        orc_sample_node(n_nodes, offsets, indices, frontier[i], hop, f, rng_seed, flat + indptr[i]);
    return 0;
}

/* Order-preserving de-duplication: the distinct values of ids in order of
 * first occurrence; inverse[j] (optional) = index in unique of ids[j].
 * [reading] first-occurrence order, so that distinct seeds stay a prefix.
 * IDs must lie in [0, n_nodes); returns the number of unique IDs or -1.   */
int64_t orc_dedup(int64_t n_nodes, const int32_t *ids, int64_t n_ids, int32_t *unique, int32_t *inverse)
{
    static int32_t *where = NULL;      /* where[id] = index in unique, or -1 */
    static int64_t where_n = 0;
    if (where_n < n_nodes) {
        free(where);
        where = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_nodes);
        where_n = n_nodes;
        for (int64_t i = 0; i < n_nodes; ++i) where[i] = -1;
    }
    int64_t u = 0;
    int64_t bad = 0;
    for (int64_t j = 0; j < n_ids; ++j) {
        int32_t id = ids[j];
        if (id < 0 || (int64_t)id >= n_nodes) { bad = 1; break; }
        if (where[id] < 0) {
            where[id] = (int32_t)u;
            unique[u] = id;
            ++u;
        }
        if (inverse) inverse[j] = where[id];
    }
    for (int64_t i = 0; i < u; ++i) where[unique[i]] = -1;   /* leave the scratch clean */
    return bad ? -1 : u;
}

/* [reading] k-hop sampling.  The frontier of hop 0 is the seed list as given
 * (order and duplicates kept); the frontier of hop h+1 is the de-duplicated
 * sample list of hop h, in first-occurrence order.  A hop is a function of
 * the previous hop's output only: nodes expanded at an earlier hop are not
 * excluded.  Caller-allocated outputs per hop h:
 *   frontier[h] : capacity B * prod_{g<h} fanouts[g]      (B = n_seeds)
 *   indptr[h]   : that capacity + 1
 *   flat[h]     : that capacity * fanouts[h]
 * sizes[2h] = |frontier h|, sizes[2h+1] = |flat h|.  Returns 0 or -1.     */
int orc_sample(int64_t n_nodes, const int64_t *offsets, const int32_t *indices,
               const int32_t *seeds, int64_t n_seeds, const int32_t *fanouts, int32_t n_hops,
               uint64_t rng_seed, int32_t **frontier, int64_t **indptr, int32_t **flat,
               int64_t *sizes)
{
    int64_t nf = n_seeds;
    for (int64_t i = 0; i < n_seeds; ++i) frontier[0][i] = seeds[i];
    for (int32_t h = 0; h < n_hops; ++h) {
        if (orc_sample_hop(n_nodes, offsets, indices, frontier[h], nf, h, fanouts[h], rng_seed,
                           indptr[h], flat[h]) != 0)
            return -1;
        int64_t nflat = indptr[h][nf];
        sizes[2 * h] = nf;
        sizes[2 * h + 1] = nflat;
        if (h + 1 < n_hops) {
            nf = orc_dedup(n_nodes, flat[h], nflat, frontier[h + 1], NULL);
            if (nf < 0) return -1;
        }
    }
    return 0;
}

/* Cache map (Sec. 3.2.2 "Cache Initialization": vertices sorted by hotness,
 * hottest rows in the GPU cache, next-hottest in the CPU cache).
 * order[r] = node of rank r; rank[order[r]] = r.  Returns -1 if order is
 * not a permutation of 0..n_nodes-1.                                      */
int orc_rank_build(const int32_t *order, int64_t n_nodes, int32_t *rank)
{
    for (int64_t v = 0; v < n_nodes; ++v) rank[v] = -1;
    for (int64_t r = 0; r < n_nodes; ++r) {
        int32_t v = order[r];
        if (v < 0 || (int64_t)v >= n_nodes || rank[v] != -1) return -1;
        rank[v] = (int32_t)r;
    }
    return 0;
}

/* Tier and slot of each ID: ranks [0, n_hbm) are tier 0 (GPU memory),
 * [n_hbm, n_hbm + n_host) tier 1 (pinned host memory), the rest tier 2
 * (storage stand-in); the slot is the rank minus the tier's first rank.   */
void orc_lookup(const int32_t *ids, int64_t n_ids, const int32_t *rank,
                int64_t n_hbm, int64_t n_host, int8_t *tier, int32_t *slot)
{
    for (int64_t j = 0; j < n_ids; ++j) {
        int64_t r = rank[ids[j]];
        if (r < n_hbm) { tier[j] = 0; slot[j] = (int32_t)r; }
        else if (r < n_hbm + n_host) { tier[j] = 1; slot[j] = (int32_t)(r - n_hbm); }
        else { tier[j] = 2; slot[j] = (int32_t)(r - n_hbm - n_host); }
    }
}

/* Gather with miss list.  Row j of out receives the feature row of ids[j]
 * when it is in tier 0 or 1; [reading] rows of tier-2 IDs are left
 * untouched and (j, id, slot) is appended to the miss list, ascending j.
 * stats = { n_ids, hits tier 0, hits tier 1, misses }.                    */
void orc_gather(const int32_t *ids, int64_t n_ids, const int32_t *rank,
                int64_t n_hbm, int64_t n_host, int32_t row_bytes,
                const uint8_t *hbm_table, const uint8_t *host_table, uint8_t *out,
                int32_t *miss_pos, int32_t *miss_id, int32_t *miss_slot, int64_t *stats)
{
    int8_t *tier = (int8_t *)malloc((size_t)(n_ids > 0 ? n_ids : 1));
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_ids > 0 ? n_ids : 1));
    orc_lookup(ids, n_ids, rank, n_hbm, n_host, tier, slot);
    int64_t n0 = 0, n1 = 0, n2 = 0;
    for (int64_t j = 0; j < n_ids; ++j) {
        if (tier[j] == 2) {
            miss_pos[n2] = (int32_t)j; miss_id[n2] = ids[j]; miss_slot[n2] = slot[j];
            ++n2;
        } else if (tier[j] == 0) ++n0;
        else ++n1;
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_ids; ++j) {
        if (tier[j] == 2) continue;
        const uint8_t *src = (tier[j] == 0 ? hbm_table : host_table) + (size_t)slot[j] * (size_t)row_bytes;
        memcpy(out + (size_t)j * (size_t)row_bytes, src, (size_t)row_bytes);
    }
    stats[0] = n_ids; stats[1] = n0; stats[2] = n1; stats[3] = n2;
    free(tier);
    free(slot);
}

/* Service of the miss list from the storage stand-in table.               */
void orc_gather_miss(const int32_t *miss_pos, const int32_t *miss_slot, int64_t n_miss,
                     int32_t row_bytes, const uint8_t *standin_table, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n_miss; ++k)
        memcpy(out + (size_t)miss_pos[k] * (size_t)row_bytes,
               standin_table + (size_t)miss_slot[k] * (size_t)row_bytes, (size_t)row_bytes);
}

/* Pre-sampling hotness (Sec. 3.2.2 "Cache Initialization": one epoch of
 * pre-sampling collects every vertex's hotness, then vertices are sorted by
 * hotness, descending).  [reading] The hotness of a vertex is the number of
 * mini-batches of the epoch whose de-duplicated ID list contains it, i.e. the
 * number of times its feature row is fetched.  One call adds one batch's
 * unique list. */
void orc_hotness_add(const int32_t *unique, int64_t n_unique, int32_t *counts)
{
    for (int64_t j = 0; j < n_unique; ++j) counts[unique[j]] += 1;
}

static const int32_t *g_sort_counts;
static int cmp_hotness(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    if (g_sort_counts[x] != g_sort_counts[y]) return g_sort_counts[x] > g_sort_counts[y] ? -1 : 1;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* order = nodes by hotness descending; [reading] ties by ascending node ID. */
void orc_hotness_order(const int32_t *counts, int64_t n_nodes, int32_t *order)
{
    for (int64_t v = 0; v < n_nodes; ++v) order[v] = (int32_t)v;
    g_sort_counts = counts;
    qsort(order, (size_t)n_nodes, sizeof(int32_t), cmp_hotness);
}

/* Batch generation (Sec. 3.3 lists it as the operator between cache lookup
 * and training): relabel node IDs to their index in the batch's unique list,
 * so that hop h becomes a block in local numbering: row i = frontier_h[i],
 * its columns = flat_h[indptr_h[i] .. indptr_h[i+1]).  out[j] = index in
 * unique of ids[j]; returns -1 if some ID is not in unique. */
int orc_local_ids(int64_t n_nodes, const int32_t *unique, int64_t n_unique,
                  const int32_t *ids, int64_t n_ids, int32_t *out)
{
    int32_t *where = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    for (int64_t v = 0; v < n_nodes; ++v) where[v] = -1;
    for (int64_t u = 0; u < n_unique; ++u) where[unique[u]] = (int32_t)u;
    int bad = 0;
    for (int64_t j = 0; j < n_ids; ++j) {
        int32_t id = ids[j];
        out[j] = (id >= 0 && (int64_t)id < n_nodes) ? where[id] : -1;
        if (out[j] < 0) bad = 1;
    }
    free(where);
    return bad ? -1 : 0;
}

/* Number of worker threads the parallel loops above use (1 without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
void orc_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int orc_num_threads(void) { return 1; }
void orc_set_num_threads(int n) { (void)n; }
#endif
