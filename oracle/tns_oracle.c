/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Plain CPU definition of one-hop temporal neighbourhood sampling.  Only tests, the
 * smoke check and the bench's cpu_baseline leg may call this; the HIP library never does
 * and shares no code with it.
 *
 * What the paper's method returns does not depend on how edges are packed into blocks
 * (section 4.1: blocks, their sizes and the ingestion batching only decide *where* an
 * edge sits), so this file uses no blocks at all.  It writes the result out from its
 * definition:
 *
 *   O1  per-node chronological edge lists        section 4.1: a node's edge data is kept
 *                                                in increasing timestamp order; a directed
 *                                                edge is stored with its source node
 *                                                (footnote there)
 *   O2  candidate window [t_s, t_e)              Algorithm 1, the step that finds the
 *                                                neighbours inside the time window; the
 *                                                closed upper bound [t - delta, t] of
 *                                                section 2.1 as an option
 *   O3  selection: recent / uniform              section 2.1: recent keeps the neighbours
 *                                                nearest in time to the query timestamp,
 *                                                uniform draws a random subset of all
 *   O4  padded result, f slots per target        section 4.2, kernel optimizations
 *                                                (a target's results lie side by side)
 *   O5  removal of the padding                   section 5, the paragraph on GPU sampling
 *
 * Tie rule (the paper fixes the order by timestamp only): order is (timestamp, arrival);
 * among equal timestamps the later arrival is the more recent one.
 * Uniform sampling draws with replacement from a counter-based generator keyed by
 * (seed, query id, slot); the paper fixes neither, see oracle_pick().
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py (worked
 * example of section 2.1, closed forms, numpy reductions, brute force, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_OK = 0, ORA_EINVAL = -1, ORA_EORDER = -2, ORA_ERANGE = -3, ORA_ENOMEM = -4 };

typedef struct {
    int64_t num_nodes;
    int64_t num_edges;   /* stored (present) edges */
    int64_t *rowptr;     /* [num_nodes + 1] : A[v] = positions rowptr[v] .. rowptr[v+1]-1 */
    int32_t *nbr;        /* neighbour id   of each stored edge, chronological per node */
    int32_t *eid;        /* edge id                                                     */
    float *ts;           /* edge timestamp                                              */
} ora_adj;

void oracle_adj_free(ora_adj *a)
{
    if (!a) return;
    free(a->rowptr); free(a->nbr); free(a->eid); free(a->ts); free(a);
}

/*
 * O1.  Build A[v] for every node from a stream given in arrival order.
 *
 *   eid          NULL: edge i has id i
 *   present      NULL: every edge exists; else present[i]==0 marks a deleted edge, which is
 *                treated as absent (section 4.1: entries marked invalid take no part in
 *                sampling)
 *   batch_rowptr NULL: the whole stream is one ingestion batch; else [num_batches+1]
 *                offsets.  Edges of one node inside one batch are put in timestamp order
 *                (stable: equal times keep arrival order); a batch that brings a node an
 *                edge older than what the node already holds is an error (ORA_EORDER), as
 *                the storage appends without re-sorting (section 4.1, advantage (2)).
 */
int oracle_adj_build(int64_t num_nodes, int64_t n, const int32_t *src, const int32_t *dst,
                     const float *ts, const int32_t *eid, const uint8_t *present,
                     const int64_t *batch_rowptr, int64_t num_batches, ora_adj **out)
{
    if (num_nodes < 0 || n < 0 || !out || (n > 0 && (!src || !dst || !ts))) return ORA_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        if (src[i] < 0 || (int64_t)src[i] >= num_nodes) return ORA_ERANGE;
        if (isnan(ts[i])) return ORA_EORDER;
    }
    ora_adj *a = (ora_adj *)calloc(1, sizeof(ora_adj));
    if (!a) return ORA_ENOMEM;
    a->num_nodes = num_nodes;
    a->rowptr = (int64_t *)calloc((size_t)num_nodes + 1, sizeof(int64_t));
    int64_t *fill = (int64_t *)calloc((size_t)num_nodes + 1, sizeof(int64_t));
    if (!a->rowptr || !fill) { free(fill); oracle_adj_free(a); return ORA_ENOMEM; }

    /* stable counting sort by source node */
    int64_t kept = 0;
    for (int64_t i = 0; i < n; ++i)
        if (!present || present[i]) { a->rowptr[src[i] + 1]++; kept++; }
    for (int64_t v = 0; v < num_nodes; ++v) a->rowptr[v + 1] += a->rowptr[v];
    a->num_edges = kept;
    size_t m = (size_t)(kept > 0 ? kept : 1);
    a->nbr = (int32_t *)malloc(m * sizeof(int32_t));
    a->eid = (int32_t *)malloc(m * sizeof(int32_t));
    a->ts = (float *)malloc(m * sizeof(float));
    int64_t *bat = (int64_t *)malloc(m * sizeof(int64_t));   /* ingestion batch of each stored edge */
    if (!a->nbr || !a->eid || !a->ts || !bat) { free(bat); free(fill); oracle_adj_free(a); return ORA_ENOMEM; }

    int64_t b = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (batch_rowptr) while (b + 1 < num_batches && i >= batch_rowptr[b + 1]) ++b;
        if (present && !present[i]) continue;
        int64_t p = a->rowptr[src[i]] + fill[src[i]]++;
        a->nbr[p] = dst[i];
        a->eid[p] = eid ? eid[i] : (int32_t)i;
        a->ts[p] = ts[i];
        bat[p] = b;
    }
    free(fill);

    /* inside one (node, batch) run: stable insertion sort by timestamp */
    for (int64_t v = 0; v < num_nodes; ++v) {
        int64_t lo = a->rowptr[v], hi = a->rowptr[v + 1];
        for (int64_t i = lo + 1; i < hi; ++i) {
            int32_t xn = a->nbr[i], xe = a->eid[i];
            float xt = a->ts[i];
            int64_t xb = bat[i];
            int64_t j = i;
            while (j > lo && bat[j - 1] == xb && a->ts[j - 1] > xt) {
                a->nbr[j] = a->nbr[j - 1]; a->eid[j] = a->eid[j - 1];
                a->ts[j] = a->ts[j - 1]; bat[j] = bat[j - 1];
                --j;
            }
            a->nbr[j] = xn; a->eid[j] = xe; a->ts[j] = xt; bat[j] = xb;
        }
        for (int64_t i = lo + 1; i < hi; ++i)
            if (a->ts[i - 1] > a->ts[i]) { free(bat); oracle_adj_free(a); return ORA_EORDER; }
    }
    free(bat);
    *out = a;
    return ORA_OK;
}

/* first position p in [lo, hi) with ts[p] >= x ; hi if none */
static int64_t first_at_least(const float *ts, int64_t lo, int64_t hi, float x)
{
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (ts[mid] >= x) hi = mid; else lo = mid + 1;
    }
    return lo;
}

/* first position p in [lo, hi) with ts[p] > x ; hi if none */
static int64_t first_greater(const float *ts, int64_t lo, int64_t hi, float x)
{
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (ts[mid] > x) hi = mid; else lo = mid + 1;
    }
    return lo;
}

/*
 * Random rank in [0, c) for slot j of query q: the 64-bit counter seed + G*(q*f + j + 1)
 * goes through the splitmix64 output function; the top 32 bits are scaled to [0, c) by a
 * multiply and shift.  The paper leaves the generator open; this one is keyed by counter
 * so that any thread mapping produces the same picks.
 */
uint64_t oracle_pick(uint64_t seed, int64_t q, int32_t f, int32_t j, uint64_t c)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * ((uint64_t)q * (uint64_t)f + (uint64_t)j + 1ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return ((z >> 32) * c) >> 32;
}

static int g_threads_used = 1;
int oracle_threads_used(void) { return g_threads_used; }

/*
 * O2-O4 for a batch of queries.
 *
 *   targets[Q], t_end[Q]   query node and window end
 *   t_start                NULL: window starts at -infinity
 *   q_ids                  NULL: query i has id i; else the id used by the uniform picks
 *   policy                 0 recent, 1 uniform
 *   inclusive_end          0: [t_s, t_e)   (Algorithm 1)    1: [t_s, t_e]   (section 2.1)
 *   out_*                  padded, f slots per query: slot j < count holds an edge,
 *                          slots >= count hold nbr=-1, eid=-1, ts=0
 * A target outside [0, num_nodes) or a NaN bound gives count 0.
 */
int oracle_sample(const ora_adj *a, int64_t Q, const int32_t *targets, const float *t_start,
                  const float *t_end, const int64_t *q_ids, int32_t f, int32_t policy,
                  int32_t inclusive_end, uint64_t seed, int32_t *out_nbr, int32_t *out_eid,
                  float *out_ts, int32_t *out_count, int32_t num_threads)
{
    if (!a || Q < 0 || f <= 0 || (policy != 0 && policy != 1)) return ORA_EINVAL;
    if (Q > 0 && (!targets || !t_end || !out_nbr || !out_eid || !out_ts || !out_count)) return ORA_EINVAL;
    if (num_threads < 1) num_threads = 1;
    int used = 1;
#ifdef _OPENMP
#pragma omp parallel for num_threads(num_threads) schedule(static)
#endif
    for (int64_t q = 0; q < Q; ++q) {
#ifdef _OPENMP
        if (q == 0) used = omp_get_num_threads();
#endif
        int32_t *on = out_nbr + q * f, *oe = out_eid + q * f;
        float *ot = out_ts + q * f;
        int64_t v = targets[q];
        float te = t_end[q];
        float tb = t_start ? t_start[q] : -INFINITY;
        int64_t c = 0, lo = 0, hi = 0;
        if (v >= 0 && v < a->num_nodes && !isnan(te) && !isnan(tb)) {
            int64_t r0 = a->rowptr[v], r1 = a->rowptr[v + 1];
            lo = first_at_least(a->ts, r0, r1, tb);
            hi = inclusive_end ? first_greater(a->ts, r0, r1, te) : first_at_least(a->ts, r0, r1, te);
            c = hi > lo ? hi - lo : 0;
        }
        int64_t k = c < f ? c : f;
        int64_t qid = q_ids ? q_ids[q] : q;
        for (int64_t j = 0; j < k; ++j) {
            int64_t p;
            if (policy == 0 || c <= f) p = hi - 1 - j;                       /* newest first */
            else p = lo + (int64_t)oracle_pick(seed, qid, f, (int32_t)j, (uint64_t)c);
            on[j] = a->nbr[p]; oe[j] = a->eid[p]; ot[j] = a->ts[p];
        }
        for (int64_t j = k; j < f; ++j) { on[j] = -1; oe[j] = -1; ot[j] = 0.0f; }
        out_count[q] = (int32_t)k;
    }
    g_threads_used = used;
    return ORA_OK;
}

/*
 * O5.  rowptr = exclusive prefix sum of count; compacted arrays list the filled slots in
 * (query, slot) order.  cmp_* may be NULL to get rowptr only.
 */
int oracle_compact(int64_t Q, int32_t f, const int32_t *nbr, const int32_t *eid, const float *ts,
                   const int32_t *count, int64_t *rowptr, int32_t *cmp_nbr, int32_t *cmp_eid,
                   float *cmp_ts)
{
    if (Q < 0 || f <= 0 || !rowptr || (Q > 0 && !count)) return ORA_EINVAL;
    int64_t w = 0;
    for (int64_t q = 0; q < Q; ++q) {
        rowptr[q] = w;
        if (count[q] < 0 || count[q] > f) return ORA_EINVAL;
        for (int32_t j = 0; j < count[q]; ++j, ++w) {
            if (cmp_nbr) cmp_nbr[w] = nbr[q * f + j];
            if (cmp_eid) cmp_eid[w] = eid[q * f + j];
            if (cmp_ts) cmp_ts[w] = ts[q * f + j];
        }
    }
    rowptr[Q] = w;
    return ORA_OK;
}
