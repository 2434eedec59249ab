/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Second, structural oracle: the paper's time-indexed block store (section 4.1) built
 * with real heap blocks and pointers, and Algorithm 1 over it in three phases (overlapping blocks, bound searches, selection;
 * section 4.2).  It exists to check (a) that sampling results do not depend on the
 * block layout, by agreeing with the layout-free definition in tns_oracle.c, and (b) the
 * layout facts themselves (block sizes, list lengths, wasted slots).  It shares no code
 * with tns_oracle.c or with the HIP library.
 *
 * Block sizing.  Section 4.1 gives b_v = min(deg(v), tau) for a new block, says space is
 * reserved for future neighbours, and that existing blocks never change size.  It does
 * not say what happens when the formula is too small (a new node has degree 0; a batch
 * can bring a node more edges than min(deg, tau)).  Reading used here: when an ingestion
 * batch brings node v more edges than its tail block can take, the tail is filled and ONE
 * new block is allocated for the remaining m' edges, with capacity
 *      adaptive :  max(m', min(deg_at_allocation, tau))
 *      strawman :  m'                      (section 6.2: exactly as many slots as the batch brings)
 *      fixed    :  ceil(m'/tau) blocks of capacity tau  (section 6.2, PlatoGL style)
 * where deg_at_allocation counts the edges already stored including those that just
 * filled the tail.  The table of list lengths and memory usage in section 6.2 supports the one-block-
 * per-batch reading (adaptive max list length 1896 ~ number of 100k batches in GDELT).
 *
 * Parity pins: tests/test_blockstore_oracle.py (sizing closed forms, structural
 * invariants, waste bound of section 4.1, agreement with tns_oracle.c over thresholds,
 * sizing methods and ingestion splits).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { BS_OK = 0, BS_EINVAL = -1, BS_EORDER = -2, BS_ERANGE = -3, BS_ENOMEM = -4 };
enum { BS_ADAPTIVE = 0, BS_STRAWMAN = 1, BS_FIXED = 2 };

typedef struct bs_block {
    int64_t cap, size;          /* block size (capacity) and edges held                  */
    int32_t *nbr, *eid;         /* graph edge data lists, same index = same edge          */
    float *ts;
    uint8_t *present;           /* validity indicators                                    */
    float t_min, t_max;         /* earliest / latest timestamp in the block               */
    struct bs_block *prev, *next;
} bs_block;

typedef struct {
    bs_block *head, *tail;      /* oldest and newest block                                */
    int64_t nblocks, degree;
    int valid;
} bs_node;

typedef struct {
    int64_t num_nodes, tau;
    int sizing;
    bs_node *nodes;
    int64_t next_eid;
} bs_store;

bs_store *bs_create(int64_t num_nodes, int64_t tau, int sizing)
{
    if (num_nodes < 0 || tau < 1 || sizing < 0 || sizing > 2) return NULL;
    bs_store *s = (bs_store *)calloc(1, sizeof(bs_store));
    if (!s) return NULL;
    s->num_nodes = num_nodes; s->tau = tau; s->sizing = sizing;
    s->nodes = (bs_node *)calloc((size_t)(num_nodes > 0 ? num_nodes : 1), sizeof(bs_node));
    if (!s->nodes) { free(s); return NULL; }
    for (int64_t v = 0; v < num_nodes; ++v) s->nodes[v].valid = 1;
    return s;
}

void bs_destroy(bs_store *s)
{
    if (!s) return;
    for (int64_t v = 0; v < s->num_nodes; ++v) {
        bs_block *b = s->nodes[v].head;
        while (b) { bs_block *nx = b->next; free(b->nbr); free(b->eid); free(b->ts); free(b->present); free(b); b = nx; }
    }
    free(s->nodes); free(s);
}

static bs_block *new_block(int64_t cap)
{
    bs_block *b = (bs_block *)calloc(1, sizeof(bs_block));
    if (!b) return NULL;
    b->cap = cap;
    b->nbr = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    b->eid = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    b->ts = (float *)malloc((size_t)cap * sizeof(float));
    b->present = (uint8_t *)malloc((size_t)cap);
    if (!b->nbr || !b->eid || !b->ts || !b->present) { free(b->nbr); free(b->eid); free(b->ts); free(b->present); free(b); return NULL; }
    return b;
}

static void link_tail(bs_node *nd, bs_block *b)
{
    b->prev = nd->tail; b->next = NULL;
    if (nd->tail) nd->tail->next = b; else nd->head = b;
    nd->tail = b; nd->nblocks++;
}

static void push_edge(bs_node *nd, int32_t nbr, int32_t eid, float ts)
{
    bs_block *b = nd->tail;
    int64_t i = b->size++;
    b->nbr[i] = nbr; b->eid[i] = eid; b->ts[i] = ts; b->present[i] = 1;
    if (i == 0) b->t_min = ts;
    b->t_max = ts;
    nd->degree++;
}

/*
 * One ingestion batch (section 4.1 advantage (2): append to the tail block while it has
 * room, else link a new block at the tail).  eid NULL = running counter.
 */
int bs_add_batch(bs_store *s, int64_t m, const int32_t *src, const int32_t *dst, const float *ts,
                 const int32_t *eid)
{
    if (!s || m < 0 || (m > 0 && (!src || !dst || !ts))) return BS_EINVAL;
    for (int64_t i = 0; i < m; ++i) {
        if (src[i] < 0 || (int64_t)src[i] >= s->num_nodes) return BS_ERANGE;
        if (isnan(ts[i])) return BS_EORDER;
    }
    if (m == 0) return BS_OK;
    /* group the batch by source node, keeping arrival order inside a group */
    int64_t *start = (int64_t *)calloc((size_t)s->num_nodes + 1, sizeof(int64_t));
    int64_t *ord = (int64_t *)malloc((size_t)m * sizeof(int64_t));
    if (!start || !ord) { free(start); free(ord); return BS_ENOMEM; }
    for (int64_t i = 0; i < m; ++i) start[src[i] + 1]++;
    for (int64_t v = 0; v < s->num_nodes; ++v) start[v + 1] += start[v];
    {
        int64_t *fill = (int64_t *)calloc((size_t)s->num_nodes, sizeof(int64_t));
        if (!fill) { free(start); free(ord); return BS_ENOMEM; }
        for (int64_t i = 0; i < m; ++i) ord[start[src[i]] + fill[src[i]]++] = i;
        free(fill);
    }
    /* inside a group: timestamp order, equal times keep arrival order */
    for (int64_t v = 0; v < s->num_nodes; ++v)
        for (int64_t i = start[v] + 1; i < start[v + 1]; ++i) {
            int64_t x = ord[i], j = i;
            while (j > start[v] && ts[ord[j - 1]] > ts[x]) { ord[j] = ord[j - 1]; --j; }
            ord[j] = x;
        }
    /* chronological arrival across batches is required; check before changing anything */
    for (int64_t v = 0; v < s->num_nodes; ++v)
        if (start[v + 1] > start[v] && s->nodes[v].tail && s->nodes[v].tail->size > 0 &&
            ts[ord[start[v]]] < s->nodes[v].tail->t_max) { free(start); free(ord); return BS_EORDER; }

    for (int64_t v = 0; v < s->num_nodes; ++v) {
        int64_t g0 = start[v], g1 = start[v + 1];
        if (g0 == g1) continue;
        bs_node *nd = &s->nodes[v];
        int64_t i = g0;
        while (i < g1 && nd->tail && nd->tail->size < nd->tail->cap) {
            int64_t e = ord[i++];
            push_edge(nd, dst[e], eid ? eid[e] : (int32_t)(s->next_eid + e), ts[e]);
        }
        int64_t rest = g1 - i;
        while (rest > 0) {
            int64_t cap;
            if (s->sizing == BS_STRAWMAN) cap = rest;
            else if (s->sizing == BS_FIXED) cap = s->tau;
            else {
                int64_t bv = nd->degree < s->tau ? nd->degree : s->tau;   /* b_v = min(deg(v), tau) */
                cap = rest > bv ? rest : bv;
            }
            bs_block *b = new_block(cap);
            if (!b) { free(start); free(ord); return BS_ENOMEM; }
            link_tail(nd, b);
            int64_t take = rest < cap ? rest : cap;
            for (int64_t k = 0; k < take; ++k) {
                int64_t e = ord[i++];
                push_edge(nd, dst[e], eid ? eid[e] : (int32_t)(s->next_eid + e), ts[e]);
            }
            rest -= take;
        }
    }
    s->next_eid += m;
    free(start); free(ord);
    return BS_OK;
}

/* tombstone deletion (section 4.1): layout and pointers stay, validity is cleared */
int bs_delete_edge(bs_store *s, int32_t node, int32_t eid)
{
    if (!s || node < 0 || node >= s->num_nodes) return BS_ERANGE;
    int hit = 0;
    for (bs_block *b = s->nodes[node].head; b; b = b->next)
        for (int64_t i = 0; i < b->size; ++i)
            if (b->eid[i] == eid && b->present[i]) { b->present[i] = 0; hit++; }
    return hit;
}

/* searches counted for bs_walk_counts: one per timestamp a bound search compares */
static int64_t g_unused_probe_sink;

static int64_t lower_pos(const float *ts, int64_t n, float x, int strict, int64_t *probes)
{
    /* first i with ts[i] >= x (strict=0) or ts[i] > x (strict=1) */
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        int ge = strict ? (ts[mid] > x) : (ts[mid] >= x);
        ++*probes;
        if (ge) hi = mid; else lo = mid + 1;
    }
    return lo;
}

static uint64_t bs_pick(uint64_t seed, int64_t q, int32_t f, int32_t j, uint64_t c)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * ((uint64_t)q * (uint64_t)f + (uint64_t)j + 1ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return ((z >> 32) * c) >> 32;
}

typedef struct { const bs_block *b; int64_t lo, hi; } span;   /* candidates [lo, hi) of one block */

/*
 * Phase 1 of Algorithm 1 for one query: the block list of node v is followed from the newest
 * block towards older ones, using only each block's (t_min, t_max).  A block that starts after
 * the window contributes nothing and is passed over; the first block that ends before the
 * window ends the walk, since every older block ends earlier still.  What remains are the blocks
 * overlapping [tb, te], newest first.  `examined` receives the number of blocks whose metadata
 * was looked at.  Returns the number of overlapping blocks, or -1 when out of memory.
 */
static int64_t overlapping(const bs_node *nd, float tb, float te, span **sp, int64_t *cap, int64_t *examined)
{
    int64_t n = 0;
    for (const bs_block *b = nd->tail; b; b = b->prev) {
        ++*examined;
        if (b->t_max < tb) break;
        if (b->t_min > te) continue;
        if (n == *cap) {
            span *n2 = (span *)realloc(*sp, (size_t)(*cap * 2) * sizeof(span));
            if (!n2) return -1;
            *sp = n2; *cap *= 2;
        }
        (*sp)[n].b = b; (*sp)[n].lo = 0; (*sp)[n].hi = 0; n++;
    }
    return n;
}

/* Phase 2: both window bounds are located in a block's sorted timestamps (section 4.1: the
 * sorted order is what allows a logarithmic search). */
static void search_span(span *s, float tb, float te, int inclusive_end, int64_t *probes)
{
    s->lo = lower_pos(s->b->ts, s->b->size, tb, 0, probes);
    s->hi = lower_pos(s->b->ts, s->b->size, te, inclusive_end, probes);
    if (s->hi < s->lo) s->hi = s->lo;
}

static int64_t live_in(const span *s)
{
    int64_t c = 0;
    for (int64_t i = s->lo; i < s->hi; ++i) c += s->b->present[i] ? 1 : 0;
    return c;
}

/* the r-th newest live candidate over the spans (r = 0: the newest) */
static void nth_newest(const span *sp, int64_t n, int64_t r, const bs_block **b, int64_t *i)
{
    for (int64_t t = 0; t < n; ++t)
        for (int64_t x = sp[t].hi - 1; x >= sp[t].lo; --x) {
            if (!sp[t].b->present[x]) continue;
            if (r-- == 0) { *b = sp[t].b; *i = x; return; }
        }
    *b = NULL; *i = -1;
}

/*
 * Algorithm 1 for a batch of queries, in its three phases: the overlapping blocks of the target
 * (walk over block metadata), the candidate range inside each of them (binary searches), the
 * selection of at most f candidates (section 2.1: the newest ones, or uniform picks among all).
 * Deleted edges are not candidates.
 */
int bs_sample(const bs_store *s, int64_t Q, const int32_t *targets, const float *t_start,
              const float *t_end, const int64_t *q_ids, int32_t f, int32_t policy,
              int32_t inclusive_end, uint64_t seed, int32_t *out_nbr, int32_t *out_eid,
              float *out_ts, int32_t *out_count)
{
    if (!s || Q < 0 || f <= 0) return BS_EINVAL;
    int64_t cap = 64;
    span *sp = (span *)malloc((size_t)cap * sizeof(span));
    if (!sp) return BS_ENOMEM;
    for (int64_t q = 0; q < Q; ++q) {
        int64_t v = targets[q], n = 0, c = 0, unused = 0;
        float te = t_end[q], tb = t_start ? t_start[q] : -INFINITY;
        if (v >= 0 && v < s->num_nodes && s->nodes[v].valid && !isnan(te) && !isnan(tb)) {
            n = overlapping(&s->nodes[v], tb, te, &sp, &cap, &unused);
            if (n < 0) { free(sp); return BS_ENOMEM; }
            for (int64_t t = 0; t < n; ++t) {
                search_span(&sp[t], tb, te, inclusive_end, &g_unused_probe_sink);
                c += live_in(&sp[t]);
            }
        }
        int64_t k = c < f ? c : f;
        int64_t qid = q_ids ? q_ids[q] : q;
        for (int64_t j = 0; j < f; ++j) {
            int32_t *on = out_nbr + q * f + j, *oe = out_eid + q * f + j;
            float *ot = out_ts + q * f + j;
            if (j >= k) { *on = -1; *oe = -1; *ot = 0.0f; continue; }
            int64_t r = j;                                   /* distance from the newest candidate */
            if (policy != 0 && c > f)                        /* the pick is a rank counted from the oldest */
                r = c - 1 - (int64_t)bs_pick(seed, qid, f, (int32_t)j, (uint64_t)c);
            const bs_block *b; int64_t i;
            nth_newest(sp, n, r, &b, &i);
            *on = b->nbr[i]; *oe = b->eid[i]; *ot = b->ts[i];
        }
        out_count[q] = (int32_t)k;
    }
    free(sp);
    return BS_OK;
}

/*
 * What the walk of Algorithm 1 touches, summed over a batch of queries (the quantities of a
 * bytes-per-query model): totals[0] = node entries looked up (queries with a valid target),
 * totals[1] = blocks whose metadata is examined, totals[2] = timestamps compared by the bound
 * searches (both bounds in every overlapping block that is searched), totals[3] = edges selected.
 * Under the recent policy the walk ends as soon as f live candidates are known, since older blocks
 * cannot displace them; under the uniform policy every overlapping block is searched.
 */
int bs_walk_counts(const bs_store *s, int64_t Q, const int32_t *targets, const float *t_start,
                   const float *t_end, int32_t f, int32_t policy, int32_t inclusive_end, int64_t *totals)
{
    if (!s || Q < 0 || f <= 0 || !totals) return BS_EINVAL;
    totals[0] = totals[1] = totals[2] = totals[3] = 0;
    for (int64_t q = 0; q < Q; ++q) {
        int64_t v = targets[q];
        float te = t_end[q], tb = t_start ? t_start[q] : -INFINITY;
        if (!(v >= 0 && v < s->num_nodes && s->nodes[v].valid) || isnan(te) || isnan(tb)) continue;
        totals[0]++;
        int64_t c = 0;
        for (const bs_block *b = s->nodes[v].tail; b; b = b->prev) {
            totals[1]++;
            if (b->t_max < tb) break;
            if (b->t_min > te) continue;
            span one = { b, 0, 0 };
            search_span(&one, tb, te, inclusive_end, &totals[2]);
            c += live_in(&one);
            if (policy == 0 && c >= f) break;
        }
        totals[3] += c < f ? c : f;
    }
    return BS_OK;
}

/* list-length and memory figures, the columns of the block-sizing table in section 6.2 */
int bs_stats(const bs_store *s, double *avg_list_len, int64_t *max_list_len, int64_t *num_blocks,
             int64_t *edge_slots, int64_t *edges, int64_t *wasted_slots)
{
    if (!s) return BS_EINVAL;
    int64_t nb = 0, mx = 0, slots = 0, ed = 0;
    for (int64_t v = 0; v < s->num_nodes; ++v) {
        nb += s->nodes[v].nblocks;
        if (s->nodes[v].nblocks > mx) mx = s->nodes[v].nblocks;
        for (bs_block *b = s->nodes[v].head; b; b = b->next) { slots += b->cap; ed += b->size; }
    }
    if (avg_list_len) *avg_list_len = s->num_nodes ? (double)nb / (double)s->num_nodes : 0.0;
    if (max_list_len) *max_list_len = mx;
    if (num_blocks) *num_blocks = nb;
    if (edge_slots) *edge_slots = slots;
    if (edges) *edges = ed;
    if (wasted_slots) *wasted_slots = slots - ed;
    return BS_OK;
}

/*
 * Flatten the layout for inspection: blocks listed node by node, head to tail.
 * Arrays must hold bs_stats().num_blocks entries.  Returns the number written.
 */
int64_t bs_export_blocks(const bs_store *s, int32_t *node, int64_t *cap, int64_t *size,
                         float *t_min, float *t_max)
{
    if (!s) return BS_EINVAL;
    int64_t w = 0;
    for (int64_t v = 0; v < s->num_nodes; ++v)
        for (bs_block *b = s->nodes[v].head; b; b = b->next, ++w) {
            node[w] = (int32_t)v; cap[w] = b->cap; size[w] = b->size;
            t_min[w] = b->t_min; t_max[w] = b->t_max;
        }
    return w;
}

/* edges of one node in list order (head block first); returns the count written (<= max) */
int64_t bs_export_node(const bs_store *s, int32_t v, int64_t max, int32_t *nbr, int32_t *eid, float *ts)
{
    if (!s || v < 0 || v >= s->num_nodes) return BS_ERANGE;
    int64_t w = 0;
    for (bs_block *b = s->nodes[v].head; b; b = b->next)
        for (int64_t i = 0; i < b->size && w < max; ++i, ++w) { nbr[w] = b->nbr[i]; eid[w] = b->eid[i]; ts[w] = b->ts[i]; }
    return w;
}
