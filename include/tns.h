/*
 * tns -- one-hop temporal neighbourhood sampling over a time-indexed, block-based dynamic
 * graph store, on one AMD MI355X (gfx950).
 *
 * The operations follow GNNFlow (arXiv 2311.17410):
 *   - the store is the node table + per-node chronological list of edge blocks of
 *     section 4.1, with the block size rule b_v = min(deg(v), tau) (the paragraph on adaptive
 *     block sizing);
 *   - tns_run executes Algorithm 1 (section 4.2) for a batch of queries, with the recent
 *     and uniform selection policies of section 2.1, writes the padded per-target result the
 *     way the kernel-optimization paragraph of section 4.2 asks for (consecutive slots per
 *     target) and optionally removes the padding (section 5, the paragraph on GPU sampling).
 *
 * Conventions
 *   - Plain C ABI.  Every pointer argument is marked HOST or DEVICE.  DEVICE pointers are
 *     ordinary HIP device allocations owned by the caller (e.g. torch tensors); HOST
 *     pointers are ordinary host memory.  The library keeps no reference to any caller
 *     buffer after a call returns (tns_run: after the work queued on the stream is done).
 *   - ids are int32, timestamps are IEEE fp32, offsets are int64.
 *   - All functions return 0 (TNS_OK) or a negative tns_status.  A failing call leaves the
 *     plan unchanged.  tns_last_error() gives a human-readable detail for the last failure
 *     on the calling thread.
 *   - A plan is not thread-safe: one caller at a time.  tns_run only enqueues work on the
 *     given stream and never blocks on the device, allocates or frees.
 */
#ifndef TNS_H
#define TNS_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define TNS_API __attribute__((visibility("default")))
#else
#define TNS_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tns_plan tns_plan; /* opaque: host-side store builder + device store */

typedef enum {
    TNS_OK = 0,
    TNS_EINVAL = -1, /* null pointer, negative size, fanout out of range, bad enum value   */
    TNS_EORDER = -2, /* NaN edge time, or a batch older than what a node already stores    */
    TNS_ERANGE = -3, /* source node id or instance outside the configured range            */
    TNS_ENOMEM = -4, /* host or device allocation failed                                   */
    TNS_EHIP = -5,   /* HIP runtime error (no device, launch failure, ...)                 */
    TNS_ESTATE = -6, /* tns_run before the first tns_commit; host batch for a device-built store
                        or the reverse                                                      */
    TNS_ESIZE = -7   /* workspace too small, or a size beyond a documented limit           */
} tns_status;

enum { TNS_POLICY_RECENT = 0, TNS_POLICY_UNIFORM = 1 };
enum { TNS_SIZING_ADAPTIVE = 0, TNS_SIZING_STRAWMAN = 1, TNS_SIZING_FIXED = 2 };
enum { TNS_MAX_FANOUT = 64 };
/* tns_config.flags */
enum {
    TNS_FLAG_NO_XCD_REMAP = 1, /* keep the hardware's round-robin workgroup->XCD order (for measurements) */
    TNS_FLAG_NO_NODE_SLAB = 2, /* do not reserve one 128-byte edge line per non-empty node for its first
                                  blocks: less memory for graphs of mostly degree-1 nodes, more lines
                                  read per query                                                        */
    /* Placement (section 4.1, the paragraph on placing graph data across GPU and CPU memory).  Default: node table, block
       records and edge data all in device memory.  EDGES_ON_HOST is the paper's hybrid placement:
       the metadata (node table, block records) in device memory, the edge data in page-locked host
       memory that the kernels read across the host link.  ALL_ON_HOST puts the metadata there too
       (the all-in-host-memory comparison point of the paper's sampling ablation).  Results are identical under all three. */
    TNS_FLAG_EDGES_ON_HOST = 4,
    TNS_FLAG_ALL_ON_HOST = 8,
    /* The store is built on the device: batches come from device memory through
       tns_add_edges_device and are visible to the next tns_run on the same stream; there is no
       host copy, tns_add_edges is refused (TNS_ESTATE) and tns_commit has nothing to upload.
       Cannot be combined with the host placements or TNS_FLAG_NO_NODE_SLAB. */
    TNS_FLAG_DEVICE_INGEST = 16,
    /* Keep edge positions as 64-bit values inside the kernels even while the edge array is small.  The
       library switches to them by itself once the array passes 2^31 four-byte words (8 GiB); the
       flag exists so that tests reach that code without such a store. */
    TNS_FLAG_WIDE_POSITIONS = 32,
    /* (64 is taken by a hook of the library's own tests.)
       Prefix layout: another placement of the same store (section 4.1 fixes what a node entry and a
       block hold, not where they lie).  A node's first eight edge slots share the 128-byte line of
       its table entry and its next thirty sit in up to three lines found from that entry, so that a
       query on a node of a few dozen edges reads one to three lines.  Block capacities, list
       lengths, tns_stats and tns_node_blocks are those of the default layout; sampling results are
       identical.  Host-built, device-resident stores only (not with the host placements,
       TNS_FLAG_DEVICE_INGEST or TNS_FLAG_NO_NODE_SLAB). */
    TNS_FLAG_PREFIX_LAYOUT = 128
};

typedef struct {
    int64_t num_nodes;       /* |V| per instance; node ids are 0 .. num_nodes-1                */
    int32_t num_instances;   /* >= 1 independent graphs sharing this plan (ids are per instance) */
    int32_t fanout;          /* f: neighbours sampled per target, 1 .. TNS_MAX_FANOUT (Alg. 1 input) */
    int32_t policy;          /* TNS_POLICY_RECENT | TNS_POLICY_UNIFORM             (section 2.1) */
    int32_t block_threshold; /* tau >= 1 of b_v = min(deg(v), tau)                 (section 4.1) */
    int32_t sizing;          /* TNS_SIZING_*: adaptive is the paper's method; strawman and fixed
                                are the comparison methods of section 6.2 (layout tests)        */
    int32_t inclusive_end;   /* 0: window [t_s, t_e) as in Algorithm 1; 1: [t_s, t_e] as in
                                section 2.1                                                    */
    uint64_t seed;           /* uniform policy: key of the counter-based generator             */
    int32_t device;          /* HIP device ordinal used by tns_commit / tns_run                */
    int32_t flags;           /* TNS_FLAG_* bits, 0 for defaults                                */
} tns_config;

/*
 * Create an empty store (section 4.1: node table with one entry per node, no blocks).
 * Touches no GPU; the device is first used by tns_commit.  *out receives the plan.
 */
TNS_API int tns_plan_create(const tns_config *cfg, tns_plan **out);

/*
 * Change the sampler settings of an existing plan without touching the store (the paper keeps
 * the dynamic graph and the sampler apart: one graph can serve samplers with different fan-outs
 * and policies).  Same value ranges as in tns_config; takes effect for the next tns_run.
 */
TNS_API int tns_set_sampler(tns_plan *plan, int32_t fanout, int32_t policy, int32_t inclusive_end, uint64_t seed);

/*
 * Ingest one batch of m edges into instance `instance` (section 4.1, edge insertion: append
 * to the node's tail block while it has room, otherwise link a new block at the tail; the
 * new block's capacity is max(remaining edges of this batch for the node,
 * min(degree so far, tau))).  All arrays are HOST, length m, in arrival order; the edge
 * src[i] -> dst[i] is stored with its source node (directed storage; store both directions
 * yourself for an undirected graph).  eid may be NULL: ids then continue a per-instance
 * running counter; given ids must be >= 0 (TNS_EINVAL otherwise).  Inside the batch a node's edges are put in timestamp order (stable);
 * TNS_EORDER if a node would receive an edge older than its newest stored edge or a NaN
 * time, TNS_ERANGE for src outside [0, num_nodes).  Nothing is visible to tns_run until
 * tns_commit.
 */
TNS_API int tns_add_edges(tns_plan *plan, int32_t instance, const int32_t *src, const int32_t *dst,
                  const float *ts, const int32_t *eid, int64_t m);

/*
 * The same insertion (section 4.1) for a plan created with TNS_FLAG_DEVICE_INGEST, run on the GPU:
 * all arrays are DEVICE, length m <= 2^24-1, d_eid may be NULL.  The batch is sorted by (source,
 * time, arrival) on the device, every source node's share is appended to its tail block and, if
 * edges remain, to new blocks sized by the same rule as tns_add_edges; block capacities, sizes and
 * time ranges per node are identical to the host builder's, only where the blocks lie in the edge
 * array differs.  Same status codes; a rejected batch changes nothing.  The call grows the
 * device pools when needed (it may allocate) and waits for the stream once, to read the batch's
 * plan; it returns with the kernels that write the batch queued on hip_stream: a later tns_run
 * on that stream sees the batch, work on another stream has to wait for hip_stream first.  No
 * tns_commit is needed.  An error of the library itself (TNS_EHIP: a pool found too small by those
 * kernels, a bounded wait that ran out) is reported by the next call that reads the builder's
 * status, at the latest the next tns_add_edges_device.
 */
TNS_API int tns_add_edges_device(tns_plan *plan, int32_t instance, const int32_t *d_src, const int32_t *d_dst,
                                 const float *d_ts, const int32_t *d_eid, int64_t m, void *hip_stream);

/*
 * Tombstone deletion (section 4.1: validity fields are cleared while data layouts and pointers
 * are preserved; invalid nodes and edges are ignored during sampling).
 *
 * tns_delete_edges: HOST arrays of m (source node, edge id) pairs of instance `instance`.  A
 * deleted edge is treated as absent by every later tns_run (after the next tns_commit): it is
 * neither counted as a candidate nor returned.  *num_deleted (may be NULL) receives how many
 * stored edges matched.  Edge ids must therefore be non-negative (tns_add_edges rejects negative
 * ids): the store marks a deleted edge by complementing its id.  Cost: a scan of the node's
 * edges per pair on the host; on the device, a query that meets a block holding deleted edges
 * checks that block's candidates one by one, and once a plan has deleted an edge tns_run removes
 * the padding in a step of its own (sampling kernel, then the kernels of tns_compact) instead of in
 * the sampling kernel: a slow query then delays nothing but itself.  tns_run_khop keeps the one-pass
 * form and reports a time-out through tns_run_status.  For a store built on the device
 * (TNS_FLAG_DEVICE_INGEST) both calls copy the requests over, apply them with a kernel on the
 * default stream and wait for it: they take effect at once, without tns_commit.
 *
 * tns_delete_nodes: HOST array of m node ids; a deleted node (deleted != 0) returns no neighbours
 * as a target; deleted = 0 restores it.  Edges that point TO a deleted node are not filtered:
 * delete them with tns_delete_edges.
 */
TNS_API int tns_delete_edges(tns_plan *plan, int32_t instance, const int32_t *src, const int32_t *eid,
                             int64_t m, int64_t *num_deleted);
TNS_API int tns_delete_nodes(tns_plan *plan, int32_t instance, const int32_t *nodes, int64_t m, int32_t deleted);

/*
 * Section 3 (system overview): the store is not changed while a training round samples from it;
 * new data is buffered and becomes visible at a defined point.  tns_commit is that point.
 * Make everything ingested so far visible to tns_run: uploads the changed parts of the
 * node table, block records and edge data to the device (allocating or growing device
 * memory as needed) on `hip_stream` (a hipStream_t, NULL = default stream) and waits for
 * the upload.  For a store built on the device there is nothing to upload; the call only makes
 * sure the (possibly empty) store exists.
 */
TNS_API int tns_commit(tns_plan *plan, void *hip_stream);

/* Bytes of DEVICE workspace tns_run needs for Q queries when the padding removal of section 5 is requested
   (scan state of that step; the first 256 bytes hold the step's status word, see tns_run_status). */
TNS_API int tns_workspace(const tns_plan *plan, int64_t Q, size_t *bytes);

/*
 * Sample Q queries (Algorithm 1).  All d_* pointers are DEVICE.
 *
 *   d_targets[Q]      target node of each query (per-instance id); ids outside
 *                     [0, num_nodes) and deleted nodes give count 0
 *   d_t_start[Q]      window start, or NULL for -infinity
 *   d_t_end[Q]        window end (open or closed per config.inclusive_end); NaN gives count 0
 *   d_inst_rowptr     NULL when num_instances == 1; else [num_instances+1] non-decreasing query
 *                     offsets, d_inst_rowptr[0] = 0, d_inst_rowptr[num_instances] = Q:
 *                     queries d_inst_rowptr[b] .. d_inst_rowptr[b+1]-1 address instance b
 *   query_id_base     id of query 0 for the uniform policy's generator (query i has id
 *                     query_id_base + i); lets a long batch be run in pieces
 *   d_out_nbr/eid/ts  [Q*fanout] padded result, row-major by query: slot j < count holds the
 *                     neighbour id, edge id and timestamp of one sampled edge (recent: newest
 *                     first; uniform: draw order); slots >= count hold -1, -1, 0.0f
 *   d_out_count[Q]    number of filled slots per query, min(fanout, candidates)
 *                     All four padded outputs may be NULL together when the padding is removed in
 *                     the same kernel (d_rowptr given, edge data in device memory, no deleted
 *                     edges; TNS_EINVAL otherwise): the padded rows are then never written, only
 *                     the dense result is (the counts are d_rowptr[q+1] - d_rowptr[q])
 *   d_rowptr[Q+1], d_cmp_nbr/eid/ts[sum of counts]
 *                     padding removed: exclusive prefix sum of counts and the filled slots in
 *                     (query, slot) order.  d_rowptr NULL (and the other three NULL) skips
 *                     this step; the compacted arrays need room for Q*fanout entries in the
 *                     worst case
 *   d_workspace       at least tns_workspace() bytes, 256-byte aligned; may be NULL when
 *                     compaction is skipped
 *   hip_stream        hipStream_t on the plan's device (NULL = default stream)
 *
 * TNS_ESTATE before the first commit, TNS_ESIZE for a short workspace, TNS_EINVAL for
 * missing pointers, TNS_EHIP if a launch fails.
 *
 * With compaction (and the edge data in device memory) both steps run in one kernel whose workgroups pass their dense
 * offsets along a chain; a workgroup waits for its predecessors for a bounded time only (about two
 * seconds).  Should that bound ever be hit, tns_run_status reports it once the stream's work is done:
 * the dense outputs are then invalid and d_rowptr[Q] reads 0 (the padded outputs are not affected).
 */
TNS_API int tns_run(tns_plan *plan, int64_t Q, const int32_t *d_targets, const float *d_t_start,
            const float *d_t_end, const int64_t *d_inst_rowptr, int64_t query_id_base,
            int32_t *d_out_nbr, int32_t *d_out_eid, float *d_out_ts, int32_t *d_out_count,
            int64_t *d_rowptr, int32_t *d_cmp_nbr, int32_t *d_cmp_eid, float *d_cmp_ts,
            void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Whether a bounded wait of the padding removal ran out in the last tns_run, tns_compact, tns_run_khop
 * (any hop; the following hops then had no queries) or tns_run_static that used `d_workspace` (DEVICE;
 * NULL = the static scratch of tns_run_static on the plan's device).  Waits for `hip_stream`, copies one
 * word to the host; *timed_out (HOST) receives 0 or 1.  Not a step of the paper's method: the error
 * report of this implementation's single-pass scan.
 */
TNS_API int tns_run_status(tns_plan *plan, const void *d_workspace, void *hip_stream, int32_t *timed_out);

/*
 * For callers that cannot allocate device memory or own no workspace (code under HIP graph capture,
 * serving loops, harnesses that forbid allocation): tns_run with padding removal (d_rowptr and the
 * dense arrays are required), its scan state kept in a static device array of the library instead of
 * a caller's workspace.  Arguments and results as tns_run.  At most 2^24 queries per call (TNS_ESIZE
 * beyond; the array is 2 MiB + 512 bytes per GPU, held until the process ends).  Calls no allocation
 * routine.  All calls on one GPU share the array: calls that overlap in time on one GPU (different
 * streams, different plans) race; on one stream they are ordered.  Status: tns_run_status with a NULL
 * workspace.
 */
TNS_API int tns_run_static(tns_plan *plan, int64_t Q, const int32_t *d_targets, const float *d_t_start,
            const float *d_t_end, const int64_t *d_inst_rowptr, int64_t query_id_base,
            int32_t *d_out_nbr, int32_t *d_out_eid, float *d_out_ts, int32_t *d_out_count,
            int64_t *d_rowptr, int32_t *d_cmp_nbr, int32_t *d_cmp_eid, float *d_cmp_ts, void *hip_stream);

/*
 * Multi-hop sampling (section 4.2: the process is repeated per layer, the nodes sampled in one
 * layer being the targets of the next).  Hop 1 samples the given queries exactly as tns_run;
 * hop h+1 has one query per dense entry of hop h, in dense order: target = the sampled
 * neighbour, window end = the timestamp of the sampled edge, window start = end - delta
 * (delta = +infinity: unbounded).  A temporal random walk is the special case fanouts = 1,1,...
 *
 *   fanouts[num_hops]   HOST; each in 1..TNS_MAX_FANOUT (the plan's own fan-out is not used)
 *   hops[num_hops]      HOST array of DEVICE buffer sets; rowptr and the three dense arrays are required,
 *                       the four padded outputs of a hop (nbr, eid, ts, count) may be NULL together: the hop
 *                       then writes its dense result only, which is all the next hop reads.  With
 *                       cap_1 = Q and cap_{h+1} = cap_h * fanouts[h] (the most queries hop h can
 *                       have), hop h needs nbr/eid/ts[cap_h * fanouts[h]], count[cap_h],
 *                       rowptr[cap_h + 1], cmp_nbr/eid/ts[cap_h * fanouts[h]].  Only the entries
 *                       of the hop's actual queries are written; their number n_h is
 *                       rowptr_{h-1}[n_{h-1}] (n_1 = Q) and rowptr_h[n_h] closes the hop.
 *   query ids (uniform policy): hop h numbers its queries from
 *                       query_id_base + cap_1 + ... + cap_{h-1}
 *   d_workspace         at least tns_workspace_khop() bytes, 256-byte aligned
 * Nothing is copied to the host between hops; the whole sequence is queued on the stream.
 */
typedef struct {
    int32_t *nbr, *eid;
    float *ts;
    int32_t *count;
    int64_t *rowptr;
    int32_t *cmp_nbr, *cmp_eid;
    float *cmp_ts;
} tns_hop_buffers;
TNS_API int tns_workspace_khop(const tns_plan *plan, int32_t num_hops, const int32_t *fanouts, int64_t Q,
                               size_t *bytes);
TNS_API int tns_run_khop(tns_plan *plan, int32_t num_hops, const int32_t *fanouts, float delta, int64_t Q,
                         const int32_t *d_targets, const float *d_t_start, const float *d_t_end,
                         const int64_t *d_inst_rowptr, int64_t query_id_base, const tns_hop_buffers *hops,
                         void *d_workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Padding removal alone (section 5: after each sampling kernel the invalid neighbours are
 * removed): the second half of tns_run, for callers that keep the two steps apart.  Reads the
 * padded arrays and counts written by tns_run (DEVICE, same layout) and writes d_rowptr[Q+1]
 * and the dense arrays as described there.  Same workspace and error rules as tns_run.
 */
TNS_API int tns_compact(tns_plan *plan, int64_t Q, const int32_t *d_out_nbr, const int32_t *d_out_eid,
                        const float *d_out_ts, const int32_t *d_out_count, int64_t *d_rowptr,
                        int32_t *d_cmp_nbr, int32_t *d_cmp_eid, float *d_cmp_ts, void *d_workspace,
                        size_t workspace_bytes, void *hip_stream);

/*
 * Byte model of a query batch: runs the walk of tns_run without producing results and adds
 * to d_counters[0..3] (DEVICE, uint64, zeroed by the caller) the number of node entries, block
 * records and edge timestamps the walk reads (Algorithm 1's node lookup, block steps and
 * binary-search probes) and the number of edges it selects.  Query arguments as in tns_run.
 */
TNS_API int tns_traffic_model(tns_plan *plan, int64_t Q, const int32_t *d_targets, const float *d_t_start,
                              const float *d_t_end, const int64_t *d_inst_rowptr, int64_t query_id_base,
                              uint64_t *d_counters, void *hip_stream);

/*
 * Layout figures of one instance (the columns of the block-sizing table in section 6.2):
 * average and maximum block-list length, bytes of edge data (all slots) and of metadata
 * (node table + block records) as stored on the device, number of unfilled edge slots,
 * number of blocks and of stored edges.  instance = -1 sums over all instances.  For a store
 * built on the device the longest list is reduced by a kernel on the default stream (the call
 * waits for it).
 */
typedef struct {
    double avg_list_len;
    int64_t max_list_len;
    int64_t edge_data_bytes;
    int64_t metadata_bytes;
    int64_t wasted_slots;
    int64_t num_blocks;
    int64_t num_edges;
} tns_stats_t;
TNS_API int tns_stats(const tns_plan *plan, int32_t instance, tns_stats_t *out);

/*
 * Inspection of the layout (for tests): the blocks of node `node` of `instance` from the
 * oldest to the newest, from the host builder's copy or, for a store built on the device, read
 * back from device memory.  Arrays are HOST with room for `max_blocks` entries (any
 * may be NULL); returns the node's block count (which may exceed max_blocks) or a negative
 * status.
 */
TNS_API int64_t tns_node_blocks(const tns_plan *plan, int32_t instance, int32_t node, int64_t max_blocks,
                        int32_t *cap, int32_t *size, float *t_min, float *t_max);

/*
 * Measurement aid, not a step of the paper's method: a streaming kernel of exactly known traffic on
 * `hip_stream`.  mode 0 copies `bytes` from d_src to d_dst (reads bytes, writes bytes), 1 only reads
 * d_src (d_dst may be NULL), 2 only writes d_dst (d_src may be NULL); nontemporal != 0 puts the
 * non-temporal hint on the loads and stores, as the sampling kernel does for data it touches once.
 * DEVICE buffers, 16-byte aligned, bytes a multiple of 16.  The bench reports the rates as the box's
 * practical ceiling and counter runs use the launches to calibrate the byte counters.
 */
TNS_API int tns_hbm_probe(int32_t mode, int32_t nontemporal, void *d_dst, const void *d_src, size_t bytes,
                          void *hip_stream);

/*
 * The same aid for a mix of the two directions: reads read_bytes from d_src and writes write_bytes to d_dst
 * in one launch, the shorter stream spread evenly over the longer one, so that the memory system sees the
 * read:write ratio of a kernel under study throughout (the sampling step reads about 1.6 bytes per byte it
 * writes in the default layout, 0.9 in the prefix layout; a plain copy 1.0).  DEVICE buffers, 16-byte aligned,
 * sizes positive multiples of 16 and at most 32 GiB each.
 */
TNS_API int tns_hbm_probe_mix(int32_t nontemporal, void *d_dst, size_t write_bytes, const void *d_src, size_t read_bytes,
                              void *hip_stream);

/* Release the plan (the dynamic graph object of section 5's interface), its host store and its device
   memory.  NULL is allowed. */
TNS_API int tns_destroy(tns_plan *plan);

/* Static description of a status code. */
TNS_API const char *tns_strerror(int status);
/* Detail of the last failure on this thread ("" if none). Valid until the next tns call on the thread. */
TNS_API const char *tns_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TNS_H */
