/*
 * tns_cache -- vectorised dynamic feature cache on one AMD MI355X (gfx950).
 *
 * Follows GNNFlow (arXiv 2311.17410), section 4.3 "Vectorized cache": a GPU-resident cache of
 * node or edge feature rows whose entries are looked up and updated a whole batch at a time.
 * LRU keeps one "recent score" per entry (0 = most recent; every update decrements all scores,
 * an access resets the entry's score to 0, the lowest scores are evicted); LFU keeps an access
 * count instead; FIFO is a ring buffer.  At most floor(lambda * capacity) entries are replaced
 * per update (the paper's default lambda is 0.2).
 *
 * Readings where the paper is silent (the same as the CPU oracle's):
 *   - a batch is looked up against the cache as it was before the batch;
 *   - a fetch always returns the true row (hit: from the cache, miss: from the backing store);
 *   - every occurrence of a cached id counts as an access; a missed id is inserted once, missed
 *     ids are taken in the order of their first occurrence in the batch;
 *   - victims: the entries with the lowest score, ties by the lower slot index (empty slots
 *     compete like any other entry); the i-th victim in ascending slot order receives the i-th
 *     missed id; a new entry starts with score 0 (LRU) or 1 (LFU).
 *
 * Plain C ABI; DEVICE pointers are caller-owned HIP allocations, HOST pointers ordinary host
 * memory.  Functions return 0 (TNS_OK) or a negative tns_status (include/tns.h); details via
 * tns_last_error().  One caller at a time per cache; calls on one cache must be stream-ordered.
 */
#ifndef TNS_CACHE_H
#define TNS_CACHE_H

#include "tns.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tns_cache tns_cache;

enum { TNS_CACHE_LRU = 0, TNS_CACHE_LFU = 1, TNS_CACHE_FIFO = 2 };

typedef struct {
    int64_t num_ids;   /* ids are 0 .. num_ids-1 (nodes or edges)                                  */
    int64_t capacity;  /* number of rows the cache holds, >= 1                                      */
    int32_t dim;       /* floats per row                                                            */
    int32_t policy;    /* TNS_CACHE_LRU | TNS_CACHE_LFU | TNS_CACHE_FIFO                            */
    float lambda;      /* 0 < lambda <= 1: at most floor(lambda * capacity) replacements per update  */
    int32_t device;    /* HIP device ordinal                                                        */
} tns_cache_config;

/* Allocates the cache on the device (rows, id <-> slot maps, scores) and empties it. */
TNS_API int tns_cache_create(const tns_cache_config *cfg, tns_cache **out);

/* Bytes of DEVICE workspace tns_cache_fetch needs for batches of up to B ids. */
TNS_API int tns_cache_workspace(const tns_cache *cache, int64_t B, size_t *bytes);

/*
 * Fetch the rows of a batch of ids and update the cache (one "update" of section 4.3).
 *
 *   d_ids[B]      DEVICE; ids outside [0, num_ids) return a row of zeros and are not cached
 *   store         [num_ids * dim] floats, row-major, readable from the device (device memory or
 *                 pinned host memory): the backing feature store, read for misses
 *   d_out[B*dim]  DEVICE; row b receives the features of d_ids[b]
 *   d_hit[B]      DEVICE, may be NULL; 1 if the row came from the cache
 *   d_workspace   at least tns_cache_workspace() bytes, 256-byte aligned
 * Only enqueues work; never allocates or blocks.  Part of the update runs on a stream the cache owns,
 * forked from hip_stream after the lookup and joined back before the insertion (event record / wait), so
 * to the caller everything is ordered on hip_stream, also when hip_stream is being captured into a graph.
 */
TNS_API int tns_cache_fetch(tns_cache *cache, int64_t B, const int32_t *d_ids, const float *store, float *d_out,
                            uint8_t *d_hit, void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Cumulative counters (waits for the stream): row hits, row misses, entries replaced.  Any may be NULL. */
TNS_API int tns_cache_stats(tns_cache *cache, void *hip_stream, int64_t *hits, int64_t *misses, int64_t *replaced);

/*
 * Cache reuse and restoration (section 4.3): copy the cache contents to HOST buffers (id per
 * slot [capacity], score per slot [capacity], rows [capacity*dim], ring position) and load them
 * back later, e.g. at the start of every epoch.  Both wait for the stream.
 */
TNS_API int tns_cache_save(tns_cache *cache, void *hip_stream, int32_t *h_id_of, int32_t *h_score, float *h_rows,
                           int64_t *h_ring);
TNS_API int tns_cache_restore(tns_cache *cache, void *hip_stream, const int32_t *h_id_of, const int32_t *h_score,
                              const float *h_rows, int64_t ring);

TNS_API int tns_cache_destroy(tns_cache *cache);

#ifdef __cplusplus
}
#endif
#endif /* TNS_CACHE_H */
