// Launch interface between the C ABI (tns_api.hip) and the gfx950 kernels (tns_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "tns_layout.h"

namespace tns {

struct SampleArgs {
    // store (device)
    const NodeLine* nodes;
    const BlockRec* dir;     // directory pool: record runs of nodes with more than kInlineBlocks blocks
    const uint32_t* dir_cum; // same indexing: number of the node's edges stored in the blocks before this one
    const uint32_t* edges;   // edge lines viewed as 4-byte words: slot s starts at word slot_word(s)
    // queries (device)
    const int32_t* targets;
    const float* t_start;        // may be null: -inf
    const float* t_end;
    const int64_t* inst_rowptr;  // may be null: one instance
    // padded outputs (device)
    int32_t* out_nbr;
    int32_t* out_eid;
    float* out_ts;
    int32_t* out_count;
    // non-null: count what the walk reads (node entries, block records, timestamp probes,
    // edges selected) into counters[0..3] instead of producing outputs
    unsigned long long* counters;
    // non-null: also remove the padding in the same pass (chained scan over workgroups);
    // scan_ws is the caller's workspace, rowptr / cmp_* the dense outputs
    void* scan_ws;
    int64_t* rowptr;
    int32_t* cmp_nbr;
    int32_t* cmp_eid;
    float* cmp_ts;
    int64_t Q;               // number of queries, or an upper bound of it when Q_dev is set
    const int64_t* Q_dev;    // may be null; device-resident number of queries (hops after the first)
    int64_t* total_out;      // may be null; fused variant: also receives the dense total (rowptr[Q])
    float delta;             // window length used when t_start is null: t_start = t_end - delta (+inf: unbounded)
    int64_t num_nodes;
    int64_t num_dir;     // records in the directory pool (walks never index past it)
    int64_t qid_base;
    uint64_t seed;
    int32_t num_instances;
    int32_t fanout;
    int32_t policy;
    int32_t inclusive_end;
    int32_t xcd_remap;
    int32_t wide_offsets;  // edge array has 2^31 or more entries: 64-bit positions in LDS
    int32_t first_ticket;  // 0; tests of the chained scan's bounded wait pass 1: tile 0 then never exists
    int32_t scan_ready;    // scan_ws is already cleared (multi-hop: one clearing launch for all hops)
    int32_t prefix_layout; // the store is in the prefix layout: `edges` is the one array of lines, node v's line is line v
    uint32_t* err_flag;    // where a chained scan whose bounded wait ran out reports it (null: the error word of scan_ws)
};

struct CompactArgs {
    const int32_t* nbr;
    const int32_t* eid;
    const float* ts;
    const int32_t* count;
    int64_t* rowptr;
    int32_t* cmp_nbr;
    int32_t* cmp_eid;
    float* cmp_ts;
    int64_t Q;
    const int64_t* Q_dev;    // may be null; device-resident number of queries
    int64_t* total_out;      // may be null; also receives the dense total
    int32_t fanout;
    void* workspace;
};

constexpr int kCompactTile = 1024;  // queries per compaction tile

size_t compact_workspace_bytes(int64_t Q);

// Both only enqueue kernels on `stream`; they return the first launch error.
hipError_t launch_sample(const SampleArgs& a, hipStream_t stream);
// The same for a store in the prefix layout (tns_kernels_prefix.hip); launch_sample forwards to it.
hipError_t launch_sample_prefix(const SampleArgs& a, hipStream_t stream);
// Clears the chained scan's state for `num_tiles` tiles before a fused launch (kernel, capturable).
hipError_t launch_scan_init(const SampleArgs& a, int64_t num_tiles, hipStream_t stream);
hipError_t launch_compact(const CompactArgs& a, hipStream_t stream);
// Clears `bytes` (a multiple of 8) of chained-scan workspace with a kernel (capturable, unlike a memset).
hipError_t launch_scan_clear(void* ws, size_t bytes, hipStream_t stream);
hipError_t launch_hop_inst_rowptr(const int64_t* cur, const int64_t* rowptr, int32_t num_instances, int64_t* next,
                                  hipStream_t stream);

}  // namespace tns
