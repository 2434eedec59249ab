// Launch interface of the device-side store builder (tns_ingest.hip): edge insertion of the
// paper's section 4.1 (append to the tail block, else a new block sized by the adaptive rule
// and linked at the tail) and tombstone deletion, run on the GPU on batches that already live
// in device memory.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "tns_layout.h"

namespace tns {

// Per-node builder state that sampling never reads (the host builder keeps the same fields in
// host vectors).
struct NodeAux {
    int32_t tail_cap;    // capacity of the node's newest block
    uint32_t slab_line;  // edge line that takes the node's next small block, + 1 (0: none)
    int32_t slab_used;   // slots of that line already given to blocks
    int32_t dir_cap;     // records reserved for the node in the directory pool (0: inline)
};
static_assert(sizeof(NodeAux) == 16, "16 bytes per node");

// Device-resident result of the planning phase, read back by the host before anything is changed.
struct IngestStatus {
    unsigned long long err_word;  // ~0: no error; else (position << 8 | -status), the smallest wins
    uint32_t unsorted;            // batch timestamps are not non-decreasing in arrival order
    uint32_t internal;            // a kernel found a pool too small (never expected: the host sizes them)
    int64_t num_segments;         // distinct source nodes in the batch
    int64_t total_lines;          // edge lines the new blocks need
    int64_t total_dir;            // directory records the new runs need
    unsigned long long new_blocks;
    unsigned long long new_slots; // sum of the new blocks' capacities
    unsigned long long counter;   // deletion: edges whose validity was cleared; statistics: longest list
};
static_assert(sizeof(IngestStatus) == 64, "one 64-byte record");

struct IngestArgs {
    // batch (device)
    const int32_t* src;
    const int32_t* dst;
    const float* ts;
    const int32_t* eid;   // may be null: eid_base + batch position
    int64_t m;
    int64_t eid_base;
    // store (device)
    NodeLine* nodes;
    NodeAux* aux;
    BlockRec* dir;
    uint32_t* dir_cum;    // per directory record: the node's edges in older blocks
    uint32_t* lines;      // edge lines as 4-byte words
    int64_t node_base;    // instance * num_nodes
    int64_t num_nodes;
    int64_t used_lines, cap_lines;   // edge lines in use before the batch / allocated
    int64_t used_dir, cap_dir;       // directory records likewise
    int32_t tau;
    int32_t sizing;
    // scratch
    void* workspace;      // ingest_workspace_bytes(m)
    IngestStatus* status;
    // optional (short pipeline only): a copy of *status in page-locked host memory that the device can write, and a
    // sequence word next to it; the plan's last workgroup copies the record there and then stores `seq`, so that
    // the host can pick the plan up by polling instead of waiting for the stream
    IngestStatus* host_status;
    unsigned long long* host_seq;
    unsigned long long seq;
};

constexpr int64_t kMaxDeviceBatch = kMaxBlockEdges;   // one new block always takes the rest of a node's share

size_t ingest_workspace_bytes(int64_t m);

// Phase 1: validate, sort by (source, time, arrival), find the per-node segments, check the order
// against what is stored, and compute what every node needs (edge lines, directory records).
// Changes nothing in the store.  The host then reads *status, makes room, and runs phase 2.
hipError_t ingest_plan(const IngestArgs& a, hipStream_t stream);
// The same phase in five launches for batches of stream size (at most 2^21 edges, at most 2^24 nodes) that
// arrive in time order: it sorts by source only and reports status->unsorted when the batch was not in time
// order, in which case the caller runs ingest_plan instead.  Expects *status reset (ingest_apply leaves it so).
bool ingest_fast_ok(int64_t m, int64_t num_nodes);
hipError_t ingest_plan_fast(const IngestArgs& a, hipStream_t stream);
// Phase 2: update node entries and block records, write the edges (num_segments as read from *status; `fast`:
// the plan came from ingest_plan_fast).  Its first kernel resets *status for the next batch, except the sticky
// `internal` word, which the next read of *status reports.
hipError_t ingest_apply(const IngestArgs& a, int64_t num_segments, bool fast, hipStream_t stream);

// Tombstone deletion on the device store: requests (node, edge id) [n]; status->counter receives the hits.
hipError_t ingest_delete_edges(NodeLine* nodes, BlockRec* dir, uint32_t* lines, int64_t node_base, const int32_t* src,
                               const int32_t* eid, int64_t n, IngestStatus* status, hipStream_t stream);
hipError_t ingest_delete_nodes(NodeLine* nodes, int64_t node_base, const int32_t* ids, int64_t n, int32_t deleted,
                               hipStream_t stream);
// status->counter = longest block list among nodes [first, first + count)
hipError_t ingest_max_list_len(const NodeLine* nodes, int64_t first, int64_t count, IngestStatus* status,
                               hipStream_t stream);
hipError_t ingest_status_reset(IngestStatus* status, hipStream_t stream);

}  // namespace tns
