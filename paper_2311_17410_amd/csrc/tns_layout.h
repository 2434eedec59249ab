// Record layouts shared by the host-side store builder and the device kernels.
//
// The paper (section 4.1) lists what a node entry and an edge block hold but not their byte
// layout ("lightweight structures (72 bytes)"), so the layout here is chosen for 64-byte HBM
// sectors: a node entry is 16 bytes, a block record 32 bytes (two per sector, never
// straddling one), an edge 12 bytes with timestamp, neighbour and edge id side by side so that
// the timestamps probed by the in-block search and the ids gathered afterwards share sectors.
// Pointers are 32-bit block indices and 64-bit edge offsets into flat device arrays.
#pragma once
#include <cstdint>

namespace tns {

// Node table entry (section 4.1: last block of the list, list length, degree, validity).
// The first block is reachable through the prev links and is kept on the host side only.
struct NodeRec {
    int32_t tail;     // index of the newest block, -1 if the node has no edge
    int32_t nblocks;  // list length
    int32_t degree;   // stored edges (out-degree)
    int32_t flags;    // bit 0: node deleted
};
static_assert(sizeof(NodeRec) == 16, "node entry is 16 bytes");

// Edge block metadata (section 4.1: capacity, fill, where the edge data is, earliest and
// latest timestamp; prev/next links of the chronological doubly-linked list).
struct BlockRec {
    float t_min, t_max;  // earliest / latest edge time in the block
    int32_t size, cap;   // edges held / block size
    int64_t off;         // offset of the block's first edge in the edge array
    int32_t prev, next;  // older / newer block of the same node, -1 at the ends
};
static_assert(sizeof(BlockRec) == 32, "block record is 32 bytes");

// One entry of the graph edge data.  Inside a block, entries are in (timestamp, arrival) order.
struct Edge {
    float ts;
    int32_t nbr;
    int32_t eid;
};
static_assert(sizeof(Edge) == 12, "edge entry is 12 bytes");

}  // namespace tns
