// Record layouts shared by the host-side store builder and the device kernels.
//
// The paper (section 4.1) lists what a node entry and an edge block hold but not their byte
// layout ("lightweight structures (72 bytes)") and links a node's blocks into a doubly-linked
// list.  On MI355X every dependent random read costs a 128-byte line from HBM, so a linked
// list of separately allocated records costs one line per block visited.  Here the records of
// one node sit next to each other instead:
//
//   * NodeLine (128 bytes, line-aligned): the node entry (list length, degree, validity) plus
//     the records of up to 7 blocks, newest first.  One line read gives Algorithm 1 everything
//     it needs to skip, stop or search for nodes with short lists.
//   * nodes with longer lists keep all their records, oldest first, in one contiguous run of
//     the directory pool; the walk starts with a binary search over it instead of stepping
//     through the newer blocks one by one.
//   * BlockRec (16 bytes): earliest and latest timestamp, number of edges, offset of the
//     block's edges.  The capacity is not needed by sampling: every block but the newest is
//     full, and the newest block's capacity is kept on the host.
//   * Edge (12 bytes): timestamp, neighbour id, edge id side by side, so the timestamps probed
//     by the in-block search and the ids gathered afterwards share lines; ten edges per
//     128-byte line (EdgeLine).
#pragma once
#include <cstdint>

namespace tns {

constexpr int kInlineBlocks = 7;
constexpr int64_t kMaxBlockEdges = (int64_t(1) << 24) - 1;  // size field is 24 bits
constexpr int64_t kMaxEdgeOffset = (int64_t(1) << 39) - 1;  // offset (slot index) field is 39 bits

// Edge block metadata (section 4.1: fill, where the edge data is, earliest and latest time).
struct BlockRec {
    float t_min, t_max;  // earliest / latest edge time in the block
    uint32_t off_lo;     // low 32 bits of the slot index of the block's first edge
    uint32_t size_hi;    // bits 0-23: edges held; bits 24-30: offset bits 32-38; bit 31: block holds deleted edges
};
static_assert(sizeof(BlockRec) == 16, "block record is 16 bytes");

#if defined(__HIPCC__)
#define TNS_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define TNS_HD inline
#endif
TNS_HD int32_t rec_size(const BlockRec& r) { return (int32_t)(r.size_hi & 0xffffffu); }
TNS_HD int64_t rec_off(const BlockRec& r) { return (int64_t)r.off_lo | ((int64_t)((r.size_hi >> 24) & 0x7fu) << 32); }
TNS_HD bool rec_tombstones(const BlockRec& r) { return (r.size_hi >> 31) != 0; }
TNS_HD BlockRec make_rec(float t_min, float t_max, int64_t off, int32_t size, bool tombstones = false) {
    BlockRec r;
    r.t_min = t_min;
    r.t_max = t_max;
    r.off_lo = (uint32_t)(off & 0xffffffffu);
    r.size_hi = ((uint32_t)size & 0xffffffu) | (((uint32_t)(off >> 32) & 0x7fu) << 24) | (tombstones ? 0x80000000u : 0u);
    return r;
}

// Node table entry (section 4.1: list length, degree, validity, access to the blocks).
struct alignas(128) NodeLine {
    int32_t nblocks;   // list length
    int32_t degree;    // stored edges (out-degree)
    uint32_t dir_line; // nblocks > kInlineBlocks: where the node's records start in the directory
                       // pool, in units of kDirAlign records (oldest record first)
    int32_t flags;     // bit 0: node deleted; bit 1: some block of the node holds deleted edges
    BlockRec rec[kInlineBlocks];  // nblocks <= kInlineBlocks: rec[0] newest ... rec[nblocks-1] oldest
};
static_assert(sizeof(NodeLine) == 128, "node entry is one 128-byte line");

constexpr int kDirAlign = 8;  // directory runs start on a 128-byte line

// One entry of the graph edge data.  Inside a block, entries are in (timestamp, arrival) order.
// Edge ids are non-negative; a deleted edge (section 4.1: validity cleared, layout kept) stores the
// bitwise complement of its id, so validity costs no extra word and the id stays recoverable.
struct Edge {
    float ts;
    int32_t nbr;
    int32_t eid;
};
static_assert(sizeof(Edge) == 12, "edge entry is 12 bytes");

// The edge array is made of 128-byte lines of 10 edge slots (8 bytes unused per line), so that
// a block of up to 10 slots allocated at a line start is read with one line, and blocks are
// addressed by slot index: slot s lives in line s / 10 at position s % 10.
constexpr int kSlotsPerLine = 10;
struct alignas(128) EdgeLine {
    Edge e[kSlotsPerLine];
    uint32_t unused[2];
};
static_assert(sizeof(EdgeLine) == 128, "edge line is 128 bytes");

// 4-byte word index of slot s inside the edge array (line * 32 + position * 3)
TNS_HD int64_t slot_word(int64_t s) {
    const int64_t line = s / kSlotsPerLine;
    return line * 32 + (s - line * kSlotsPerLine) * 3;
}

}  // namespace tns
