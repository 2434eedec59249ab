// Record layouts shared by the host-side store builder and the device kernels.
//
// The paper (section 4.1) lists what a node entry and an edge block hold but not their byte
// layout (it only gives the size of a block's metadata) and links a node's blocks into a doubly-linked
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

// ---- prefix layout (TNS_FLAG_PREFIX_LAYOUT) ------------------------------------------------------
//
// A second placement of the same logical structure (node table, chronological block lists, block
// capacities by the sizing rule of section 4.1), made to cut the number of 128-byte lines a query
// touches.  Node table and edge data share ONE array of 128-byte lines of 10 slot positions each, so
// that every edge is addressed by one slot index whatever line it lives in:
//
//   * line v (v < number of nodes) is node v's line: slot positions 0..7 hold the node's first eight
//     edge slots, the last 32 bytes (slot positions 8, 9 and the line's spare 8 bytes) the node entry;
//   * a node's first blocks are carved, in order, out of its "prefix": 38 consecutive slots = the 8
//     slots in its own line plus up to three extension lines of 10 (allocated when a block reaches
//     into them, never moved).  A block belongs to the prefix while the capacities so far fit; the
//     first block that does not fit, and every later one, is placed on its own as in the default
//     layout and gets a 16-byte record in the node's run of the directory pool;
//   * inside the prefix, blocks are contiguous and all but the newest are full, so edge i of the node
//     sits in prefix slot i: the time index over the prefix is one fence per extension line (the
//     timestamp of its first slot), kept in the node entry.  Block capacities of prefix blocks are
//     needed by insertion and inspection only and stay on the host.
constexpr int kInlineSlots = 8;                                    // edge slots in the node's own line
constexpr int kPrefixExtLines = 3;                                 // extension lines of the prefix
constexpr int kPrefixSlots = kInlineSlots + kPrefixExtLines * kSlotsPerLine;   // 38

// Node entry = words 24..31 of the node's line.
constexpr int kNodeHdrWord = 24;
struct PrefixNodeHdr {
    int32_t degree;      // stored edges
    uint32_t meta;       // bit 0: node deleted; bit 1: node holds deleted edges; bits 2-3: extension lines that
                         // hold edges; bits 4-9: slots of the prefix given to blocks; bits 10-31: blocks outside the prefix
    uint32_t ext0;       // line index of the first extension line
    uint32_t ext12;      // line index of the second extension line; the third follows it
    float fence[kPrefixExtLines];   // timestamp of the first slot of each extension line
    uint32_t dir_line;   // blocks outside the prefix: start of the node's record run, in units of kDirAlign records
};
static_assert(sizeof(PrefixNodeHdr) == 32, "node entry is 32 bytes");
TNS_HD int32_t pmeta_ext_lines(uint32_t m) { return (int32_t)((m >> 2) & 3u); }
TNS_HD int32_t pmeta_prefix_slots(uint32_t m) { return (int32_t)((m >> 4) & 63u); }
TNS_HD int32_t pmeta_big_blocks(uint32_t m) { return (int32_t)(m >> 10); }
TNS_HD uint32_t make_pmeta(uint32_t flags, int32_t ext_lines, int32_t prefix_slots, int32_t big_blocks) {
    return (flags & 3u) | ((uint32_t)ext_lines << 2) | ((uint32_t)prefix_slots << 4) | ((uint32_t)big_blocks << 10);
}
constexpr int32_t kMaxBigBlocks = (1 << 22) - 1;
// A line of the prefix layout's array, seen as edge data or as a node's line.
struct alignas(128) PrefixNodeLine {
    Edge e[kInlineSlots];
    PrefixNodeHdr hdr;
};
union alignas(128) StoreLine {
    EdgeLine edges;
    PrefixNodeLine node;
};
static_assert(sizeof(StoreLine) == 128, "a line is 128 bytes");

}  // namespace tns
