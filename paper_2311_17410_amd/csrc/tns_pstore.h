// Host-side builder of the block store in the prefix layout (tns_layout.h, "prefix layout"): same
// insertion and sizing rules as tns_store.h (section 4.1 of the paper), other placement.  The host
// arrays are kept in the device layout; a commit copies the parts that changed.  No HIP in this file.
#pragma once
#include <string>
#include <unordered_map>
#include <vector>

#include "tns_store.h"

namespace tns {

class PrefixStore {
public:
    explicit PrefixStore(const StoreConfig& cfg);

    int add_edges(int32_t inst, const int32_t* src, const int32_t* dst, const float* ts, const int32_t* eid,
                  int64_t m, std::string& err);
    int64_t delete_edge(int32_t inst, int32_t v, int32_t e);
    void set_node_deleted(int32_t inst, int32_t v, bool deleted);

    const StoreConfig& config() const { return cfg_; }
    const InstanceTotals& totals(int32_t inst) const { return totals_[inst]; }
    int64_t node_index(int32_t inst, int64_t v) const { return (int64_t)inst * cfg_.num_nodes + v; }
    int64_t total_nodes() const { return total_nodes_; }
    int32_t num_blocks(int64_t nidx) const { return nblocks_[(size_t)nidx]; }
    // i-th block of a node in chronological order (0 = oldest): capacity, fill, earliest and latest time
    void block_info(int64_t nidx, int32_t i, int32_t* cap, int32_t* size, float* t_min, float* t_max) const;

    // One array of 128-byte lines: lines 0 .. total_nodes-1 are the node lines, edge lines follow.
    Paged<StoreLine, 18, 9> lines;
    Paged<BlockRec> dir;            // records of the blocks outside the prefixes, one run per node, oldest first
    Paged<uint32_t> dir_cum;        // same indexing: edges of the node stored before this block (prefix included)

private:
    PrefixNodeHdr& hdr(int64_t nidx) { return lines.raw(nidx).node.hdr; }
    const PrefixNodeHdr& hdr(int64_t nidx) const { return lines[nidx].node.hdr; }
    // slot index (in the whole array) of prefix slot s of a node whose extension lines exist
    int64_t prefix_slot(int64_t nidx, const PrefixNodeHdr& h, int32_t s) const {
        if (s < kInlineSlots) return nidx * kSlotsPerLine + s;
        const int32_t e = (s - kInlineSlots) / kSlotsPerLine, r = (s - kInlineSlots) % kSlotsPerLine;
        return (int64_t)(e == 0 ? h.ext0 : h.ext12 + (uint32_t)(e - 1)) * kSlotsPerLine + r;
    }
    Edge& edge_at(int64_t slot) { return lines.raw(slot / kSlotsPerLine).edges.e[slot % kSlotsPerLine]; }
    const Edge& edge_at(int64_t slot) const { return lines[slot / kSlotsPerLine].edges.e[slot % kSlotsPerLine]; }
    void mark_slots(int64_t slot, int64_t count) {
        if (count > 0) lines.mark(slot / kSlotsPerLine, (slot + count - 1) / kSlotsPerLine - slot / kSlotsPerLine + 1);
    }
    int64_t place_big_block(int64_t cap);
    void append_big_record(int64_t nidx, PrefixNodeHdr& h, const BlockRec& r);
    uint8_t prefix_cap(int64_t nidx, int32_t i) const;
    void push_prefix_cap(int64_t nidx, int32_t cap);

    StoreConfig cfg_;
    int64_t total_nodes_ = 0;
    std::vector<InstanceTotals> totals_;
    std::vector<int32_t> nblocks_;        // list length per node
    std::vector<int32_t> tail_cap_;       // capacity of each node's newest block
    std::vector<int32_t> dir_cap_;        // records reserved for the node in the directory pool
    std::vector<uint8_t> n_prefix_;       // blocks inside the prefix
    std::vector<uint8_t> pcaps_;          // capacities of the first kCapsInline prefix blocks, per node
    static constexpr int kCapsInline = 8;
    std::unordered_map<int64_t, std::vector<uint8_t>> pcaps_more_;   // nodes with more prefix blocks than that
    struct Partial { int64_t slot; int32_t free; };
    std::vector<Partial> partial_;        // edge lines with unused slots at their end (bounded list)
    std::vector<uint32_t> ord_, tmp_;
};

}  // namespace tns
