// Host-side builder of the time-indexed block store (section 4.1 of the paper): node table,
// chronological block lists with b_v = min(deg(v), tau) sizing, edge data.  The host arrays
// are kept in exactly the device layout (tns_layout.h) so that a commit is a plain copy of the
// parts that changed.  No HIP in this file.
#pragma once
#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "tns_layout.h"

namespace tns {

// Growable array in fixed pages (no reallocation, so ingestion never copies what is already
// stored) with change tracking in sub-pages for incremental upload.
template <class T, int PAGE_LOG2 = 20, int SUB_LOG2 = 12>
class Paged {
public:
    static constexpr int64_t kPage = int64_t(1) << PAGE_LOG2;
    static constexpr int64_t kSub = int64_t(1) << SUB_LOG2;

    Paged() = default;
    Paged(const Paged&) = delete;
    Paged& operator=(const Paged&) = delete;
    ~Paged() {
        for (T* p : pages_) std::free(p);
    }

    int64_t size() const { return n_; }
    const T& operator[](int64_t i) const { return pages_[i >> PAGE_LOG2][i & (kPage - 1)]; }
    // Writable access without marking; the caller marks the range it wrote.
    T& raw(int64_t i) { return pages_[i >> PAGE_LOG2][i & (kPage - 1)]; }
    T& mut(int64_t i) {
        dirty_[i >> SUB_LOG2] = 1;
        return raw(i);
    }
    void mark(int64_t start, int64_t count) {
        if (count <= 0) return;
        for (int64_t s = start >> SUB_LOG2, e = (start + count - 1) >> SUB_LOG2; s <= e; ++s) dirty_[s] = 1;
    }
    // Append `count` zero-initialised elements; returns the index of the first.
    int64_t grow(int64_t count) {
        int64_t start = n_;
        int64_t need_pages = (n_ + count + kPage - 1) >> PAGE_LOG2;
        while ((int64_t)pages_.size() < need_pages) {
            // 128-byte aligned (records are line-sized) and zero-filled
            T* p = static_cast<T*>(std::aligned_alloc(128, (size_t)kPage * sizeof(T)));
            if (!p) throw std::bad_alloc();
            std::memset(static_cast<void*>(p), 0, (size_t)kPage * sizeof(T));
            pages_.push_back(p);
        }
        n_ += count;
        dirty_.resize((size_t)((n_ + kSub - 1) >> SUB_LOG2), 0);
        return start;
    }
    void mark_all() { std::fill(dirty_.begin(), dirty_.end(), 1); }
    void clear_dirty() { std::fill(dirty_.begin(), dirty_.end(), 0); }
    // Calls fn(first_index, count, host_pointer) for every maximal run of changed sub-pages
    // that is contiguous in host memory (i.e. inside one page).
    template <class F>
    void for_each_dirty(F&& fn) const {
        const int64_t nsub = (int64_t)dirty_.size();
        const int64_t sub_per_page = kPage >> SUB_LOG2;
        int64_t s = 0;
        while (s < nsub) {
            if (!dirty_[s]) { ++s; continue; }
            int64_t e = s + 1;
            const int64_t page_end = ((s / sub_per_page) + 1) * sub_per_page;
            while (e < nsub && e < page_end && dirty_[e]) ++e;
            int64_t first = s << SUB_LOG2;
            int64_t last = e << SUB_LOG2;
            if (last > n_) last = n_;
            fn(first, last - first, &(*this)[first]);
            s = e;
        }
    }

private:
    std::vector<T*> pages_;
    std::vector<uint8_t> dirty_;
    int64_t n_ = 0;
};

struct StoreConfig {
    int64_t num_nodes = 0;
    int32_t num_instances = 1;
    int32_t tau = 1;
    int32_t sizing = 0;  // 0 adaptive, 1 strawman, 2 fixed
    bool node_slab = true;  // give each node one edge line of its own for its first blocks
};

struct InstanceTotals {
    int64_t edges = 0, slots = 0, blocks = 0, next_eid = 0;   // slots: sum of block capacities
    int64_t deleted = 0;                                         // edges whose validity was cleared
    float newest_ts = 0.0f;  // newest timestamp stored so far (valid if edges > 0)
};

class Store {
public:
    explicit Store(const StoreConfig& cfg);

    // One ingestion batch for one instance; status codes as in tns.h, detail in err.
    int add_edges(int32_t inst, const int32_t* src, const int32_t* dst, const float* ts, const int32_t* eid,
                  int64_t m, std::string& err);

    // Tombstone deletion (section 4.1): clears the validity of the edge (node v, edge id e); returns
    // how many stored edges matched (0 or 1 for unique ids).
    int64_t delete_edge(int32_t inst, int32_t v, int32_t e);
    // Marks a node deleted / restores it.
    void set_node_deleted(int32_t inst, int32_t v, bool deleted);
    bool any_tombstones() const { return any_tombstones_; }

    const StoreConfig& config() const { return cfg_; }
    const InstanceTotals& totals(int32_t inst) const { return totals_[inst]; }
    int64_t node_index(int32_t inst, int64_t v) const { return (int64_t)inst * cfg_.num_nodes + v; }
    // i-th block of a node in chronological order (0 = oldest) and its capacity
    const BlockRec& block_of(int64_t nidx, int32_t i) const;
    int32_t block_cap(int64_t nidx, int32_t i) const;

    Paged<NodeLine, 18, 9> nodes;   // 128-byte entries: 2^18 per page, change tracking per 64 KiB
    Paged<BlockRec> dir;            // directory pool: record runs of nodes with long lists
    Paged<uint32_t> dir_cum;        // same indexing as dir: edges the node holds in the blocks before this one
    Paged<EdgeLine, 18, 9> lines;   // edge data, 10 slots per 128-byte line

    Edge& edge_at(int64_t slot) { return lines.raw(slot / kSlotsPerLine).e[slot % kSlotsPerLine]; }
    void mark_slots(int64_t slot, int64_t count) {
        if (count > 0) lines.mark(slot / kSlotsPerLine, (slot + count - 1) / kSlotsPerLine - slot / kSlotsPerLine + 1);
    }

private:
    // Placement of a new block's slots.  Blocks of 10 slots or more start on a line; smaller
    // ones go to the node's own line while it has room (node_slab), else into the leftover of
    // some line, never across a line boundary.
    int64_t place_block(int64_t nidx, int64_t cap);
    struct Partial { int64_t slot; int32_t free; };
    std::vector<Partial> partial_;        // lines with unused slots at their end (bounded list)
    std::vector<uint32_t> slab_line_;     // node's own line + 1 (0: none yet)
    std::vector<uint8_t> slab_used_;      // slots of it already given to blocks
    BlockRec& tail_rec(NodeLine& nd);
    void append_block(int64_t nidx, NodeLine& nd, const BlockRec& r, int32_t cap);

    StoreConfig cfg_;
    bool any_tombstones_ = false;
    std::vector<InstanceTotals> totals_;
    std::vector<int32_t> tail_cap_;       // capacity of each node's newest block (host side only)
    std::vector<int32_t> dir_cap_;        // records reserved for the node in the directory pool (0: inline)
    std::vector<uint32_t> ord_, tmp_;     // scratch: batch positions grouped by source node
};

// Stable grouping of batch positions by source node id (shared by the two builders).
void group_by_source(const int32_t* src, int64_t m, int64_t num_nodes, std::vector<uint32_t>& ord,
                     std::vector<uint32_t>& tmp);

}  // namespace tns
