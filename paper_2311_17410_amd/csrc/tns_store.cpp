// Host-side store builder: edge insertion of section 4.1 with the adaptive block sizing rule.
#include "tns_store.h"

#include <algorithm>
#include <climits>
#include <cmath>

#include "../../include/tns.h"

namespace tns {

Store::Store(const StoreConfig& cfg) : cfg_(cfg), totals_((size_t)cfg.num_instances) {
    const int64_t total_nodes = (int64_t)cfg.num_instances * cfg.num_nodes;
    if (total_nodes > 0) {
        nodes.grow(total_nodes);   // zero-filled: no blocks, degree 0, valid
        nodes.mark_all();
    }
    tail_cap_.assign((size_t)total_nodes, 0);
    dir_cap_.assign((size_t)total_nodes, 0);
    if (cfg.node_slab) {
        slab_line_.assign((size_t)total_nodes, 0);
        slab_used_.assign((size_t)total_nodes, 0);
    }
}

int64_t Store::place_block(int64_t nidx, int64_t cap) {
    if (cap >= kSlotsPerLine) {
        const int64_t nlines = (cap + kSlotsPerLine - 1) / kSlotsPerLine;
        const int64_t slot = lines.grow(nlines) * kSlotsPerLine;
        const int32_t left = (int32_t)(nlines * kSlotsPerLine - cap);
        if (left > 0) {
            if (partial_.size() >= 64) partial_.erase(partial_.begin());
            partial_.push_back({slot + cap, left});
        }
        return slot;
    }
    if (cfg_.node_slab) {
        // the node's own line: its first blocks (capacities 1, 1, 2, 4 under the adaptive rule)
        // end up next to each other, so the walk reads one line for all of them
        uint32_t& sl = slab_line_[(size_t)nidx];
        uint8_t& used = slab_used_[(size_t)nidx];
        if (sl == 0) {
            const int64_t line = lines.grow(1);
            if (line + 1 > (int64_t)UINT32_MAX) throw std::bad_alloc();
            sl = (uint32_t)(line + 1);
            used = 0;
        }
        if (used + cap <= kSlotsPerLine) {
            const int64_t slot = (int64_t)(sl - 1) * kSlotsPerLine + used;
            used = (uint8_t)(used + cap);
            return slot;
        }
    }
    for (size_t i = 0; i < partial_.size(); ++i)
        if (partial_[i].free >= cap) {
            const int64_t slot = partial_[i].slot;
            partial_[i].slot += cap;
            partial_[i].free -= (int32_t)cap;
            if (partial_[i].free == 0) partial_.erase(partial_.begin() + (long)i);
            return slot;
        }
    const int64_t slot = lines.grow(1) * kSlotsPerLine;
    if (partial_.size() >= 64) partial_.erase(partial_.begin());
    partial_.push_back({slot + cap, (int32_t)(kSlotsPerLine - cap)});
    return slot;
}

const BlockRec& Store::block_of(int64_t nidx, int32_t i) const {
    const NodeLine& nd = nodes[nidx];
    if (nd.nblocks <= kInlineBlocks) return nd.rec[nd.nblocks - 1 - i];
    return dir[(int64_t)nd.dir_line * kDirAlign + i];
}

int32_t Store::block_cap(int64_t nidx, int32_t i) const {
    const NodeLine& nd = nodes[nidx];
    // only the newest block can have room
    return i == nd.nblocks - 1 ? tail_cap_[(size_t)nidx] : rec_size(block_of(nidx, i));
}

BlockRec& Store::tail_rec(NodeLine& nd) {
    if (nd.nblocks <= kInlineBlocks) return nd.rec[0];
    const int64_t i = (int64_t)nd.dir_line * kDirAlign + nd.nblocks - 1;
    return dir.mut(i);
}

// Link a new (newest) block to the node: O(1) inline shift, or an append to the node's run in
// the directory pool (runs grow by doubling into a fresh place; the old run is abandoned).
void Store::append_block(int64_t nidx, NodeLine& nd, const BlockRec& r, int32_t cap) {
    if (nd.nblocks < kInlineBlocks) {
        for (int j = nd.nblocks; j > 0; --j) nd.rec[j] = nd.rec[j - 1];
        nd.rec[0] = r;
    } else {
        int32_t& dcap = dir_cap_[(size_t)nidx];
        if (nd.nblocks == dcap || dcap == 0) {
            const int32_t ncap = dcap ? dcap * 2 : 2 * kDirAlign;
            const int64_t start = dir.grow(ncap);
            dir_cum.grow(ncap);
            if (dcap == 0) {
                uint32_t before = 0;
                for (int j = 0; j < kInlineBlocks; ++j) {
                    const BlockRec& o = nd.rec[kInlineBlocks - 1 - j];
                    dir.raw(start + j) = o;
                    dir_cum.raw(start + j) = before;
                    before += (uint32_t)rec_size(o);
                }
            } else {
                const int64_t old = (int64_t)nd.dir_line * kDirAlign;
                for (int32_t j = 0; j < nd.nblocks; ++j) {
                    dir.raw(start + j) = dir[old + j];
                    dir_cum.raw(start + j) = dir_cum[old + j];
                }
            }
            dir.mark(start, nd.nblocks);
            dir_cum.mark(start, nd.nblocks);
            nd.dir_line = (uint32_t)(start / kDirAlign);
            dcap = ncap;
        }
        dir.mut((int64_t)nd.dir_line * kDirAlign + nd.nblocks) = r;
        dir_cum.mut((int64_t)nd.dir_line * kDirAlign + nd.nblocks) = (uint32_t)nd.degree;   // edges in the older blocks
    }
    nd.nblocks += 1;
    tail_cap_[(size_t)nidx] = cap;
}

int64_t Store::delete_edge(int32_t inst, int32_t v, int32_t e) {
    const int64_t nidx = node_index(inst, v);
    NodeLine& nd = nodes.raw(nidx);
    int64_t hit = 0;
    for (int32_t b = 0; b < nd.nblocks; ++b) {
        // block records in chronological order; the record is rewritten when a tombstone is set
        BlockRec* r = nd.nblocks <= kInlineBlocks ? &nd.rec[nd.nblocks - 1 - b]
                                                  : &dir.raw((int64_t)nd.dir_line * kDirAlign + b);
        const int64_t off = rec_off(*r);
        const int32_t size = rec_size(*r);
        bool here = false;
        for (int32_t i = 0; i < size; ++i) {
            Edge& ed = edge_at(off + i);
            if (ed.eid == e) {
                ed.eid = ~e;
                mark_slots(off + i, 1);
                here = true;
                ++hit;
            }
        }
        if (here) {
            *r = make_rec(r->t_min, r->t_max, off, size, true);
            if (nd.nblocks > kInlineBlocks) dir.mark((int64_t)nd.dir_line * kDirAlign + b, 1);
        }
    }
    if (hit) {
        nd.flags |= 2;
        nodes.mark(nidx, 1);
        totals_[(size_t)inst].deleted += hit;
        any_tombstones_ = true;
    }
    return hit;
}

void Store::set_node_deleted(int32_t inst, int32_t v, bool deleted) {
    NodeLine& nd = nodes.mut(node_index(inst, v));
    nd.flags = deleted ? (nd.flags | 1) : (nd.flags & ~1);
}

// Stable LSD radix sort of batch positions by source node id (11 bits per pass).
void group_by_source(const int32_t* src, int64_t m, int64_t num_nodes, std::vector<uint32_t>& ord,
                     std::vector<uint32_t>& tmp) {
    ord.resize((size_t)m);
    tmp.resize((size_t)m);
    for (int64_t i = 0; i < m; ++i) ord[(size_t)i] = (uint32_t)i;
    int bits = 0;
    while (bits < 31 && (int64_t(1) << bits) < num_nodes) ++bits;
    constexpr int kRadix = 11;
    for (int shift = 0; shift < bits; shift += kRadix) {
        int64_t hist[(1 << kRadix) + 1] = {0};
        const uint32_t mask = (1u << kRadix) - 1;
        for (int64_t i = 0; i < m; ++i) hist[(((uint32_t)src[i]) >> shift & mask) + 1]++;
        for (int b = 0; b < (1 << kRadix); ++b) hist[b + 1] += hist[b];
        for (int64_t i = 0; i < m; ++i) {
            uint32_t e = ord[(size_t)i];
            tmp[(size_t)hist[((uint32_t)src[e]) >> shift & mask]++] = e;
        }
        ord.swap(tmp);
    }
}

int Store::add_edges(int32_t inst, const int32_t* src, const int32_t* dst, const float* ts, const int32_t* eid,
                     int64_t m, std::string& err) {
    if (inst < 0 || inst >= cfg_.num_instances) {
        err = "instance out of range";
        return TNS_ERANGE;
    }
    if (m < 0 || (m > 0 && (!src || !dst || !ts))) {
        err = "null array or negative batch size";
        return TNS_EINVAL;
    }
    if (m == 0) return TNS_OK;
    if (m > (int64_t)INT32_MAX) {
        err = "batch larger than 2^31-1 edges: split it";
        return TNS_ESIZE;
    }
    const int64_t V = cfg_.num_nodes;
    bool globally_sorted = true;
    for (int64_t i = 0; i < m; ++i) {
        if ((uint32_t)src[i] >= (uint64_t)V) {
            err = "source node id outside [0, num_nodes) at batch position " + std::to_string(i);
            return TNS_ERANGE;
        }
        if (std::isnan(ts[i])) {
            err = "NaN timestamp at batch position " + std::to_string(i);
            return TNS_EORDER;
        }
        if (eid && eid[i] < 0) {
            err = "negative edge id at batch position " + std::to_string(i);
            return TNS_EINVAL;
        }
        if (i > 0 && ts[i - 1] > ts[i]) globally_sorted = false;
    }
    if (!eid && totals_[(size_t)inst].next_eid + m > (int64_t)INT32_MAX) {
        err = "running edge id would exceed 2^31-1";
        return TNS_ESIZE;
    }
    InstanceTotals& tot = totals_[(size_t)inst];
    // A batch that is in time order as a whole and starts no earlier than anything stored in
    // this instance cannot violate any node's order: skip the per-node checks.
    const bool fast_order = globally_sorted && (tot.edges == 0 || ts[0] >= tot.newest_ts);

    group_by_source(src, m, V, ord_, tmp_);
    uint32_t* ord = ord_.data();

    if (!fast_order) {
        for (int64_t g0 = 0; g0 < m;) {
            const int32_t v = src[ord[g0]];
            int64_t g1 = g0 + 1;
            bool sorted = true;
            while (g1 < m && src[ord[g1]] == v) {
                if (ts[ord[g1 - 1]] > ts[ord[g1]]) sorted = false;
                ++g1;
            }
            if (!sorted)
                std::stable_sort(ord + g0, ord + g1, [ts](uint32_t a, uint32_t b) { return ts[a] < ts[b]; });
            const int64_t nidx = node_index(inst, v);
            const NodeLine& nd = nodes[nidx];
            if (nd.nblocks > 0 && ts[ord[g0]] < block_of(nidx, nd.nblocks - 1).t_max) {
                err = "node " + std::to_string(v) + " would receive an edge older than its newest stored edge";
                return TNS_EORDER;
            }
            g0 = g1;
        }
    }

    // Limit of the record encoding, checked before anything is changed.  Worst case: every edge
    // of the batch opens a block, of at most max(batch share, min(degree, tau)) slots.
    int64_t stored = 0;
    for (const InstanceTotals& t : totals_) stored += t.edges;
    const int64_t by_tau = m * std::max<int64_t>(1, cfg_.tau);   // m, tau < 2^31: no overflow
    const int64_t worst_new_slots = m + (cfg_.sizing == TNS_SIZING_FIXED ? by_tau : std::min(by_tau, stored + m));
    if (lines.size() * kSlotsPerLine + worst_new_slots + 2 * kSlotsPerLine * m > kMaxEdgeOffset) {
        err = "edge array would exceed 2^40 slots";
        return TNS_ESIZE;
    }

    const int64_t eid_base = tot.next_eid;
    float newest = tot.edges ? tot.newest_ts : ts[ord[0]];
    for (int64_t g0 = 0; g0 < m;) {
        const int32_t v = src[ord[g0]];
        int64_t g1 = g0 + 1;
        while (g1 < m && src[ord[g1]] == v) ++g1;
        const int64_t nidx = node_index(inst, v);
        NodeLine& nd = nodes.mut(nidx);
        int64_t i = g0;
        auto put = [&](int64_t pos, uint32_t e) {
            Edge& ed = edge_at(pos);
            ed.ts = ts[e];
            ed.nbr = dst[e];
            ed.eid = eid ? eid[e] : (int32_t)(eid_base + (int64_t)e);
        };
        if (nd.nblocks > 0) {
            BlockRec& tb = tail_rec(nd);
            const int32_t size = rec_size(tb);
            const int64_t off = rec_off(tb);
            const int64_t take = std::min<int64_t>(tail_cap_[(size_t)nidx] - size, g1 - i);
            if (take > 0) {
                for (int64_t k = 0; k < take; ++k) put(off + size + k, ord[i + k]);
                mark_slots(off + size, take);
                tb = make_rec(tb.t_min, ts[ord[i + take - 1]], off, size + (int32_t)take, rec_tombstones(tb));
                nd.degree += (int32_t)take;
                i += take;
            }
        }
        int64_t rest = g1 - i;
        while (rest > 0) {
            int64_t cap;
            if (cfg_.sizing == TNS_SIZING_STRAWMAN) cap = rest;
            else if (cfg_.sizing == TNS_SIZING_FIXED) cap = cfg_.tau;
            else cap = std::max<int64_t>(rest, std::min<int64_t>(nd.degree, cfg_.tau));  // b_v = min(deg(v), tau)
            cap = std::min(cap, kMaxBlockEdges);   // limit of the record's size field
            const int64_t take = std::min(rest, cap);
            const int64_t off = place_block(nidx, cap);
            for (int64_t k = 0; k < take; ++k) put(off + k, ord[i + k]);
            mark_slots(off, take);
            append_block(nidx, nd, make_rec(ts[ord[i]], ts[ord[i + take - 1]], off, (int32_t)take), (int32_t)cap);
            nd.degree += (int32_t)take;
            tot.slots += cap;
            tot.blocks += 1;
            i += take;
            rest -= take;
        }
        if (ts[ord[g1 - 1]] > newest) newest = ts[ord[g1 - 1]];
        g0 = g1;
    }
    tot.edges += m;
    tot.next_eid += m;
    tot.newest_ts = newest;
    return TNS_OK;
}

}  // namespace tns
