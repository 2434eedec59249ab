// Host-side store builder, prefix layout: edge insertion of section 4.1 with the adaptive block sizing
// rule; a node's first blocks are carved out of its prefix (its own line + up to three extension lines).
#include "tns_pstore.h"

#include <algorithm>
#include <climits>
#include <cmath>

#include "../../include/tns.h"

namespace tns {

PrefixStore::PrefixStore(const StoreConfig& cfg) : cfg_(cfg), totals_((size_t)cfg.num_instances) {
    total_nodes_ = (int64_t)cfg.num_instances * cfg.num_nodes;
    if (total_nodes_ > 0) {
        lines.grow(total_nodes_);   // zero-filled node lines: degree 0, no blocks, valid
        lines.mark_all();
    }
    nblocks_.assign((size_t)total_nodes_, 0);
    tail_cap_.assign((size_t)total_nodes_, 0);
    dir_cap_.assign((size_t)total_nodes_, 0);
    n_prefix_.assign((size_t)total_nodes_, 0);
    pcaps_.assign((size_t)total_nodes_ * kCapsInline, 0);
}

uint8_t PrefixStore::prefix_cap(int64_t nidx, int32_t i) const {
    if (i < kCapsInline) return pcaps_[(size_t)nidx * kCapsInline + i];
    return pcaps_more_.at(nidx)[(size_t)(i - kCapsInline)];
}

void PrefixStore::push_prefix_cap(int64_t nidx, int32_t cap) {
    const int32_t i = n_prefix_[(size_t)nidx]++;
    if (i < kCapsInline) pcaps_[(size_t)nidx * kCapsInline + i] = (uint8_t)cap;
    else pcaps_more_[nidx].push_back((uint8_t)cap);
}

// Blocks outside the prefix: 10 slots or more start on a line, smaller ones go into the leftover of
// some line, never across a line boundary.
int64_t PrefixStore::place_big_block(int64_t cap) {
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

// Append the record of a new block outside the prefix to the node's run (runs grow by doubling into a
// fresh place; the old run is abandoned).
void PrefixStore::append_big_record(int64_t nidx, PrefixNodeHdr& h, const BlockRec& r) {
    const int32_t nbig = pmeta_big_blocks(h.meta);
    int32_t& dcap = dir_cap_[(size_t)nidx];
    if (nbig == dcap) {
        const int32_t ncap = dcap ? dcap * 2 : kDirAlign;
        const int64_t start = dir.grow(ncap);
        dir_cum.grow(ncap);
        const int64_t old = (int64_t)h.dir_line * kDirAlign;
        for (int32_t j = 0; j < nbig; ++j) {
            dir.raw(start + j) = dir[old + j];
            dir_cum.raw(start + j) = dir_cum[old + j];
        }
        dir.mark(start, nbig);
        dir_cum.mark(start, nbig);
        h.dir_line = (uint32_t)(start / kDirAlign);
        dcap = ncap;
    }
    dir.mut((int64_t)h.dir_line * kDirAlign + nbig) = r;
    dir_cum.mut((int64_t)h.dir_line * kDirAlign + nbig) = (uint32_t)h.degree;   // edges stored before this block
}

void PrefixStore::block_info(int64_t nidx, int32_t i, int32_t* cap, int32_t* size, float* t_min, float* t_max) const {
    const PrefixNodeHdr& h = hdr(nidx);
    const int32_t npre = n_prefix_[(size_t)nidx];
    if (i < npre) {
        int32_t start = 0;
        for (int32_t j = 0; j < i; ++j) start += prefix_cap(nidx, j);
        const int32_t c = prefix_cap(nidx, i);
        const int32_t sz = std::min<int32_t>(c, h.degree - start);
        if (cap) *cap = c;
        if (size) *size = sz;
        if (t_min) *t_min = edge_at(prefix_slot(nidx, h, start)).ts;
        if (t_max) *t_max = edge_at(prefix_slot(nidx, h, start + sz - 1)).ts;
        return;
    }
    const BlockRec& r = dir[(int64_t)h.dir_line * kDirAlign + (i - npre)];
    if (cap) *cap = i == nblocks_[(size_t)nidx] - 1 ? tail_cap_[(size_t)nidx] : rec_size(r);
    if (size) *size = rec_size(r);
    if (t_min) *t_min = r.t_min;
    if (t_max) *t_max = r.t_max;
}

int64_t PrefixStore::delete_edge(int32_t inst, int32_t v, int32_t e) {
    const int64_t nidx = node_index(inst, v);
    PrefixNodeHdr& h = hdr(nidx);
    int64_t hit = 0;
    const int32_t fill = std::min<int32_t>(h.degree, pmeta_prefix_slots(h.meta));
    for (int32_t s = 0; s < fill; ++s) {
        const int64_t slot = prefix_slot(nidx, h, s);
        Edge& ed = edge_at(slot);
        if (ed.eid == e) {
            ed.eid = ~e;
            mark_slots(slot, 1);
            ++hit;
        }
    }
    const int32_t nbig = pmeta_big_blocks(h.meta);
    for (int32_t b = 0; b < nbig; ++b) {
        BlockRec& r = dir.raw((int64_t)h.dir_line * kDirAlign + b);
        const int64_t off = rec_off(r);
        const int32_t size = rec_size(r);
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
            r = make_rec(r.t_min, r.t_max, off, size, true);
            dir.mark((int64_t)h.dir_line * kDirAlign + b, 1);
        }
    }
    if (hit) {
        h.meta |= 2u;
        lines.mark(nidx, 1);
        totals_[(size_t)inst].deleted += hit;
    }
    return hit;
}

void PrefixStore::set_node_deleted(int32_t inst, int32_t v, bool deleted) {
    const int64_t nidx = node_index(inst, v);
    PrefixNodeHdr& h = hdr(nidx);
    h.meta = deleted ? (h.meta | 1u) : (h.meta & ~1u);
    lines.mark(nidx, 1);
}

int PrefixStore::add_edges(int32_t inst, const int32_t* src, const int32_t* dst, const float* ts, const int32_t* eid,
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
            if (nblocks_[(size_t)nidx] > 0) {
                float newest;
                block_info(nidx, nblocks_[(size_t)nidx] - 1, nullptr, nullptr, nullptr, &newest);
                if (ts[ord[g0]] < newest) {
                    err = "node " + std::to_string(v) + " would receive an edge older than its newest stored edge";
                    return TNS_EORDER;
                }
            }
            g0 = g1;
        }
    }

    // Limits of the encodings, checked before anything is changed.  Worst case: every edge of the batch opens
    // a block of at most max(batch share, min(degree, tau)) slots, plus two extension lines.
    int64_t stored = 0;
    for (const InstanceTotals& t : totals_) stored += t.edges;
    const int64_t by_tau = m * std::max<int64_t>(1, cfg_.tau);
    const int64_t worst_new_slots = m + (cfg_.sizing == TNS_SIZING_FIXED ? by_tau : std::min(by_tau, stored + m));
    const int64_t worst_lines = lines.size() + worst_new_slots / kSlotsPerLine + 4 * m + 4;
    if (worst_lines > (int64_t)UINT32_MAX || worst_lines * kSlotsPerLine > kMaxEdgeOffset) {
        err = "edge array would exceed 2^32 lines";
        return TNS_ESIZE;
    }

    const int64_t eid_base = tot.next_eid;
    float newest = tot.edges ? tot.newest_ts : ts[ord[0]];
    for (int64_t g0 = 0; g0 < m;) {
        const int32_t v = src[ord[g0]];
        int64_t g1 = g0 + 1;
        while (g1 < m && src[ord[g1]] == v) ++g1;
        const int64_t nidx = node_index(inst, v);
        PrefixNodeHdr& h = hdr(nidx);
        lines.mark(nidx, 1);
        int32_t P = pmeta_prefix_slots(h.meta);
        int32_t nbig = pmeta_big_blocks(h.meta);
        int64_t i = g0;
        auto fill_edge = [&](Edge& ed, uint32_t e) {
            ed.ts = ts[e];
            ed.nbr = dst[e];
            ed.eid = eid ? eid[e] : (int32_t)(eid_base + (int64_t)e);
        };
        // edge number `s` of the node goes to prefix slot s; the first slot of an extension line sets its fence
        auto put_prefix = [&](int32_t s, uint32_t e) {
            const int64_t slot = prefix_slot(nidx, h, s);
            fill_edge(edge_at(slot), e);
            mark_slots(slot, 1);
            if (s >= kInlineSlots && (s - kInlineSlots) % kSlotsPerLine == 0) h.fence[(s - kInlineSlots) / kSlotsPerLine] = ts[e];
        };
        if (nblocks_[(size_t)nidx] > 0) {
            if (nbig == 0) {
                const int64_t take = std::min<int64_t>(P - h.degree, g1 - i);
                for (int64_t k = 0; k < take; ++k) put_prefix(h.degree + (int32_t)k, ord[i + k]);
                h.degree += (int32_t)take;
                i += take;
            } else {
                BlockRec& tb = dir.mut((int64_t)h.dir_line * kDirAlign + nbig - 1);
                const int32_t size = rec_size(tb);
                const int64_t off = rec_off(tb);
                const int64_t take = std::min<int64_t>(tail_cap_[(size_t)nidx] - size, g1 - i);
                if (take > 0) {
                    for (int64_t k = 0; k < take; ++k) fill_edge(edge_at(off + size + k), ord[i + k]);
                    mark_slots(off + size, take);
                    tb = make_rec(tb.t_min, ts[ord[i + take - 1]], off, size + (int32_t)take, rec_tombstones(tb));
                    h.degree += (int32_t)take;
                    i += take;
                }
            }
        }
        int64_t rest = g1 - i;
        while (rest > 0) {
            int64_t cap;
            if (cfg_.sizing == TNS_SIZING_STRAWMAN) cap = rest;
            else if (cfg_.sizing == TNS_SIZING_FIXED) cap = cfg_.tau;
            else cap = std::max<int64_t>(rest, std::min<int64_t>(h.degree, cfg_.tau));  // b_v = min(deg(v), tau)
            cap = std::min(cap, kMaxBlockEdges);
            const int64_t take = std::min(rest, cap);
            if (nbig == 0 && P + cap <= kPrefixSlots) {
                // the block is carved out of the prefix; extension lines are allocated when first reached
                const int32_t reach = P + (int32_t)cap;
                if (reach > kInlineSlots && h.ext0 == 0) h.ext0 = (uint32_t)lines.grow(1);
                if (reach > kInlineSlots + kSlotsPerLine && h.ext12 == 0) h.ext12 = (uint32_t)lines.grow(2);
                push_prefix_cap(nidx, (int32_t)cap);
                P = reach;
                for (int64_t k = 0; k < take; ++k) put_prefix(h.degree + (int32_t)k, ord[i + k]);
            } else {
                if (nbig >= kMaxBigBlocks) {      // cannot happen below 2^22 blocks per node; the batch is cut short rather than corrupt
                    err = "node " + std::to_string(v) + " would exceed 2^22 blocks";
                    h.meta = make_pmeta(h.meta, 0, P, nbig);
                    return TNS_ESIZE;
                }
                const int64_t off = place_big_block(cap);
                for (int64_t k = 0; k < take; ++k) fill_edge(edge_at(off + k), ord[i + k]);
                mark_slots(off, take);
                append_big_record(nidx, h, make_rec(ts[ord[i]], ts[ord[i + take - 1]], off, (int32_t)take));
                ++nbig;
                h.meta = make_pmeta(h.meta, 0, P, nbig);     // append_big_record reads the count from the entry
            }
            h.degree += (int32_t)take;
            nblocks_[(size_t)nidx] += 1;
            tail_cap_[(size_t)nidx] = (int32_t)cap;
            tot.slots += cap;
            tot.blocks += 1;
            i += take;
            rest -= take;
        }
        const int32_t fill = std::min<int32_t>(h.degree, P);
        const int32_t n_ext = fill <= kInlineSlots ? 0 : (fill - kInlineSlots + kSlotsPerLine - 1) / kSlotsPerLine;
        h.meta = make_pmeta(h.meta, n_ext, P, nbig);
        if (ts[ord[g1 - 1]] > newest) newest = ts[ord[g1 - 1]];
        g0 = g1;
    }
    tot.edges += m;
    tot.next_eid += m;
    tot.newest_ts = newest;
    return TNS_OK;
}

}  // namespace tns
