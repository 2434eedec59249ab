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
        nodes.grow(total_nodes);
        for (int64_t i = 0; i < total_nodes; ++i) nodes.raw(i).tail = -1;
        nodes.mark_all();
    }
    head_.assign((size_t)total_nodes, -1);
}

namespace {

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

}  // namespace

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
        if (i > 0 && ts[i - 1] > ts[i]) globally_sorted = false;
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
            const NodeRec& nd = nodes[node_index(inst, v)];
            if (nd.tail >= 0 && ts[ord[g0]] < blocks[nd.tail].t_max) {
                err = "node " + std::to_string(v) + " would receive an edge older than its newest stored edge";
                return TNS_EORDER;
            }
            g0 = g1;
        }
    }

    // Capacity checks before anything is changed.
    if (blocks.size() + m >= (int64_t)INT32_MAX) {
        err = "more than 2^31-1 blocks";
        return TNS_ESIZE;
    }

    const int64_t eid_base = tot.next_eid;
    float newest = tot.edges ? tot.newest_ts : ts[ord[0]];
    for (int64_t g0 = 0; g0 < m;) {
        const int32_t v = src[ord[g0]];
        int64_t g1 = g0 + 1;
        while (g1 < m && src[ord[g1]] == v) ++g1;
        const int64_t nidx = node_index(inst, v);
        NodeRec& nd = nodes.mut(nidx);
        int64_t i = g0;
        auto put = [&](int64_t pos, uint32_t e) {
            Edge& ed = edges.raw(pos);
            ed.ts = ts[e];
            ed.nbr = dst[e];
            ed.eid = eid ? eid[e] : (int32_t)(eid_base + (int64_t)e);
        };
        if (nd.tail >= 0) {
            BlockRec& tb = blocks.raw(nd.tail);
            int64_t take = std::min<int64_t>(tb.cap - tb.size, g1 - i);
            if (take > 0) {
                for (int64_t k = 0; k < take; ++k) put(tb.off + tb.size + k, ord[i + k]);
                edges.mark(tb.off + tb.size, take);
                tb.size += (int32_t)take;
                tb.t_max = ts[ord[i + take - 1]];
                blocks.mark(nd.tail, 1);
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
            const int64_t take = std::min(rest, cap);
            const int64_t bi = blocks.grow(1);
            const int64_t off = edges.grow(cap);
            for (int64_t k = 0; k < take; ++k) put(off + k, ord[i + k]);
            edges.mark(off, cap);
            BlockRec& nb = blocks.mut(bi);
            nb.t_min = ts[ord[i]];
            nb.t_max = ts[ord[i + take - 1]];
            nb.size = (int32_t)take;
            nb.cap = (int32_t)cap;
            nb.off = off;
            nb.prev = nd.tail;
            nb.next = -1;
            if (nd.tail >= 0) blocks.mut(nd.tail).next = (int32_t)bi;
            else head_[(size_t)nidx] = (int32_t)bi;
            nd.tail = (int32_t)bi;
            nd.nblocks += 1;
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
