// gfx950 kernels: temporal neighbourhood sampling (Algorithm 1 of the paper, section 4.2) over
// the block store of section 4.1, and removal of the padding (section 5).
//
// Thread mapping.  The paper runs one thread per sampled neighbour with the f threads of a
// target adjacent.  On a 64-wide wavefront with dependent random reads (node entry -> block
// record -> timestamps -> edge data) what limits throughput is the number of independent
// chains in flight and the number of different 128-byte lines a load instruction touches, so:
//   * the walk runs one query per lane (64 independent chains per wave);
//   * the node entries are fetched by the wave together, eight lanes per 128-byte line, and
//     handed to their lanes through LDS;
//   * each lane leaves the edge positions it selected in LDS (the paper stages candidate
//     positions in shared memory for uniform sampling; here both policies do);
//   * the in-block search of the window end (recent policy) and the gather of the selected edges
//     are done by the whole wave, all loads of a phase issued before the first result is used:
//     lane l handles flat slot it*64+l of the wave's 64*f slots, so every store instruction
//     covers 256 consecutive bytes of each output array;
//   * with the dense outputs requested, the workgroups pass their dense offsets along a chain
//     (single-pass scan over tiles) and write the dense rows from registers.
#include "tns_kernels.h"
#include "tns_device.h"

#include <algorithm>
#include <type_traits>

namespace tns {
namespace {

// Clears the ticket, the error flag and the tile states before a fused launch (a kernel rather
// than a memset, so that the launch sequence can be captured into a graph).
__global__ void __launch_bounds__(256) tns_scan_init(ScanWorkspace* ws, int64_t num_tiles, int64_t* rowptr0, int64_t Q,
                                                     const int64_t* Q_dev, int64_t* total_out, uint32_t first_ticket) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i == 0) {
        ws->ticket = first_ticket;
        ws->error = 0;
        if (Q_dev && *Q_dev < Q) Q = *Q_dev;
        if (Q <= 0) {          // no query will write the end of rowptr
            rowptr0[0] = 0;
            if (total_out) *total_out = 0;
        }
    }
    if (i < num_tiles) ws->status[i] = 0;
}

__global__ void __launch_bounds__(256) tns_scan_clear(uint64_t* ws, int64_t words) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < words) ws[i] = 0;
}

// FUSED: also removes the padding in the same pass (rowptr and dense arrays), with the tile
// offsets obtained from a chained scan over the workgroups.
template <int POLICY, bool INCL, typename pos_t, bool COUNT, bool FUSED>
__global__ void __launch_bounds__(FUSED ? 1024 : 256, FUSED ? 4 : 6) tns_sample_kernel(const SampleArgs p, const int32_t stride,
                                                                          const uint32_t f_magic, const int32_t gshift,
                                                                          const uint32_t chunk) {
    // LDS: one chunk per wave.  First the staging area of the node lines (3 KiB), later, in the same bytes,
    // the wave's rows of selected positions and, behind them, the descriptors of the cooperative search.
    constexpr bool COOP_NODE = !COUNT;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int64_t s_tile_base;
    __shared__ int32_t s_wave_sum[16];
    __shared__ int32_t s_arrived;      // fused: waves of the tile that have finished their searches
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int waves_per_wg = blockDim.x >> 6;

    int64_t tile;
    if (FUSED) {
        // tiles are numbered in the order workgroups start
        ScanWorkspace* ws = static_cast<ScanWorkspace*>(p.scan_ws);
        if (threadIdx.x == 0) {
            s_tile_base = (int64_t)atomicAdd(&ws->ticket, 1u);
            s_arrived = 0;
        }
        __syncthreads();
        tile = s_tile_base;
        __syncthreads();
    } else {
        tile = p.xcd_remap ? xcd_tile(blockIdx.x, gridDim.x) : (int64_t)blockIdx.x;
    }
    const int64_t q0 = (tile * waves_per_wg + wave) * kWave;
    const int64_t q = q0 + lane;
    const int32_t f = p.fanout;
    // number of queries: the host's bound, or fewer when the count lives on the device (later hops)
    const int64_t Q = p.Q_dev ? min(p.Q, *p.Q_dev) : p.Q;
    if (FUSED && Q <= 0 && tile == 0 && threadIdx.x == 0) {      // no query will write the end of rowptr
        p.rowptr[0] = 0;
        if (p.total_out) *p.total_out = 0;
    }

    Walk<POLICY, INCL, pos_t> w;
    w.f = f;
    unsigned char* const my_lds = smem + (size_t)wave * chunk;
    w.s_pos = reinterpret_cast<pos_t*>(my_lds) + (size_t)lane * stride;
    w.edges = p.edges;
    w.group = (POLICY == 0 && gshift >= 0) ? (1 << gshift) : 0;
    w.te = 0.0f;
    w.tb = 0.0f;
    int32_t n_nodes = 0;
    int64_t nidx = -1;           // index of the target's entry in the node table, -1: no walk
    if (q < Q) {
        const int32_t v = __builtin_nontemporal_load(&p.targets[q]);
        w.te = __builtin_nontemporal_load(&p.t_end[q]);
        w.tb = p.t_start ? p.t_start[q] : (p.delta == INFINITY ? -INFINITY : w.te - p.delta);
        int64_t nbase = 0;
        bool ok = (uint32_t)v < (uint64_t)p.num_nodes && !(w.te != w.te) && !(w.tb != w.tb);
        if (p.inst_rowptr) {
            // instance b owns queries inst_rowptr[b] .. inst_rowptr[b+1]-1
            int32_t lo = 0, hi = p.num_instances;
            while (lo < hi) {
                const int32_t mid = lo + ((hi - lo) >> 1);
                if (p.inst_rowptr[mid + 1] <= q) lo = mid + 1; else hi = mid;
            }
            ok = ok && lo < p.num_instances;
            nbase = (int64_t)lo * p.num_nodes;
        }
        if (ok) nidx = nbase + v;
    }
    // the node's 128-byte line: header + the records of up to 7 blocks, newest first
    uint4 hd = make_uint4(0u, 0u, 0u, 0u);
    uint4 L[kInlineBlocks];
    if (COOP_NODE) {
        // Eight lanes fetch one query's line with one instruction (16 bytes each), eight queries per
        // instruction; the pieces reach their owner through LDS.  One request per line lets the loads
        // carry the non-temporal hint: a node line is used once and should not push edge lines out
        // of the L2.
        unsigned char* stage = my_lds;
        const int piece = lane & 7, sub = lane >> 3;
        u32x4 R[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t src = shfl64(nidx, i * 8 + sub);
            R[i] = u32x4{0u, 0u, 0u, 0u};
            if (src >= 0) R[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.nodes + src) + piece);
        }
        u32x4 P[8];
        // through LDS in three rounds of 24, 24 and 16 queries (3 KiB of staging); 16-byte pieces are
        // swizzled by the query number so that neither the writes nor the reads collide on banks
#pragma unroll
        for (int r = 0; r < 3; ++r) {
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                if (r * 3 + i < 8) {
                    const int ql = i * 8 + sub;             // query within the round
                    *reinterpret_cast<u32x4*>(stage + ql * 128 + ((piece ^ (ql & 7)) << 4)) = R[(r * 3 + i) & 7];
                }
            }
            wave_lds_sync();
            const int ql = lane - r * 24;
            if (ql >= 0 && ql < 24) {
#pragma unroll
                for (int j = 0; j < 8; ++j) P[j] = *reinterpret_cast<const u32x4*>(stage + ql * 128 + ((j ^ (ql & 7)) << 4));
            }
            wave_lds_sync();
        }
        hd = make_uint4(P[0].x, P[0].y, P[0].z, P[0].w);
#pragma unroll
        for (int j = 0; j < kInlineBlocks; ++j) L[j] = make_uint4(P[1 + j].x, P[1 + j].y, P[1 + j].z, P[1 + j].w);
    } else if (nidx >= 0) {
        // all eight 16-byte pieces are requested at once: the records are needed right after the
        // header for all but empty nodes and long lists
        const uint4* __restrict__ line = reinterpret_cast<const uint4*>(p.nodes + nidx);
        hd = line[0];
#pragma unroll
        for (int j = 0; j < kInlineBlocks; ++j) L[j] = line[1 + j];
    }
    if (nidx >= 0) {
        {
            ++n_nodes;
            const int32_t nb = (hd.w & 1) ? 0 : (int32_t)hd.x;      // deleted node: no blocks
            if (nb > 0 && nb <= kInlineBlocks) {
                bool go = true;
#pragma unroll
                for (int j = 0; j < kInlineBlocks; ++j)
                    if (go && j < nb) go = w.step(as_rec(L[j]), j);
                if (POLICY == 1 && w.c > (int64_t)f) {
                    w.draw(p.seed, p.qid_base + q);
                    int64_t cum = 0;
#pragma unroll
                    for (int j = 0; j < kInlineBlocks; ++j)
                        if (j >= w.t_first && j <= w.t_last) w.resolve(as_rec(L[j]), j, cum);
                }
            } else if (nb > kInlineBlocks) {
                // long list: all records of the node, oldest first, in one run of the directory
                const int64_t d0 = (int64_t)hd.z * kDirAlign;
                if (POLICY == 1 && d0 + nb <= p.num_dir && !(hd.w & 2)) {
                    // Uniform policy on a long list without deleted edges: the node's edges, blocks
                    // concatenated, form one chronological sequence and the candidates are a contiguous
                    // range [L, R) of it.  With the number of edges before each block kept next to the
                    // records, both ends and every pick cost a binary search over the run instead of
                    // two walks over all overlapping blocks.
                    const BlockRec* __restrict__ d = p.dir + d0;
                    const uint32_t* __restrict__ cum = p.dir_cum + d0;
                    // index in the sequence of the first edge with ts >= x (STRICT: ts > x)
                    auto first_at = [&](float x, auto strict) -> int64_t {
                        constexpr bool STRICT = decltype(strict)::value;
                        int32_t lo = 0, hi = nb;          // first block whose newest edge is not before x
                        while (lo < hi) {
                            const int32_t mid = lo + ((hi - lo) >> 1);
                            const float tm = d[mid].t_max;
                            ++w.n_blocks;
                            if (STRICT ? (tm > x) : (tm >= x)) hi = mid; else lo = mid + 1;
                        }
                        if (lo == nb) return (int64_t)cum[nb - 1] + rec_size(d[nb - 1]);
                        const BlockRec r = d[lo];
                        ++w.n_blocks;
                        int32_t pos = 0;
                        if (!(STRICT ? (r.t_min > x) : (r.t_min >= x)))
                            pos = w.template first_not_before<STRICT>(rec_off(r), rec_size(r), x);
                        return (int64_t)cum[lo] + pos;
                    };
                    const int64_t R = first_at(w.te, std::integral_constant<bool, INCL>{});
                    const int64_t L = w.tb == -INFINITY ? 0 : first_at(w.tb, std::false_type{});
                    const int64_t c = R > L ? R - L : 0;
                    const int32_t kk = (int32_t)min(c, (int64_t)f);
                    for (int32_t j = 0; j < kk; ++j) {
                        const int64_t g = c <= (int64_t)f ? R - 1 - j
                                                          : L + (int64_t)pick_rank(p.seed, p.qid_base + q, f, j, (uint64_t)c);
                        int32_t lo = 0, hi = nb;          // newest block that starts at or before g
                        while (lo < hi) {
                            const int32_t mid = lo + ((hi - lo) >> 1);
                            ++w.n_probes;
                            if ((int64_t)cum[mid] <= g) lo = mid + 1; else hi = mid;
                        }
                        const int32_t b = lo - 1;
                        ++w.n_blocks;
                        w.s_pos[j] = (pos_t)slot_word(rec_off(d[b]) + (g - (int64_t)cum[b]));
                    }
                    w.k = kk;
                } else if (d0 + nb <= p.num_dir) {
                    const BlockRec* __restrict__ d = p.dir + d0;
                    // newest block that starts before the window end (binary search instead of
                    // stepping through the newer blocks one by one)
                    int32_t lo = 0, hi = nb;
                    while (lo < hi) {
                        const int32_t mid = lo + ((hi - lo) >> 1);
                        const float tm = d[mid].t_min;
                        ++w.n_blocks;
                        if (INCL ? (tm > w.te) : (tm >= w.te)) hi = mid; else lo = mid + 1;
                    }
                    const int32_t j0 = lo - 1;
                    bool go = true;
                    for (int32_t j = j0; j >= 0 && go; --j) go = w.step(d[j], j0 - j);
                    if (POLICY == 1 && w.c > (int64_t)f) {
                        w.draw(p.seed, p.qid_base + q);
                        int64_t cum = 0;
                        for (int32_t t = w.t_first; t <= w.t_last; ++t) w.resolve(d[j0 - t], t, cum);
                    }
                }
            }
        }
    }
    // Recent policy, stage 1 of the cooperative part: finish the searches the lanes left open.
    // A group of 16 lanes serves one query: lane j of the group reads the timestamp of slot j of
    // the query's search window; the number of qualifying slots comes from a ballot.  All loads are
    // issued before the first result is used, so the wave pays the memory latency once.
    int32_t h = 0;               // edges of the searched block that lie before the window end
    if (POLICY == 0 && gshift >= 0) {
        constexpr int G = kCoopGroup, groups = kWave / G;
        unsigned char* extra = my_lds + (size_t)kWave * stride * sizeof(pos_t);
        // per query: window start (40-bit slot index) with the window size in the upper bits,
        // the window end time, and the result
        uint2* s_q = reinterpret_cast<uint2*>(extra);
        float* s_te = reinterpret_cast<float*>(extra + (size_t)kWave * sizeof(uint2));
        int32_t* s_h = reinterpret_cast<int32_t*>(extra + (size_t)kWave * (sizeof(uint2) + sizeof(float)));
        const int64_t win0 = w.d_off + w.d_lo;
        s_q[lane] = make_uint2((uint32_t)(win0 & 0xffffffffll), ((uint32_t)(win0 >> 32) & 0xffu) | ((uint32_t)w.d_n << 8));
        s_te[lane] = w.te;
        wave_lds_sync();
        const int g = lane / G, j = lane % G;
        float tj[G];
#pragma unroll
        for (int it = 0; it < G; ++it) {
            const uint2 d = s_q[it * groups + g];
            tj[it] = 0.0f;
            if (j < (int32_t)(d.y >> 8)) {
                const auto w = (typename index_of<pos_t>::type)slot_word((((int64_t)(d.y & 0xffu)) << 32 | d.x) + j);
                tj[it] = __uint_as_float(p.edges[w]);
            }
        }
#pragma unroll
        for (int it = 0; it < G; ++it) {
            const int32_t n = (int32_t)(s_q[it * groups + g].y >> 8);
            const float teq = s_te[it * groups + g];
            const bool qual = j < n && (INCL ? (tj[it] <= teq) : (tj[it] < teq));
            const uint64_t m = __ballot(qual);
            if (j == 0) s_h[it * groups + g] = __popcll((m >> (g * G)) & ((1ull << G) - 1));
        }
        wave_lds_sync();
        if (w.d_off >= 0) h = w.d_lo + s_h[lane];
    }
    const int32_t k = POLICY == 0 ? min(f, h + w.k) : w.k;
    if (POLICY == 0 && h > 0) {
        // The first min(h, f) slots come from the block whose search the wave finished (newest
        // first); the positions recorded from older blocks move up behind them.
        const int32_t hh = min(h, f);
        for (int32_t j = k - 1; j >= hh; --j) w.s_pos[j] = w.s_pos[j - hh];
        for (int32_t j = 0; j < hh; ++j) w.s_pos[j] = (pos_t)slot_word(w.d_off + h - 1 - j);
    }
    if (COUNT) {
        // totals of what this launch reads: node entries, block records, timestamp probes, edges
        unsigned long long v4[4] = {(unsigned long long)n_nodes, (unsigned long long)w.n_blocks,
                                    (unsigned long long)w.n_probes, (unsigned long long)k};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned long long v = v4[i];
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
            if (lane == 0 && v) atomicAdd(&p.counters[i], v);
        }
        return;
    }
    const pos_t* __restrict__ w_pos = reinterpret_cast<const pos_t*>(my_lds);

    if (FUSED) {
        // Chained scan over the workgroup tiles for the dense offsets.
        ScanWorkspace* ws = static_cast<ScanWorkspace*>(p.scan_ws);
        const int32_t inc = wave_inclusive_scan(k, lane);
        auto publish_total = [&](int32_t wg_total) {
            // the tile total is published at once, so that later tiles can look past this one
            if (lane == 0 && tile > 0)
                __hip_atomic_store(&ws->status[tile], kStTotal | (uint64_t)wg_total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        auto chain = [&](int32_t wg_total) {      // one wave: look back for the tile's offset, publish the prefix
            const int64_t excl = tile > 0 ? lookback_exclusive(ws, p.err_flag, tile, lane) : 0;
            if (lane == 0) {
                __hip_atomic_store(&ws->status[tile], kStPrefix | (uint64_t)(excl + wg_total), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                s_tile_base = excl;
            }
        };
        auto write_rowptr = [&](int64_t row) {
            if (q < Q) {
                __builtin_nontemporal_store(row, &p.rowptr[q]);
                if (q == Q - 1) {
                    // The last query's tile has looked back over every other tile.  If any wait ran into
                    // its bound the dense rows are not valid: the total then reads 0, so that a hop chained
                    // to this one has no queries.
                    __threadfence();
                    const bool bad = __hip_atomic_load(p.err_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
                    const int64_t tot = bad ? 0 : row + k;
                    p.rowptr[Q] = tot;
                    if (p.total_out) *p.total_out = tot;
                }
            }
        };
        auto offset_of_wave = [&]() {
            int32_t off = 0;
            for (int i = 0; i < wave; ++i) off += s_wave_sum[i];
            return off;
        };
        GatherRegs g;
        if (f <= kGatherChunk) {
            // No barrier between a wave's searches and its gather (the lines the searches fetched are
            // then still in the L2): the waves count themselves in, and the one that arrives last
            // adds up the tile total and publishes it.  Every wave gathers (one batch of loads) and
            // writes its padded rows, the gathered edges stay in registers; the last wave then looks
            // back for the tile's offset (the earlier tiles have had the time of a gather to publish
            // their totals), and only the dense copy waits for it.
            int is_last = 0;
            if (lane == kWave - 1) {
                s_wave_sum[wave] = inc;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                is_last = __hip_atomic_fetch_add(&s_arrived, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == waves_per_wg - 1;
            }
            is_last = __shfl(is_last, kWave - 1, kWave);
            int32_t wg_total = 0;
            if (is_last) {
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                for (int i = 0; i < waves_per_wg; ++i) wg_total += s_wave_sum[i];
                publish_total(wg_total);
            }
            wave_lds_sync();      // the positions were written by this wave's own lanes
            gather_load<pos_t, POLICY == 1>(g, p, f_magic, stride, w_pos, lane, 0, k);
            // Recent policy: the look-back reads come before this wave's stores (a load result can only be
            // waited for together with every store issued before it).  Uniform policy: the other order
            // measured faster (C5 step 31.2 against 36.6 ms; its waves reach this point far apart).
            if (is_last && POLICY == 0) chain(wg_total);
            store_padded(g, p, f_magic, lane, 0, q0, Q);
            if (is_last && POLICY != 0) chain(wg_total);
            lds_barrier();
            const int64_t row = s_tile_base + offset_of_wave() + (inc - k);
            write_rowptr(row);
            store_dense(g, p, f_magic, lane, 0, row);
        } else {
            // larger fan-outs: offset first, then gather in batches and write both
            if (lane == kWave - 1) s_wave_sum[wave] = inc;
            __syncthreads();
            int32_t wg_total = 0;
            for (int i = 0; i < waves_per_wg; ++i) wg_total += s_wave_sum[i];
            if (wave == 0) {
                publish_total(wg_total);
                chain(wg_total);
            }
            __syncthreads();
            const int64_t row = s_tile_base + offset_of_wave() + (inc - k);
            write_rowptr(row);
            for (int32_t it0 = 0; it0 < f; it0 += kGatherChunk) {
                gather_load<pos_t, POLICY == 1>(g, p, f_magic, stride, w_pos, lane, it0, k);
                store_padded(g, p, f_magic, lane, it0, q0, Q);
                store_dense(g, p, f_magic, lane, it0, row);
            }
        }
    } else {
        wave_lds_sync();
        GatherRegs g;
        for (int32_t it0 = 0; it0 < f; it0 += kGatherChunk) {
            gather_load<pos_t, POLICY == 1>(g, p, f_magic, stride, w_pos, lane, it0, k);
            store_padded(g, p, f_magic, lane, it0, q0, Q);
        }
    }
    if (q < Q && p.out_count) __builtin_nontemporal_store(k, &p.out_count[q]);
}

// ---- padding removal -------------------------------------------------------------------

// sum of counts per tile of kCompactTile queries
__global__ void __launch_bounds__(256) tns_count_tile_sums(const int32_t* __restrict__ count, int64_t Q,
                                                           const int64_t* __restrict__ Q_dev,
                                                           int32_t* __restrict__ tile_sums) {
    __shared__ int32_t s_w[4];
    if (Q_dev) Q = min(Q, *Q_dev);
    const int64_t base = (int64_t)blockIdx.x * kCompactTile;
    int32_t v = 0;
#pragma unroll
    for (int i = 0; i < kCompactTile / 256; ++i) {
        const int64_t q = base + i * 256 + threadIdx.x;
        if (q < Q) v += count[q];
    }
    const int lane = threadIdx.x & 63;
    v = wave_inclusive_scan(v, lane);
    if (lane == 63) s_w[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// exclusive scan of the tile sums (int64), one workgroup; also writes rowptr[Q]
__global__ void __launch_bounds__(1024) tns_scan_tile_sums(const int32_t* __restrict__ tile_sums, int64_t num_tiles,
                                                           int64_t* __restrict__ tile_offs, int64_t* __restrict__ rowptr,
                                                           int64_t Q, const int64_t* __restrict__ Q_dev,
                                                           int64_t* __restrict__ total_out, uint32_t* __restrict__ ws_head) {
    __shared__ int32_t s_w[16];
    __shared__ int64_t s_carry;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < num_tiles; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int32_t v = i < num_tiles ? tile_sums[i] : 0;
        const int32_t inc = wave_inclusive_scan(v, lane);
        if (lane == 63) s_w[wave] = inc;
        __syncthreads();
        int32_t wave_off = 0, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int32_t t = s_w[w];
            if (w < wave) wave_off += t;
            all += t;
        }
        const int64_t carry = s_carry;
        if (i < num_tiles) tile_offs[i] = carry + wave_off + (inc - v);
        __syncthreads();
        if (threadIdx.x == 0) s_carry = carry + all;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (Q_dev) Q = min(Q, *Q_dev);
        rowptr[Q < 0 ? 0 : Q] = s_carry;          // end of rowptr for the actual number of queries
        if (total_out) *total_out = s_carry;
        ws_head[0] = 0;                           // the workspace's status word: no chained scan ran, nothing timed out
        ws_head[1] = 0;
    }
}

// rowptr of the tile's queries and scatter of the filled slots to the dense arrays
__global__ void __launch_bounds__(256) tns_compact_scatter(const CompactArgs a, const int64_t* __restrict__ tile_offs,
                                                           const uint32_t f_magic) {
    __shared__ int32_t s_excl[kCompactTile];
    __shared__ int32_t s_cnt[kCompactTile];
    __shared__ int32_t s_w[4];
    constexpr int kPer = kCompactTile / 256;
    const int64_t Q = a.Q_dev ? min(a.Q, *a.Q_dev) : a.Q;
    const int64_t base = (int64_t)blockIdx.x * kCompactTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t c[kPer];
    int32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int64_t q = base + threadIdx.x * kPer + i;
        c[i] = q < Q ? a.count[q] : 0;
        sum += c[i];
    }
    const int32_t inc = wave_inclusive_scan(sum, lane);
    if (lane == 63) s_w[wave] = inc;
    __syncthreads();
    int32_t excl = inc - sum;
    for (int w = 0; w < wave; ++w) excl += s_w[w];
    const int64_t tile_off = tile_offs[blockIdx.x];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int ql = threadIdx.x * kPer + i;
        s_excl[ql] = excl;
        s_cnt[ql] = c[i];
        if (base + ql < Q) a.rowptr[base + ql] = tile_off + excl;
        excl += c[i];
    }
    __syncthreads();
    if (!a.cmp_nbr) return;
    const uint32_t f = (uint32_t)a.fanout;
    const uint32_t slots = kCompactTile * f;
    const int64_t in0 = base * f;
    const int64_t in_end = Q * (int64_t)f;
    for (uint32_t s = threadIdx.x; s < slots; s += 256) {
        if (in0 + s >= in_end) break;
        const uint32_t ql = div_by(s, f, f_magic);
        const uint32_t j = s - ql * f;
        if ((int32_t)j < s_cnt[ql]) {
            const int64_t d = tile_off + s_excl[ql] + j;
            a.cmp_nbr[d] = a.nbr[in0 + s];
            a.cmp_eid[d] = a.eid[in0 + s];
            a.cmp_ts[d] = a.ts[in0 + s];
        }
    }
}

// Next hop's instance offsets: instance b's queries of the next hop are the dense entries of its
// queries of this hop, so next[b] = rowptr[cur[b]] (cur[I] = number of queries of this hop).
__global__ void __launch_bounds__(256) tns_hop_inst_rowptr(const int64_t* __restrict__ cur, const int64_t* __restrict__ rowptr,
                                                           int32_t num_instances, int64_t* __restrict__ next) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b <= num_instances) next[b] = rowptr[cur[b]];
}

inline uint32_t magic_for(int32_t f) { return f <= 1 ? 0u : (uint32_t)(((uint64_t(1) << 32) + (uint64_t)f - 1) / (uint64_t)f); }

template <int POLICY, bool INCL, typename pos_t, bool COUNT, bool FUSED>
hipError_t launch_sample_t(const SampleArgs& a, hipStream_t stream) {
    const int32_t stride = a.fanout | 1;                                    // odd: conflict-free per-lane rows
    const size_t per_wave = (size_t)kWave * stride * sizeof(pos_t);
    // The fused variant uses large workgroups under the recent policy: one chained-scan step per 1024
    // queries keeps the rate at which tiles publish their totals low enough for the look-back to keep
    // up.  Under the uniform policy the waves of a tile finish far apart (two walks, per-lane searches)
    // and wait for each other before the dense copy, so small tiles win there (C5: 36.5 ms with 16
    // waves, 32.6 with 8, 31.3 with 4, 34.1 with 2).
    // recent policy with fan-out <= 16: the wave finishes the in-block searches together
    // (16 more bytes of LDS per query); otherwise each lane searches alone
    int32_t gshift = (POLICY == 0 && a.fanout <= kCoopGroup) ? 4 : -1;
    // per wave: position rows + search descriptors, and at least the 3 KiB in which the node lines are staged first
    const size_t chunk = std::max<size_t>(per_wave + (gshift >= 0 ? (size_t)kWave * 16 : 0), COUNT ? 0 : 3072);
    int waves = (int)std::min<size_t>(FUSED ? (POLICY == 1 ? 4 : 16) : 4, std::max<size_t>(1, (62u << 10) / chunk));
    // small batches: smaller workgroups, so that the queries spread over the compute units instead of
    // queueing at the address units of a few
    while (waves > 1 && (a.Q + (int64_t)waves * kWave - 1) / ((int64_t)waves * kWave) < 512) waves >>= 1;
    const int64_t per_wg = (int64_t)waves * kWave;
    const int64_t grid = (a.Q + per_wg - 1) / per_wg;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (FUSED && !a.scan_ready) {
        // one state more than tiles: the workspace has it, and a test that starts the tickets at 1 uses it
        const hipError_t e = launch_scan_init(a, grid + 1, stream);
        if (e != hipSuccess) return e;
    }
    if (grid <= 0) return hipGetLastError();
    const size_t lds = chunk * waves;
    SampleArgs b = a;
    if (FUSED && !b.err_flag) b.err_flag = &static_cast<ScanWorkspace*>(a.scan_ws)->error;
    hipLaunchKernelGGL((tns_sample_kernel<POLICY, INCL, pos_t, COUNT, FUSED>), dim3((unsigned)grid), dim3(waves * kWave),
                       lds, stream, b, stride, magic_for(a.fanout), gshift, (uint32_t)chunk);
    return hipGetLastError();
}

}  // namespace

size_t compact_workspace_bytes(int64_t Q) {
    // enough for either use: tile sums + offsets of the stand-alone compaction, or the ticket
    // and one state per 64-query wave (the smallest workgroup) of the fused chained scan
    const int64_t tiles = (Q + kCompactTile - 1) / kCompactTile;
    const size_t sums = ((size_t)tiles * sizeof(int32_t) + 255) & ~size_t(255);
    const size_t offs = ((size_t)tiles * sizeof(int64_t) + 255) & ~size_t(255);
    const size_t fused = 256 + (size_t)((Q + kWave - 1) / kWave + 1) * sizeof(uint64_t);
    return std::max(sums + offs + 256, (fused + 255) & ~size_t(255));
}

hipError_t launch_scan_init(const SampleArgs& a, int64_t num_tiles, hipStream_t stream) {
    const unsigned init_grid = (unsigned)std::max<int64_t>(1, (num_tiles + 255) / 256);
    hipLaunchKernelGGL(tns_scan_init, dim3(init_grid), dim3(256), 0, stream, static_cast<ScanWorkspace*>(a.scan_ws), num_tiles,
                       a.rowptr, a.Q, a.Q_dev, a.total_out, (uint32_t)a.first_ticket);
    return hipGetLastError();
}

hipError_t launch_sample(const SampleArgs& a, hipStream_t stream) {
    if (a.prefix_layout) return launch_sample_prefix(a, stream);
    const bool incl = a.inclusive_end != 0;
    const bool wide = a.wide_offsets != 0;
#define TNS_DISPATCH(POL, CNT, FUS)                                                          \
    (incl ? (wide ? launch_sample_t<POL, true, int64_t, CNT, FUS>(a, stream)                 \
                  : launch_sample_t<POL, true, int32_t, CNT, FUS>(a, stream))                \
          : (wide ? launch_sample_t<POL, false, int64_t, CNT, FUS>(a, stream)                \
                  : launch_sample_t<POL, false, int32_t, CNT, FUS>(a, stream)))
    if (a.counters) return a.policy == 0 ? TNS_DISPATCH(0, true, false) : TNS_DISPATCH(1, true, false);
    if (a.scan_ws) return a.policy == 0 ? TNS_DISPATCH(0, false, true) : TNS_DISPATCH(1, false, true);
    return a.policy == 0 ? TNS_DISPATCH(0, false, false) : TNS_DISPATCH(1, false, false);
#undef TNS_DISPATCH
}

hipError_t launch_scan_clear(void* ws, size_t bytes, hipStream_t stream) {
    const int64_t words = (int64_t)(bytes / 8);
    if (words > 0)
        hipLaunchKernelGGL(tns_scan_clear, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, static_cast<uint64_t*>(ws), words);
    return hipGetLastError();
}

hipError_t launch_hop_inst_rowptr(const int64_t* cur, const int64_t* rowptr, int32_t num_instances, int64_t* next,
                                  hipStream_t stream) {
    hipLaunchKernelGGL(tns_hop_inst_rowptr, dim3((unsigned)(num_instances / 256 + 1)), dim3(256), 0, stream, cur, rowptr,
                       num_instances, next);
    return hipGetLastError();
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t stream) {
    const int64_t tiles = (a.Q + kCompactTile - 1) / kCompactTile;
    // the first 256 bytes of a workspace hold the status word of the step (read by tns_run_status)
    uint32_t* ws_head = static_cast<uint32_t*>(a.workspace);
    unsigned char* ws = static_cast<unsigned char*>(a.workspace) + 256;
    int32_t* sums = reinterpret_cast<int32_t*>(ws);
    const size_t sums_bytes = ((size_t)tiles * sizeof(int32_t) + 255) & ~size_t(255);
    int64_t* offs = reinterpret_cast<int64_t*>(ws + sums_bytes);
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    if (tiles > 0) {
        hipLaunchKernelGGL(tns_count_tile_sums, dim3((unsigned)tiles), dim3(256), 0, stream, a.count, a.Q, a.Q_dev, sums);
    }
    hipLaunchKernelGGL(tns_scan_tile_sums, dim3(1), dim3(1024), 0, stream, sums, tiles, offs, a.rowptr, a.Q, a.Q_dev,
                       a.total_out, ws_head);
    if (tiles > 0) {
        hipLaunchKernelGGL(tns_compact_scatter, dim3((unsigned)tiles), dim3(256), 0, stream, a, offs,
                           magic_for(a.fanout));
    }
    return hipGetLastError();
}

}  // namespace tns
