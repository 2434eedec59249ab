// gfx950 sampling kernel for a store in the prefix layout (tns_layout.h): Algorithm 1 of the paper
// (section 4.2) with the padded write of section 4.2's kernel notes and the padding removal of
// section 5 fused in, as in tns_kernels.hip, but arranged around the fact that a node's first 38 edge
// slots sit in at most four 128-byte lines reachable from its table entry.
//
// What a query reads.  The node's line (entry + first eight edge slots) always.  The entry holds one
// fence per extension line (the timestamp of its first slot), so the line that contains the window end
// is known without touching any other: if it is the node's own line the query is done; otherwise that
// one extension line is read, and the line before it only if the newest f candidates reach back into it
// (from the node's own line, already there, when the window end lies in the first extension line).
//
// How the wave reads it.  Every 128-byte line is fetched exactly once and nothing is read twice:
//   * node lines: eight lanes per line, 16 bytes each, handed to the owning lane through LDS; the lane
//     counts the qualifying slots of its own line in registers (eight compares, no search loop);
//   * extension lines: the requests of a wave are compacted, sixteen lanes serve one request, lane j
//     loads the 12-byte edge of slot j; two ballots give the window ends inside the line, and the lanes
//     whose edges are selected write them straight into the query's result row in LDS;
//   * result rows (f edges per query, newest first up to a rotation that makes the row position of an
//     edge independent of how many newer edges another line contributes) feed the same coalesced padded
//     and dense stores as the other kernel.
// Queries the fast path does not cover (uniform policy, nodes with deleted edges or with blocks outside
// the prefix, fan-outs above ten) take the per-lane block walk: directory records for the blocks outside
// the prefix, then the prefix's lines as blocks of their own, the node's own line from registers.  They
// leave edge positions in their row and the output stage loads those edges from memory.
#include <algorithm>

#include "tns_device.h"
#include "tns_kernels.h"

namespace tns {
namespace {

constexpr int kMaxFastFanout = kSlotsPerLine;
constexpr int kExtraLds = 192;        // per wave, behind the result rows: owner and counts of every line request (one byte
                                      // each) and the counts of the walking lanes' cooperative searches

__device__ __forceinline__ int ceil_log2_outcomes(int n) { return n <= 0 ? 0 : 32 - __clz(n); }   // probes of a binary search over n sorted items

// One round of extension-line reads for a wave, in two halves so that other work can run while the lines
// are on their way.  A lane with `need` asks for the first n slots of line `line`; of the slots before its
// window end (all of them if open_end) and not before its window start the newest `cap` are written into
// the lane's result row, the newest at row position (from_f ? f - a : 0), a = how many are taken.
//
// The requests are compacted; sixteen lanes serve one request, lane j loads the 12-byte edge of slot j.
// A request's parameters stay in the registers of the lane that made it and reach the serving lanes by
// shuffles; LDS only holds who made request number r (one byte) and, afterwards, its two counts.
constexpr int kBatch = 8;             // load instructions issued together = 32 requests
struct ExtBatch {
    Edge ed[kBatch];
    uint32_t par[kBatch];             // owner | n << 8 | cap << 16 | from_f << 24 | open_end << 25 | valid << 31
};

__device__ __forceinline__ void ext_issue(ExtBatch& x, const uint32_t* __restrict__ lines, const unsigned char* owner_of, int b0,
                                          int total, int lane, uint32_t my_line, uint32_t my_par) {
    const int g = lane >> 4, j = lane & 15;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
        const int req = b0 + i * 4 + g;
        const bool valid = req < total;
        const int owner = valid ? (int)owner_of[req] : lane;
        const uint32_t line = (uint32_t)__shfl((int)my_line, owner, kWave);
        // (every lane takes part in the shuffles: a lane that sat one out could not be read by the others)
        const uint32_t par = (uint32_t)__shfl((int)my_par, owner, kWave);
        x.par[i] = valid ? (par | 0x80000000u) : 0u;
        x.ed[i].ts = 0.0f; x.ed[i].nbr = -1; x.ed[i].eid = -1;
        if (valid && j < (int)((x.par[i] >> 8) & 0xffu))
            x.ed[i] = *reinterpret_cast<const Edge*>(lines + (uint64_t)line * 32u + (uint32_t)(3 * j));
    }
}

template <bool INCL>
__device__ __forceinline__ void ext_process(const ExtBatch& x, unsigned char* result_of, uint32_t* rows, int rs, int f, int b0,
                                            int lane, float my_te, float my_tb) {
    const int g = lane >> 4, j = lane & 15;
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
        const bool valid = (x.par[i] >> 31) != 0;
        const int nn = (int)((x.par[i] >> 8) & 0xffu), cp = (int)((x.par[i] >> 16) & 0xffu);
        const bool in = valid && j < nn;
        const float qe = __shfl(my_te, (int)(x.par[i] & 0xffu), kWave), qb = __shfl(my_tb, (int)(x.par[i] & 0xffu), kWave);
        const bool before = in && (((x.par[i] >> 25) & 1u) || (INCL ? (x.ed[i].ts <= qe) : (x.ed[i].ts < qe)));
        const bool early = in && x.ed[i].ts < qb;
        const int r = __popcll((__ballot(before) >> (g * 16)) & 0xffffull);
        const int l = __popcll((__ballot(early) >> (g * 16)) & 0xffffull);
        const int lo_sel = max(l, r - cp);
        const int a = max(r - lo_sel, 0);
        const int base = ((x.par[i] >> 24) & 1u) ? f - a : 0;
        if (in && j >= lo_sel && j < r) {
            uint32_t* dst = rows + (x.par[i] & 0xffu) * rs + 3 * (base + (r - 1 - j));
            dst[0] = __float_as_uint(x.ed[i].ts);
            dst[1] = (uint32_t)x.ed[i].nbr;
            dst[2] = (uint32_t)x.ed[i].eid;
        }
        if (valid && j == 0) result_of[b0 + i * 4 + g] = (unsigned char)(r | (l << 4));
    }
}

// Output stage, fan-outs up to ten: every query's edges are in its result row by now (fast-path queries at a
// rotated row position, queries that walked at position j after walked_gather).  info = k | rot << 8 of the
// lane's own query.  No memory loads here: the stores that follow go out back to back.
__device__ __forceinline__ void rows_load(GatherRegs& g, const SampleArgs& p, uint32_t f_magic, const uint32_t* rows,
                                          int rs, int lane, int32_t info) {
    const int32_t f = p.fanout;
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        g.nbr[i] = -1; g.eid[i] = -1; g.ts[i] = 0.0f;
        if (i < f) {
            const uint32_t s = (uint32_t)(i * kWave + lane);
            const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
            const int32_t j = (int32_t)(s - ql * (uint32_t)f);
            const int32_t inf = __shfl(info, (int)ql, kWave);
            if (j < (inf & 0xff)) {
                const uint32_t* row = rows + ql * (uint32_t)rs;
                int32_t ps = j + f - ((inf >> 8) & 0xff);
                if (ps >= f) ps -= f;
                g.ts[i] = __uint_as_float(row[3 * ps]);
                g.nbr[i] = (int32_t)row[3 * ps + 1];
                g.eid[i] = (int32_t)row[3 * ps + 2];
            }
        }
    }
}

// Fan-outs up to ten: the queries that walked left edge positions at the start of their rows; the wave
// fetches those edges together (flat slot order: consecutive lanes read consecutive edges of one query)
// and puts them into the rows, slot j at row position j, where rows_load expects them.  All positions
// are read before the first edge is written, so the two may overlap in the row.
template <typename pos_t>
__device__ __forceinline__ void walked_gather(const SampleArgs& p, uint32_t f_magic, uint32_t* rows, int rs, int lane,
                                              int32_t winfo /* walked ? k : 0 of the lane's own query */) {
    const int32_t f = p.fanout;
    bool filled[kGatherChunk];
    Edge raw[kGatherChunk];
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        filled[i] = false;
        raw[i].ts = 0.0f; raw[i].nbr = -1; raw[i].eid = -1;
        if (i < f) {
            const uint32_t s = (uint32_t)(i * kWave + lane);
            const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
            const int32_t j = (int32_t)(s - ql * (uint32_t)f);
            filled[i] = j < __shfl(winfo, (int)ql, kWave);
            const uint64_t m = __ballot(filled[i]);       // empty slots read what the first filled one reads
            const pos_t own = filled[i] ? reinterpret_cast<const pos_t*>(rows + ql * (uint32_t)rs)[j] : (pos_t)0;
            const pos_t other = sizeof(pos_t) == 8 ? (pos_t)shfl64((int64_t)own, m ? __builtin_ctzll(m) : 0)
                                                   : (pos_t)__shfl((int)own, m ? __builtin_ctzll(m) : 0, kWave);
            const auto pos = (typename index_of<pos_t>::type)(filled[i] ? own : other);
            raw[i] = *reinterpret_cast<const Edge*>(p.edges + pos);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0070);     // all loads and all LDS reads of the positions have returned
    __builtin_amdgcn_sched_barrier(0);
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        if (i < f && filled[i]) {
            const uint32_t s = (uint32_t)(i * kWave + lane);
            const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
            const int32_t j = (int32_t)(s - ql * (uint32_t)f);
            uint32_t* dst = rows + ql * (uint32_t)rs + 3 * j;
            dst[0] = __float_as_uint(raw[i].ts);
            dst[1] = (uint32_t)raw[i].nbr;
            dst[2] = (uint32_t)raw[i].eid;
        }
    }
    wave_lds_sync();
}

template <int POLICY, bool INCL, typename pos_t, bool COUNT, bool FUSED>
__global__ void __launch_bounds__(1024) tns_sample_prefix_kernel(const SampleArgs p, const int32_t rs, const uint32_t f_magic,
                                                                 const int32_t gshift, const uint32_t chunk,
                                                                 const uint32_t rows_bytes) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int64_t s_tile_base;
    __shared__ int32_t s_wave_sum[16];
    __shared__ int32_t s_arrived;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int waves_per_wg = blockDim.x >> 6;

    int64_t tile;
    if (FUSED) {
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
    const int64_t Q = p.Q_dev ? min(p.Q, *p.Q_dev) : p.Q;
    if (FUSED && Q <= 0 && tile == 0 && threadIdx.x == 0) {
        p.rowptr[0] = 0;
        if (p.total_out) *p.total_out = 0;
    }

    unsigned char* const my_lds = smem + (size_t)wave * chunk;
    uint32_t* const rows = reinterpret_cast<uint32_t*>(my_lds);
    const uint32_t* __restrict__ lines = p.edges;

    // ---- the query and its node ------------------------------------------------------------
    float te = 0.0f, tb = 0.0f;
    int64_t nidx = -1;
    if (q < Q) {
        const int32_t v = __builtin_nontemporal_load(&p.targets[q]);
        te = __builtin_nontemporal_load(&p.t_end[q]);
        tb = p.t_start ? p.t_start[q] : (p.delta == INFINITY ? -INFINITY : te - p.delta);
        int64_t nbase = 0;
        bool ok = (uint32_t)v < (uint64_t)p.num_nodes && !(te != te) && !(tb != tb);
        if (p.inst_rowptr) {
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
    // ---- node lines: eight lanes per line, handed over through LDS ------------------------------------
    uint32_t w[3 * kInlineSlots];     // the eight edge slots of the node's own line
    uint32_t h_degree, h_meta, h_ext0, h_ext12, h_fence0, h_fence1, h_fence2, h_dir;   // the node entry
    {
        const int piece = lane & 7, sub = lane >> 3;
        u32x4 R[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t src = shfl64(nidx, i * 8 + sub);
            R[i] = u32x4{0u, 0u, 0u, 0u};
            if (src >= 0) R[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(lines + src * 32) + piece);
        }
        // through LDS in two rounds of 32 queries (4 KiB of staging); 16-byte pieces are swizzled by the query
        // number so that neither the writes nor the reads collide on banks
        u32x4 v6 = u32x4{0u, 0u, 0u, 0u}, v7 = v6;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ql = i * 8 + sub;             // query within the round
                *reinterpret_cast<u32x4*>(my_lds + ql * 128 + ((piece ^ (ql & 7)) << 4)) = R[r * 4 + i];
            }
            wave_lds_sync();
            if ((lane >> 5) == r) {
                const int ql = lane & 31;
#pragma unroll
                for (int j = 0; j < 6; ++j) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(my_lds + ql * 128 + ((j ^ (ql & 7)) << 4));
                    w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
                }
                v6 = *reinterpret_cast<const u32x4*>(my_lds + ql * 128 + ((6 ^ (ql & 7)) << 4));
                v7 = *reinterpret_cast<const u32x4*>(my_lds + ql * 128 + ((7 ^ (ql & 7)) << 4));
            }
            wave_lds_sync();
        }
        h_degree = v6.x; h_meta = v6.y; h_ext0 = v6.z; h_ext12 = v6.w;
        h_fence0 = v7.x; h_fence1 = v7.y; h_fence2 = v7.z; h_dir = v7.w;
    }
    static_assert(kNodeHdrWord == 24 && sizeof(PrefixNodeHdr) == 32, "the node entry is the last two 16-byte pieces of the line");
    // ---- per query: where the window end falls ----------------------------------------------------
    const int32_t degree = (int32_t)h_degree;
    const uint32_t meta = h_meta;
    const bool alive = nidx >= 0 && !(meta & 1u) && degree > 0;
    const bool tomb = (meta & 2u) != 0;
    const int32_t nbig = pmeta_big_blocks(meta);
    const int32_t fill = min(degree, pmeta_prefix_slots(meta));       // edges stored in the prefix
    const int32_t n_in = min(fill, kInlineSlots);
    const int32_t n_ext = fill <= kInlineSlots ? 0 : (fill - kInlineSlots + kSlotsPerLine - 1) / kSlotsPerLine;
    // extension line x (0..2) and its fence, selected without indexing registers by a run-time value
    auto ext_line = [&](int32_t x) -> uint32_t { return x == 0 ? h_ext0 : h_ext12 + (uint32_t)(x - 1); };
    auto fence = [&](int32_t x) -> float { return __uint_as_float(x == 0 ? h_fence0 : (x == 1 ? h_fence1 : h_fence2)); };
    const bool fast = POLICY == 0 && f <= kMaxFastFanout && alive && !tomb && nbig == 0;
    const bool walked = alive && !fast;
    uint32_t* const my_row = rows + lane * rs;
    unsigned char* const owner_of = my_lds + rows_bytes;       // who made line request number r
    unsigned char* const result_of = owner_of + kWave;        // its two counts
    int32_t k = 0, rot = 0;
    int32_t n_blocks = 0, n_probes = 0;       // byte model (COUNT)

    // ---- fast path -----------------------------------------------------------------------------------
    // The extension line that holds the window end (-1: the node's own line) follows from the fences alone,
    // so its read is started first; the node's own line is worked on while that read is on its way.
    int32_t e = -1;
    if (fast) {
#pragma unroll
        for (int j = 0; j < kPrefixExtLines; ++j)
            if (j < n_ext && (INCL ? (fence(j) <= te) : (fence(j) < te))) e = j;
    }
    const bool need1 = fast && e >= 0;
    const int32_t n_e = need1 ? min(fill - kInlineSlots - kSlotsPerLine * e, kSlotsPerLine) : 0;
    const uint32_t line1 = need1 ? ext_line(e) : 0u;
    const uint32_t par1 = (uint32_t)lane | ((uint32_t)n_e << 8) | ((uint32_t)f << 16) | (1u << 24);
    ExtBatch xb;
    int total1 = 0, rank1 = 0;
    if (!COUNT) {
        const uint64_t mask = __ballot(need1);
        total1 = __popcll(mask);
        rank1 = __popcll(mask & ((1ull << lane) - 1ull));
        if (need1) owner_of[rank1] = (unsigned char)lane;
        wave_lds_sync();
        if (total1 > 0) ext_issue(xb, lines, owner_of, 0, total1, lane, line1, par1);
    }
    // slots of the node's own line before the window end / before the window start
    int32_t hi_in = 0, lo_in = 0;
#pragma unroll
    for (int i = 0; i < kInlineSlots; ++i) {
        const float t = __uint_as_float(w[3 * i]);
        hi_in += (i < n_in && (INCL ? (t <= te) : (t < te))) ? 1 : 0;
        lo_in += (i < n_in && t < tb) ? 1 : 0;
    }
    if (fast) {
        if (e < 0) {
            const int32_t a = max(min(f, hi_in - lo_in), 0);
            if (!COUNT) {
#pragma unroll
                for (int i = 0; i < kInlineSlots; ++i)
                    if (i >= hi_in - a && i < hi_in) {
                        uint32_t* dst = my_row + 3 * (f - a + (hi_in - 1 - i));
                        dst[0] = w[3 * i]; dst[1] = w[3 * i + 1]; dst[2] = w[3 * i + 2];
                    }
            }
            k = a;
            rot = a;
            n_probes += ceil_log2_outcomes(n_in) + (tb > -INFINITY ? ceil_log2_outcomes(hi_in) : 0);
        } else if (e == 0 && !COUNT) {
            // the node's own line is the older neighbour of the first extension line: its newest edges go
            // to the row positions they have whatever that line contributes (newer edges overwrite the rest)
#pragma unroll
            for (int i = 0; i < kInlineSlots; ++i)
                if (i >= lo_in && kInlineSlots - 1 - i < f) {
                    uint32_t* dst = my_row + 3 * (kInlineSlots - 1 - i);
                    dst[0] = w[3 * i]; dst[1] = w[3 * i + 1]; dst[2] = w[3 * i + 2];
                }
        }
    }
    {
        // round 1: the line with the window end; round 2: the line before it, where the row is not full yet
        int r1 = 0, l1 = 0;
        if (COUNT) {
            // the counting variant reads the line's timestamps itself (it writes no rows)
            if (need1) {
                const uint32_t* src = lines + (uint64_t)line1 * 32u;
                for (int x = 0; x < n_e; ++x) {
                    const float t = __uint_as_float(src[3 * x]);
                    r1 += (INCL ? (t <= te) : (t < te)) ? 1 : 0;
                    l1 += t < tb ? 1 : 0;
                }
            }
        } else if (total1 > 0) {
            wave_lds_sync();
            ext_process<INCL>(xb, result_of, rows, rs, f, 0, lane, te, tb);
#pragma unroll 1
            for (int b0 = 4 * kBatch; b0 < total1; b0 += 4 * kBatch) {
                ext_issue(xb, lines, owner_of, b0, total1, lane, line1, par1);
                ext_process<INCL>(xb, result_of, rows, rs, f, b0, lane, te, tb);
            }
            wave_lds_sync();
            if (need1) {
                const int v = result_of[rank1];
                r1 = v & 15;
                l1 = v >> 4;
            }
            wave_lds_sync();
        }
        if (need1) {
            const int32_t a = max(r1 - max(l1, r1 - f), 0);
            k = a;
            rot = a;
            n_probes += ceil_log2_outcomes(n_e) + (tb > -INFINITY ? ceil_log2_outcomes(r1) : 0);
        }
        const bool more = need1 && l1 == 0 && k < f;
        if (more && e == 0) {
            k += min(f - k, kInlineSlots - lo_in);
            if (tb > -INFINITY) n_probes += ceil_log2_outcomes(kInlineSlots);
        }
        const bool need2 = more && e >= 1;
        int r2 = 0, l2 = 0;
        if (COUNT) {
            if (need2) {
                const uint32_t* src = lines + (uint64_t)ext_line(e - 1) * 32u;
                for (int x = 0; x < kSlotsPerLine; ++x) l2 += __uint_as_float(src[3 * x]) < tb ? 1 : 0;
                r2 = kSlotsPerLine;
            }
        } else {
            const uint64_t mask = __ballot(need2);
            const int total2 = __popcll(mask);
            if (total2 > 0) {
                const int rank2 = __popcll(mask & ((1ull << lane) - 1ull));
                if (need2) owner_of[rank2] = (unsigned char)lane;
                wave_lds_sync();
                const uint32_t line2 = need2 ? ext_line(e - 1) : 0u;
                const uint32_t par2 = (uint32_t)lane | ((uint32_t)kSlotsPerLine << 8) | ((uint32_t)(f - k) << 16) | (1u << 25);
#pragma unroll 1
                for (int b0 = 0; b0 < total2; b0 += 4 * kBatch) {
                    ext_issue(xb, lines, owner_of, b0, total2, lane, line2, par2);
                    ext_process<INCL>(xb, result_of, rows, rs, f, b0, lane, te, tb);
                }
                wave_lds_sync();
                if (need2) {
                    const int v = result_of[rank2];
                    r2 = v & 15;
                    l2 = v >> 4;
                }
                wave_lds_sync();
            }
        }
        if (need2) {
            k += max(r2 - max(l2, r2 - (f - k)), 0);
            if (tb > -INFINITY) n_probes += ceil_log2_outcomes(kSlotsPerLine);
        }
    }
    // ---- queries that walk the blocks (Algorithm 1 per lane) -------------------------------------------
    Walk<POLICY, INCL, pos_t> wk;
    wk.f = f;
    wk.s_pos = reinterpret_cast<pos_t*>(my_row);
    wk.edges = lines;
    wk.group = (POLICY == 0 && gshift >= 0) ? (1 << gshift) : 0;
    wk.te = te;
    wk.tb = tb;
    if (walked) {
        // the node's blocks, newest first: blocks outside the prefix (records in the directory run, oldest
        // first), then the prefix line by line.  A prefix line is presented as a block record whose latest
        // time is an upper bound (the next fence), which the walk's tests allow.
        const int64_t d0 = (int64_t)h_dir * kDirAlign;
        const bool dir_ok = nbig > 0 && d0 + nbig <= p.num_dir;
        const BlockRec* __restrict__ d = p.dir + d0;
        int32_t j0 = -1;                       // newest block outside the prefix that starts before the window end
        if (dir_ok) {
            int32_t lo = 0, hi = nbig;
            while (lo < hi) {
                const int32_t mid = lo + ((hi - lo) >> 1);
                const float tm = d[mid].t_min;
                ++wk.n_blocks;
                if (INCL ? (tm > te) : (tm >= te)) hi = mid; else lo = mid + 1;
            }
            j0 = lo - 1;
        }
        const int32_t n_big_walk = j0 + 1;     // visiting numbers 0 .. n_big_walk-1 are directory blocks
        const float after_prefix = dir_ok ? d[0].t_min : INFINITY;
        auto prefix_rec = [&](int32_t line_no) -> BlockRec {        // line_no: 0 = own line, 1..3 = extension lines
            if (line_no == 0)
                return make_rec(__uint_as_float(w[0]), n_ext > 0 ? fence(0) : after_prefix, nidx * kSlotsPerLine, n_in, tomb);
            const int32_t x = line_no - 1;
            const int32_t n = min(fill - kInlineSlots - kSlotsPerLine * x, kSlotsPerLine);
            return make_rec(fence(x), x + 1 < n_ext ? fence(x + 1) : after_prefix, (int64_t)ext_line(x) * kSlotsPerLine, n, tomb);
        };
        auto rec_at = [&](int32_t t) -> BlockRec {                   // record of visiting number t
            return t < n_big_walk ? d[j0 - t] : prefix_rec(n_ext - (t - n_big_walk));
        };
        bool go = true;
        int32_t t = 0;
        for (; t < n_big_walk && go; ++t) go = wk.step(d[j0 - t], t);
        for (int32_t x = n_ext; x >= 1 && go; --x, ++t) go = wk.step(prefix_rec(x), t);
        if (go && n_in > 0) {
            // the node's own line: both window ends are known from the registers
            ++wk.n_blocks;
            wk.n_probes += ceil_log2_outcomes(n_in) + (tb > -INFINITY ? ceil_log2_outcomes(hi_in) : 0);
            if (hi_in > lo_in) wk.record(nidx * kSlotsPerLine, lo_in, hi_in, tomb, n_big_walk + n_ext);
        }
        if (POLICY == 1 && wk.c > (int64_t)f) {
            wk.draw(p.seed, p.qid_base + q);
            int64_t cum = 0;
            for (int32_t u = wk.t_first; u <= wk.t_last; ++u) wk.resolve(rec_at(u), u, cum);
        }
    }
    // Recent policy: the wave finishes the in-block searches the walking lanes left open (sixteen lanes per query).
    int32_t h = 0;
    if (POLICY == 0 && gshift >= 0 && __ballot(walked && wk.d_off >= 0)) {
        // group g serves query it * groups + g in iteration it; the query's search window reaches the group
        // by shuffles, the count goes back through LDS
        constexpr int G = kCoopGroup, groups = kWave / G;
        unsigned char* s_h = my_lds + rows_bytes + 2 * kWave;
        static_assert(kExtraLds >= 3 * kWave, "room for one byte per query behind the request bytes");
        const int64_t win0 = wk.d_off + wk.d_lo;
        const int32_t my_n = (walked && wk.d_off >= 0) ? wk.d_n : 0;
        const int g = lane / G, j = lane % G;
        float tj[G];
#pragma unroll
        for (int it = 0; it < G; ++it) {
            const int src = it * groups + g;
            const int64_t w0 = shfl64(win0, src);
            tj[it] = 0.0f;
            if (j < __shfl(my_n, src, kWave)) {
                const auto wi = (typename index_of<pos_t>::type)slot_word(w0 + j);
                tj[it] = __uint_as_float(lines[wi]);
            }
        }
#pragma unroll
        for (int it = 0; it < G; ++it) {
            const int src = it * groups + g;
            const int32_t n = __shfl(my_n, src, kWave);
            const float teq = __shfl(te, src, kWave);
            const bool qual = j < n && (INCL ? (tj[it] <= teq) : (tj[it] < teq));
            const uint64_t m = __ballot(qual);
            if (j == 0) s_h[src] = (unsigned char)__popcll((m >> (g * G)) & ((1ull << G) - 1));
        }
        wave_lds_sync();
        if (walked && wk.d_off >= 0) h = wk.d_lo + (int32_t)s_h[lane];
        wave_lds_sync();
    }
    if (walked) {
        k = POLICY == 0 ? min(f, h + wk.k) : wk.k;
        if (POLICY == 0 && h > 0) {
            const int32_t hh = min(h, f);
            for (int32_t j = k - 1; j >= hh; --j) wk.s_pos[j] = wk.s_pos[j - hh];
            for (int32_t j = 0; j < hh; ++j) wk.s_pos[j] = (pos_t)slot_word(wk.d_off + h - 1 - j);
        }
        n_blocks += wk.n_blocks;
        n_probes += wk.n_probes;
    }
    if (COUNT) {
        unsigned long long v4[4] = {(unsigned long long)(nidx >= 0 ? 1 : 0), (unsigned long long)n_blocks,
                                    (unsigned long long)n_probes, (unsigned long long)k};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned long long v = v4[i];
            for (int dd = 32; dd >= 1; dd >>= 1) v += __shfl_xor(v, dd, kWave);
            if (lane == 0 && v) atomicAdd(&p.counters[i], v);
        }
        return;
    }
    // Fan-outs up to ten: everything goes through the rows (walked queries: rotation 0 after walked_gather).
    // Larger fan-outs: every query walked, the rows hold positions, the output stage gathers from memory.
    const bool row_path = POLICY == 0 && f <= kMaxFastFanout;
    const int32_t info = k | ((walked ? 0 : rot) << 8);
    const int32_t pstride = (int32_t)(rs * 4 / (int)sizeof(pos_t));     // row stride in positions
    const pos_t* __restrict__ w_pos = reinterpret_cast<const pos_t*>(rows);
    wave_lds_sync();      // rows were written by this wave's own lanes
    if (row_path && __ballot(walked && k > 0)) walked_gather<pos_t>(p, f_magic, rows, rs, lane, walked ? k : 0);

    // ---- outputs --------------------------------------------------------------------------------------
    if (FUSED) {
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
            // as in the other kernel: the waves count themselves in, the last one publishes the tile total,
            // every wave writes its padded rows, then the last wave looks back and only the dense copy waits
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
            if (row_path) rows_load(g, p, f_magic, rows, rs, lane, info);
            else gather_load<pos_t, POLICY == 1>(g, p, f_magic, pstride, w_pos, lane, 0, k);
            // Recent policy: the look-back reads come before this wave's stores (a load result can only be
            // waited for together with every store issued before it, and a store takes microseconds to be
            // taken).  Uniform policy: the other order measured faster, as in the other kernel.
            if (is_last && POLICY == 0) chain(wg_total);
            store_padded(g, p, f_magic, lane, 0, q0, Q);
            if (is_last && POLICY != 0) chain(wg_total);
            lds_barrier();
            const int64_t row = s_tile_base + offset_of_wave() + (inc - k);
            write_rowptr(row);
            store_dense(g, p, f_magic, lane, 0, row);
        } else {
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
            for (int32_t it0 = 0; it0 < f; it0 += kGatherChunk) {      // larger fan-outs: positions in the rows
                gather_load<pos_t, POLICY == 1>(g, p, f_magic, pstride, w_pos, lane, it0, k);
                store_padded(g, p, f_magic, lane, it0, q0, Q);
                store_dense(g, p, f_magic, lane, it0, row);
            }
        }
    } else {
        GatherRegs g;
        if (row_path) {
            rows_load(g, p, f_magic, rows, rs, lane, info);
            store_padded(g, p, f_magic, lane, 0, q0, Q);
        } else {
            for (int32_t it0 = 0; it0 < f; it0 += kGatherChunk) {
                gather_load<pos_t, POLICY == 1>(g, p, f_magic, pstride, w_pos, lane, it0, k);
                store_padded(g, p, f_magic, lane, it0, q0, Q);
            }
        }
    }
    if (q < Q && p.out_count) __builtin_nontemporal_store(k, &p.out_count[q]);
}

inline uint32_t magic_of(int32_t f) { return f <= 1 ? 0u : (uint32_t)(((uint64_t(1) << 32) + (uint64_t)f - 1) / (uint64_t)f); }

template <int POLICY, bool INCL, typename pos_t, bool COUNT, bool FUSED>
hipError_t launch_prefix_t(const SampleArgs& a, hipStream_t stream) {
    const int32_t f = a.fanout;
    const bool fast_rows = POLICY == 0 && f <= kMaxFastFanout;       // rows hold edges (3 words per slot)
    // row stride in 4-byte words: odd (conflict-free per-lane rows) for 32-bit contents, even when the row
    // holds 64-bit positions
    int32_t rs;
    if (sizeof(pos_t) == 8) rs = std::max(fast_rows ? (3 * f + 1) & ~1 : 0, 2 * (f | 1));
    else rs = fast_rows ? ((3 * f) | 1) : (f | 1);
    const size_t rows_bytes = ((size_t)kWave * rs * 4 + 15) & ~size_t(15);
    const int32_t gshift = (POLICY == 0 && f <= kCoopGroup) ? 4 : -1;
    // per wave: result rows, then 256 bytes for the line requests' owners and counts (the counts of the walking
    // lanes' cooperative searches); at least the 4 KiB in which the node lines are staged first, 32 at a time
    const size_t chunk = std::max<size_t>(rows_bytes + kExtraLds, 4096);
    // Workgroup size.  With the padding removal fused in, a workgroup is a tile of the chained scan: tiles
    // finish out of order (a tile of four waves is on average several hundred tiles ahead of the oldest
    // unfinished one when it has its total, and waits about as long as it sampled), so large tiles win
    // although a compute unit then holds a single workgroup (C5 at 2^26 queries, recent: 7.98 / 7.56 / 6.79 ms
    // with 4 / 8 / 16 waves; uniform: 7.10 / 6.91 / 7.83).  Without the scan small workgroups come and go more
    // evenly (4.33 / 4.43 / 4.87 / 6.17 ms with 1 / 2 / 4 / 16 waves).
    int waves = FUSED ? (POLICY == 0 ? 16 : 8) : 2;
    while (waves > 1 && (size_t)waves * chunk > (size_t)(159u << 10)) --waves;      // LDS of a workgroup: 160 KiB
    // small batches: smaller workgroups, so that the queries spread over the compute units
    while (waves > 1 && (a.Q + (int64_t)waves * kWave - 1) / ((int64_t)waves * kWave) < 512) waves >>= 1;
    const int64_t per_wg = (int64_t)waves * kWave;
    const int64_t grid = (a.Q + per_wg - 1) / per_wg;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (FUSED && !a.scan_ready) {
        const hipError_t e = launch_scan_init(a, grid + 1, stream);
        if (e != hipSuccess) return e;
    }
    if (grid <= 0) return hipGetLastError();
    const size_t lds = chunk * waves;
    auto kern = tns_sample_prefix_kernel<POLICY, INCL, pos_t, COUNT, FUSED>;
    SampleArgs b = a;
    if (FUSED && !b.err_flag) b.err_flag = &static_cast<ScanWorkspace*>(a.scan_ws)->error;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(waves * kWave), lds, stream, b, rs, magic_of(f), gshift, (uint32_t)chunk,
                       (uint32_t)rows_bytes);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sample_prefix(const SampleArgs& a, hipStream_t stream) {
    const bool incl = a.inclusive_end != 0;
    const bool wide = a.wide_offsets != 0;
#define TNS_DISPATCH(POL, CNT, FUS)                                                          \
    (incl ? (wide ? launch_prefix_t<POL, true, int64_t, CNT, FUS>(a, stream)                 \
                  : launch_prefix_t<POL, true, int32_t, CNT, FUS>(a, stream))                \
          : (wide ? launch_prefix_t<POL, false, int64_t, CNT, FUS>(a, stream)                \
                  : launch_prefix_t<POL, false, int32_t, CNT, FUS>(a, stream)))
    if (a.counters) return a.policy == 0 ? TNS_DISPATCH(0, true, false) : TNS_DISPATCH(1, true, false);
    if (a.scan_ws) return a.policy == 0 ? TNS_DISPATCH(0, false, true) : TNS_DISPATCH(1, false, true);
    return a.policy == 0 ? TNS_DISPATCH(0, false, false) : TNS_DISPATCH(1, false, false);
#undef TNS_DISPATCH
}

}  // namespace tns
