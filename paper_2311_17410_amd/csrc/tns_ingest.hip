// gfx950 kernels of the device-side store builder: edge insertion (section 4.1 of the paper:
// append to the node's tail block while it has room, else link a new block at the tail, sized by
// b_v = min(deg(v), tau)) and tombstone deletion, on batches that already live in device memory.
//
// One batch runs in two phases with one host read-back between them:
//   plan   validate -> stable LSD radix sort of (source, time) keys, arrival order as the tie-break ->
//          segment heads (one segment = the batch's edges of one source node) -> per segment: order
//          check against the stored tail, edges that still fit the tail block, capacity and number
//          of the new blocks, edge lines and directory records they need -> exclusive scans of
//          those needs (every segment gets its own range of the pools: no allocation atomics, the
//          layout is reproducible);
//   apply  per segment: tail record, new block records (inline shift or directory run, runs grow
//          by doubling), node entry; per edge: its slot from the segment's plan, one 12-byte store.
// Nothing is changed before the host has seen the plan's status (errors reject the whole batch)
// and made room in the pools.
#include "tns_ingest.h"
#include "tns_chain.h"

#include <algorithm>

#include "../../include/tns.h"

namespace tns {
namespace {

constexpr int kWave = 64;
constexpr int kThreads = 256;
constexpr int kScanPer = 8;
constexpr int kScanTile = kThreads * kScanPer;

struct SegPlan {
    int64_t tail_slot;   // slot after the tail block's last edge: where the first `take` edges go
    int64_t slab_slot;   // small blocks: slot of the first free position of the node's current line
    int32_t take;        // edges that fit the tail block
    int32_t cap;         // capacity of each new block (0: none)
    int32_t nbn;         // number of new blocks
    int32_t k0;          // small blocks: how many fit the node's current line
};
static_assert(sizeof(SegPlan) == 32, "32 bytes per segment");

__device__ __forceinline__ void report(IngestStatus* st, int status, int64_t pos) {
    atomicMin(&st->err_word, ((unsigned long long)pos << 8) | (unsigned long long)(-status));
}

__device__ __forceinline__ int64_t wave_sum64(int64_t v) {
    for (int d = 32; d >= 1; d >>= 1) v += (int64_t)__shfl_xor((long long)v, d, kWave);
    return v;
}

__global__ void __launch_bounds__(64) k_status_reset(IngestStatus* st) {
    if (threadIdx.x == 0) {
        st->err_word = ~0ull;
        st->unsorted = 0;
        st->num_segments = 0;
        st->total_lines = 0;
        st->total_dir = 0;
        st->new_blocks = 0;
        st->new_slots = 0;
        st->counter = 0;
    }
}

// ---- exclusive scan of an int64 array (three launches) -------------------------------------

__global__ void __launch_bounds__(kThreads) k_scan64_sums(const int64_t* __restrict__ in, int64_t n, int64_t* __restrict__ sums) {
    __shared__ int64_t s_w[kThreads / kWave];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPer;
    int64_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanPer; ++i)
        if (base + i < n) s += in[base + i];
    s = wave_sum64(s);
    if ((threadIdx.x & (kWave - 1)) == 0) s_w[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

__device__ __forceinline__ int64_t wave_inclusive64(int64_t v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int64_t u = (int64_t)__shfl_up((long long)v, d, kWave);
        if (lane >= d) v += u;
    }
    return v;
}

// one workgroup: exclusive scan of the tile sums in place, total to *total_out
__global__ void __launch_bounds__(1024) k_scan64_top(int64_t* __restrict__ sums, int64_t nb, int64_t* __restrict__ total_out) {
    __shared__ int64_t s_w[16];
    __shared__ int64_t s_carry;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < nb; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int64_t v = i < nb ? sums[i] : 0;
        const int64_t inc = wave_inclusive64(v, lane);
        if (lane == kWave - 1) s_w[wave] = inc;
        __syncthreads();
        int64_t off = 0, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int64_t t = s_w[w];
            if (w < wave) off += t;
            all += t;
        }
        const int64_t carry = s_carry;
        if (i < nb) sums[i] = carry + off + (inc - v);
        __syncthreads();
        if (threadIdx.x == 0) s_carry = carry + all;
        __syncthreads();
    }
    if (threadIdx.x == 0 && total_out) *total_out = s_carry;
}

__global__ void __launch_bounds__(kThreads) k_scan64_apply(const int64_t* in, int64_t* out, int64_t n,
                                                           const int64_t* __restrict__ sums) {
    __shared__ int64_t s_w[kThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPer;
    int64_t v[kScanPer];
    int64_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) {
        v[i] = base + i < n ? in[base + i] : 0;
        s += v[i];
    }
    const int64_t inc = wave_inclusive64(s, lane);
    if (lane == kWave - 1) s_w[wave] = inc;
    __syncthreads();
    int64_t run = sums[blockIdx.x] + (inc - s);
    for (int w = 0; w < wave; ++w) run += s_w[w];
#pragma unroll
    for (int i = 0; i < kScanPer; ++i) {
        if (base + i < n) out[base + i] = run;
        run += v[i];
    }
}

hipError_t exclusive_scan64(const int64_t* in, int64_t* out, int64_t n, int64_t* sums, int64_t* total_out, hipStream_t stream) {
    const int64_t nb = (n + kScanTile - 1) / kScanTile;
    if (nb > 0) hipLaunchKernelGGL(k_scan64_sums, dim3((unsigned)nb), dim3(kThreads), 0, stream, in, n, sums);
    hipLaunchKernelGGL(k_scan64_top, dim3(1), dim3(1024), 0, stream, sums, nb, total_out);
    if (nb > 0) hipLaunchKernelGGL(k_scan64_apply, dim3((unsigned)nb), dim3(kThreads), 0, stream, in, out, n, sums);
    return hipGetLastError();
}

// ---- keys, radix sort ----------------------------------------------------------------------

// Key = (source id, order-preserving image of the timestamp); the value is the batch position.
// -0.0 and +0.0 compare equal, so both take the key of +0.0 and keep their arrival order.
__global__ void __launch_bounds__(kThreads) k_keys(const IngestArgs a, uint64_t* __restrict__ key, uint32_t* __restrict__ val) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= a.m) return;
    const int32_t v = a.src[i];
    const float t = a.ts[i];
    if ((uint64_t)(uint32_t)v >= (uint64_t)a.num_nodes) report(a.status, TNS_ERANGE, i);
    else if (t != t) report(a.status, TNS_EORDER, i);
    else if (a.eid && a.eid[i] < 0) report(a.status, TNS_EINVAL, i);
    if (i > 0 && a.ts[i - 1] > t) atomicOr(&a.status->unsorted, 1u);
    uint32_t u = t == 0.0f ? 0u : __float_as_uint(t);
    u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
    key[i] = ((uint64_t)(uint32_t)v << 32) | u;
    val[i] = (uint32_t)i;
}

// The four passes over the timestamp bits are skipped (on the device) when the batch arrived
// in time order, the usual case for a stream.
__global__ void __launch_bounds__(kThreads) k_radix_hist(const uint64_t* __restrict__ key, int64_t m, int shift, int64_t chunk,
                                                         int nblk, uint32_t* __restrict__ hist, const IngestStatus* st, int skippable) {
    if (skippable && !st->unsorted) return;
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * chunk, hi = min(m, lo + chunk);
    for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) atomicAdd(&h[(uint32_t)(key[i] >> shift) & 255u], 1u);
    __syncthreads();
    hist[(size_t)threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];   // digit-major
}

__global__ void __launch_bounds__(1024) k_radix_scan(uint32_t* __restrict__ hist, int64_t n, const IngestStatus* st, int skippable) {
    if (skippable && !st->unsorted) return;
    __shared__ uint32_t s_w[16];
    __shared__ uint32_t s_carry;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < n; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const uint32_t v = i < n ? hist[i] : 0;
        uint32_t inc = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint32_t u = __shfl_up(inc, d, kWave);
            if (lane >= d) inc += u;
        }
        if (lane == kWave - 1) s_w[wave] = inc;
        __syncthreads();
        uint32_t off = 0, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const uint32_t t = s_w[w];
            if (w < wave) off += t;
            all += t;
        }
        const uint32_t carry = s_carry;
        if (i < n) hist[i] = carry + off + (inc - v);
        __syncthreads();
        if (threadIdx.x == 0) s_carry = carry + all;
        __syncthreads();
    }
}

// Stable scatter: a workgroup walks its chunk in tiles of 256 keys; inside a tile a key's rank among
// the keys with the same digit comes from wave ballots (lanes with equal digits) plus the counts of
// the earlier waves.
__global__ void __launch_bounds__(kThreads) k_radix_scatter(const uint64_t* __restrict__ kin, const uint32_t* __restrict__ vin,
                                                            uint64_t* __restrict__ kout, uint32_t* __restrict__ vout, int64_t m,
                                                            int shift, int64_t chunk, int nblk, const uint32_t* __restrict__ hist,
                                                            const IngestStatus* st, int skippable) {
    if (skippable && !st->unsorted) return;
    __shared__ uint32_t s_off[256];
    __shared__ uint32_t s_cnt[kThreads / kWave][256];
    const int t = threadIdx.x, lane = t & (kWave - 1), wave = t / kWave;
    s_off[t] = hist[(size_t)t * nblk + blockIdx.x];
#pragma unroll
    for (int w = 0; w < kThreads / kWave; ++w) s_cnt[w][t] = 0;
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * chunk, hi = min(m, lo + chunk);
    for (int64_t base = lo; base < hi; base += kThreads) {
        const int64_t i = base + t;
        const bool valid = i < hi;
        const uint64_t k = valid ? kin[i] : 0;
        const uint32_t d = (uint32_t)(k >> shift) & 255u;
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t bal = __ballot(bit);
            same &= bit ? bal : ~bal;
        }
        const uint32_t rank = (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
        if (valid && rank == 0) s_cnt[wave][d] = (uint32_t)__popcll(same);
        __syncthreads();
        if (valid) {
            uint32_t pos = s_off[d] + rank;
            for (int w = 0; w < wave; ++w) pos += s_cnt[w][d];
            if ((int64_t)pos < m) {
                kout[pos] = k;
                vout[pos] = vin[i];
            }
        }
        __syncthreads();
        uint32_t add = 0;
#pragma unroll
        for (int w = 0; w < kThreads / kWave; ++w) {
            add += s_cnt[w][t];
            s_cnt[w][t] = 0;
        }
        s_off[t] += add;
        __syncthreads();
    }
}

// ---- segments ------------------------------------------------------------------------------

__device__ __forceinline__ bool is_head(const uint64_t* key, int64_t p) {
    return p == 0 || (uint32_t)(key[p] >> 32) != (uint32_t)(key[p - 1] >> 32);
}

__global__ void __launch_bounds__(kThreads) k_heads(const uint64_t* __restrict__ key, int64_t m, int64_t* __restrict__ head) {
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p < m) head[p] = is_head(key, p) ? 1 : 0;
}

__global__ void __launch_bounds__(kThreads) k_seg_start(const uint64_t* __restrict__ key, int64_t m,
                                                        const int64_t* __restrict__ head_excl, int32_t* __restrict__ seg_start) {
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= m) return;
    const bool h = is_head(key, p);
    if (h) seg_start[head_excl[p]] = (int32_t)p;
    if (p == m - 1) seg_start[head_excl[p] + (h ? 1 : 0)] = (int32_t)m;
}

__device__ __forceinline__ int64_t dir_run_for(int64_t blocks, int64_t have) {
    int64_t n = have > 2 * kDirAlign ? have : 2 * kDirAlign;
    while (n < blocks) n *= 2;
    return n;
}

__device__ __forceinline__ int64_t lines_of_blocks(int32_t cap, int32_t nbn, int32_t k0) {
    if (nbn == 0) return 0;
    if (cap >= kSlotsPerLine) return (int64_t)nbn * ((cap + kSlotsPerLine - 1) / kSlotsPerLine);
    const int32_t per_line = kSlotsPerLine / cap;
    return (nbn - k0 + per_line - 1) / per_line;
}

// slot of the first edge of the segment's j-th new block; `line0` = first edge line of the segment's range
__device__ __forceinline__ int64_t block_slot(const SegPlan& P, int64_t line0, int32_t j) {
    if (P.cap >= kSlotsPerLine) return (line0 + (int64_t)j * ((P.cap + kSlotsPerLine - 1) / kSlotsPerLine)) * kSlotsPerLine;
    if (j < P.k0) return P.slab_slot + (int64_t)j * P.cap;
    const int32_t per_line = kSlotsPerLine / P.cap, jj = j - P.k0;
    return (line0 + jj / per_line) * kSlotsPerLine + (int64_t)(jj % per_line) * P.cap;
}

__device__ __forceinline__ const BlockRec* tail_of(const IngestArgs& a, const NodeLine& nd, int64_t nidx) {
    if (nd.nblocks <= kInlineBlocks) return &a.nodes[nidx].rec[0];
    return &a.dir[(int64_t)nd.dir_line * kDirAlign + nd.nblocks - 1];
}

// What one segment (the batch's edges p0..p1 of one source node, sorted) needs: how many edges the tail block
// still takes, the new blocks' capacity and number, the edge lines and directory records to reserve.
__device__ __forceinline__ void plan_segment(const IngestArgs& a, const uint64_t* __restrict__ key, const uint32_t* __restrict__ val,
                                             int32_t p0, int32_t p1, SegPlan& P, int64_t& lines, int64_t& dirs, int64_t& blocks,
                                             int64_t& slots) {
    const int64_t mm = p1 - p0;
    const uint32_t v = (uint32_t)(key[p0] >> 32);
    if ((uint64_t)v >= (uint64_t)a.num_nodes) return;      // out-of-range ids were reported with the keys
    const int64_t nidx = a.node_base + v;
    // the node entry's header and its newest inline record lie side by side: both are requested at once, with the
    // builder state and the segment's first timestamp, so that the plan is two dependent round trips, not four
    const uint4 h = *reinterpret_cast<const uint4*>(&a.nodes[nidx]);
    const uint4 r0 = *(reinterpret_cast<const uint4*>(&a.nodes[nidx]) + 1);
    const NodeAux ax = a.aux[nidx];
    const float t_first = a.ts[val[p0]];
    NodeLine nd;
    nd.nblocks = (int32_t)h.x; nd.degree = (int32_t)h.y; nd.dir_line = h.z;
    int64_t room = 0;
    if (nd.nblocks > 0) {
        BlockRec tr;
        if (nd.nblocks <= kInlineBlocks) {
            tr.t_min = __uint_as_float(r0.x); tr.t_max = __uint_as_float(r0.y); tr.off_lo = r0.z; tr.size_hi = r0.w;
        } else {
            tr = *tail_of(a, nd, nidx);
        }
        if (t_first < tr.t_max) report(a.status, TNS_EORDER, a.m + (int64_t)v);
        room = ax.tail_cap - rec_size(tr);
        P.tail_slot = rec_off(tr) + rec_size(tr);
    }
    const int64_t take = room < mm ? (room > 0 ? room : 0) : mm;
    const int64_t rest = mm - take;
    P.take = (int32_t)take;
    if (rest > 0) {
        int64_t cap;
        if (a.sizing == TNS_SIZING_STRAWMAN) cap = rest;
        else if (a.sizing == TNS_SIZING_FIXED) cap = a.tau;
        else cap = max(rest, min((int64_t)nd.degree + take, (int64_t)a.tau));   // b_v = min(deg(v), tau)
        cap = min(cap, kMaxBlockEdges);
        P.cap = (int32_t)cap;
        P.nbn = (int32_t)((rest + cap - 1) / cap);
        if (cap < kSlotsPerLine && ax.slab_line) {
            P.k0 = min(P.nbn, (kSlotsPerLine - ax.slab_used) / (int32_t)cap);
            P.slab_slot = (int64_t)(ax.slab_line - 1) * kSlotsPerLine + ax.slab_used;
        }
        lines = lines_of_blocks(P.cap, P.nbn, P.k0);
        const int64_t after = (int64_t)nd.nblocks + P.nbn;
        if (after > kInlineBlocks && after > ax.dir_cap) dirs = dir_run_for(after, ax.dir_cap);
        blocks = P.nbn;
        slots = (int64_t)P.nbn * cap;
    }
}

// totals of the new blocks and their capacities: one pair of atomics per workgroup (atomics on one word serialise)
template <int WAVES = kThreads / kWave>
__device__ __forceinline__ void add_block_totals(IngestStatus* st, int64_t blocks, int64_t slots) {
    __shared__ int64_t s_blocks[WAVES], s_slots[WAVES];
    blocks = wave_sum64(blocks);
    slots = wave_sum64(slots);
    if ((threadIdx.x & (kWave - 1)) == 0) {
        s_blocks[threadIdx.x / kWave] = blocks;
        s_slots[threadIdx.x / kWave] = slots;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        blocks = slots = 0;
        for (int w = 0; w < WAVES; ++w) {
            blocks += s_blocks[w];
            slots += s_slots[w];
        }
        if (blocks) {
            atomicAdd(&st->new_blocks, (unsigned long long)blocks);
            atomicAdd(&st->new_slots, (unsigned long long)slots);
        }
    }
}

__global__ void __launch_bounds__(kThreads) k_plan(const IngestArgs a, const uint64_t* __restrict__ key, const uint32_t* __restrict__ val,
                                                   const int32_t* __restrict__ seg_start, SegPlan* __restrict__ plan,
                                                   int64_t* __restrict__ need_lines, int64_t* __restrict__ need_dir) {
    const int64_t s = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int64_t blocks = 0, slots = 0;
    if (s < a.m) {
        int64_t lines = 0, dirs = 0;
        if (s < a.status->num_segments) {
            SegPlan P{};
            plan_segment(a, key, val, seg_start[s], seg_start[s + 1], P, lines, dirs, blocks, slots);
            plan[s] = P;
        }
        need_lines[s] = lines;
        need_dir[s] = dirs;
    }
    add_block_totals(a.status, blocks, slots);
}

// One thread per segment: tail record, new block records, node entry, builder state.
__global__ void __launch_bounds__(kThreads) k_apply_nodes(const IngestArgs a, const uint32_t* __restrict__ val,
                                                          const int32_t* __restrict__ seg_start, const SegPlan* __restrict__ plan,
                                                          const int64_t* __restrict__ lines_base, const int64_t* __restrict__ dir_base,
                                                          int64_t num_segments, const uint64_t* __restrict__ key) {
    const int64_t s = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (s >= num_segments) return;
    const SegPlan P = plan[s];
    const int32_t p0 = seg_start[s], p1 = seg_start[s + 1];
    const int64_t mm = p1 - p0;
    const int64_t nidx = a.node_base + (uint32_t)(key[p0] >> 32);
    NodeLine* N = &a.nodes[nidx];
    NodeAux ax = a.aux[nidx];
    const int32_t nb = N->nblocks;
    if (P.take > 0) {
        BlockRec* tr = nb <= kInlineBlocks ? &N->rec[0] : &a.dir[(int64_t)N->dir_line * kDirAlign + nb - 1];
        const BlockRec o = *tr;
        *tr = make_rec(o.t_min, a.ts[val[p0 + P.take - 1]], rec_off(o), rec_size(o) + P.take, rec_tombstones(o));
    }
    const int64_t degree_before = N->degree;
    N->degree += (int32_t)mm;
    if (P.nbn > 0) {
        const int64_t lines = lines_of_blocks(P.cap, P.nbn, P.k0);
        const int64_t line0 = a.used_lines + lines_base[s];
        if (line0 + lines > a.cap_lines) { atomicOr(&a.status->internal, 1u); return; }
        const int64_t after = (int64_t)nb + P.nbn;
        const int64_t rest = mm - P.take;
        BlockRec* run = nullptr;
        if (after > kInlineBlocks) {
            if (after > ax.dir_cap) {
                const int64_t n = dir_run_for(after, ax.dir_cap);
                const int64_t start = a.used_dir + dir_base[s];
                if (start + n > a.cap_dir) { atomicOr(&a.status->internal, 2u); return; }
                BlockRec* dst = a.dir + start;
                uint32_t* dcum = a.dir_cum + start;
                if (nb <= kInlineBlocks) {
                    uint32_t before = 0;
                    for (int j = 0; j < nb; ++j) {                                       // oldest first
                        const BlockRec o = N->rec[nb - 1 - j];
                        dst[j] = o;
                        dcum[j] = before;
                        before += (uint32_t)rec_size(o);
                    }
                } else {
                    const BlockRec* old = a.dir + (int64_t)N->dir_line * kDirAlign;
                    const uint32_t* ocum = a.dir_cum + (int64_t)N->dir_line * kDirAlign;
                    for (int32_t j = 0; j < nb; ++j) {
                        dst[j] = old[j];
                        dcum[j] = ocum[j];
                    }
                }
                N->dir_line = (uint32_t)(start / kDirAlign);
                ax.dir_cap = (int32_t)n;
            }
            run = a.dir + (int64_t)N->dir_line * kDirAlign;
        } else {
            for (int j = nb - 1; j >= 0; --j) N->rec[j + P.nbn] = N->rec[j];            // newest first: make room in front
        }
        uint32_t* run_cum = run ? a.dir_cum + (int64_t)N->dir_line * kDirAlign : nullptr;
        for (int32_t j = 0; j < P.nbn; ++j) {
            const int64_t first = (int64_t)p0 + P.take + (int64_t)j * P.cap;
            const int64_t size = min((int64_t)P.cap, rest - (int64_t)j * P.cap);
            const BlockRec r = make_rec(a.ts[val[first]], a.ts[val[first + size - 1]], block_slot(P, line0, j), (int32_t)size);
            if (run) {
                run[nb + j] = r;
                run_cum[nb + j] = (uint32_t)(degree_before + P.take + (int64_t)j * P.cap);   // edges in the older blocks
            } else {
                N->rec[P.nbn - 1 - j] = r;
            }
        }
        N->nblocks = (int32_t)after;
        ax.tail_cap = P.cap;
        if (P.cap < kSlotsPerLine) {
            const int32_t per_line = kSlotsPerLine / P.cap, rem = P.nbn - P.k0;
            if (rem > 0) {
                ax.slab_line = (uint32_t)(line0 + lines - 1 + 1);
                ax.slab_used = ((rem - 1) % per_line + 1) * P.cap;
            } else {
                ax.slab_used += P.nbn * P.cap;
            }
        }
    }
    a.aux[nidx] = ax;
}

// One thread per edge (sorted position): its slot from the segment's plan.
__global__ void __launch_bounds__(kThreads) k_apply_edges(const IngestArgs a, const uint64_t* __restrict__ key,
                                                          const uint32_t* __restrict__ val, const int64_t* __restrict__ head_excl,
                                                          const int32_t* __restrict__ seg_start, const SegPlan* __restrict__ plan,
                                                          const int64_t* __restrict__ lines_base, int reset_status) {
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= a.m) return;
    if (p == 0 && reset_status) {
        // the host has read the plan; the record is made ready for the next batch here, so that the next
        // plan needs no launch of its own for it (`internal` stays: it is reported by the next read-back)
        IngestStatus* st = a.status;
        st->err_word = ~0ull;
        st->unsorted = 0;
        st->num_segments = 0;
        st->total_lines = 0;
        st->total_dir = 0;
        st->new_blocks = 0;
        st->new_slots = 0;
        st->counter = 0;
    }
    const int64_t s = head_excl[p] + (is_head(key, p) ? 1 : 0) - 1;
    const SegPlan P = plan[s];
    const int64_t r = p - seg_start[s];
    int64_t slot;
    if (r < P.take) {
        slot = P.tail_slot + r;
    } else {
        const int64_t rr = r - P.take;
        const int32_t j = (int32_t)(rr / P.cap);
        slot = block_slot(P, a.used_lines + lines_base[s], j) + (rr - (int64_t)j * P.cap);
    }
    if (slot / kSlotsPerLine >= a.cap_lines) { atomicOr(&a.status->internal, 4u); return; }
    const uint32_t e = val[p];
    const int64_t w = slot_word(slot);
    a.lines[w] = __float_as_uint(a.ts[e]);
    a.lines[w + 1] = (uint32_t)a.dst[e];
    a.lines[w + 2] = (uint32_t)(a.eid ? a.eid[e] : (int32_t)(a.eid_base + (int64_t)e));
}

// ---- short pipeline for stream-sized batches -------------------------------------------------
//
// A batch of the size streams are ingested in (the paper's 100 K edges) spends its time in launches,
// not in memory traffic, so the planning phase above (about 40 dependent launches) is cut to five
// for batches that fit kFastMaxBatch and arrive in time order, the usual case for a stream:
//   k_fast_keys      validation, keys, and every tile's histogram of the first digit;
//   k_fast_scatter   x 2: stable radix pass over one half of the source id's bits.  Every tile adds
//                    up the histograms of the tiles before it by itself (at most kFastMaxTiles rows, read
//                    from the L2), so a pass needs no separate scan launch and no tile waits for another;
//                    the first pass also counts the second digit per destination tile for the second pass;
//   k_fast_segments  segment heads, their numbering (chained scan over tiles) and the segment starts;
//   k_fast_plan      the per-segment plan and the pool offsets (two chained scans) in one launch.
// Time order is assumed, not known: k_fast_keys sets `unsorted` as the general pipeline does, and
// the host, which reads the status before anything is changed, then runs the general pipeline instead.
// keys per sort tile: small batches take smaller tiles so that they still spread over the compute units, large ones
// larger tiles so that the table of tile histograms every tile reads stays short (measured: 2^14 edges 0.071 / 0.090 ms
// with 1024 / 4096 keys per tile, 2^17 edges 0.117 / 0.125 ms with 2048 / 4096, 2^20 edges 0.635 / 0.538 ms)
constexpr int kFastTileMax = 4096;
inline int fast_tile_keys(int64_t m) { return m <= (int64_t(1) << 16) ? 1024 : (m <= (int64_t(1) << 17) ? 2048 : kFastTileMax); }
constexpr int kScatThreads = 512;                       // the radix passes: 8 waves x 8 keys per lane on the same tiles
constexpr int kFastMaxTiles = 512;
constexpr int64_t kFastMaxBatch = (int64_t)kFastTileMax * kFastMaxTiles;   // 2^21 edges
constexpr int kFastMaxBits = 12;                        // bits per digit: two digits cover 2^24 nodes
constexpr int kSegItems = 4;                            // positions per thread in k_fast_segments
constexpr int kPlanThreads = 1024;                      // k_fast_plan: one segment per thread, 1024 per tile
constexpr uint32_t kInternalScan = 8u;                  // IngestStatus::internal: a chained scan's bounded wait ran out


template <int WAVES = kThreads / kWave>
__device__ __forceinline__ int64_t block_exclusive_scan(int64_t v, int64_t* s_wave /* [WAVES] */, int64_t& total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    int64_t inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int64_t u = (int64_t)__shfl_up((long long)inc, d, kWave);
        if (lane >= d) inc += u;
    }
    if (lane == kWave - 1) s_wave[wave] = inc;
    __syncthreads();
    int64_t off = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const int64_t t = s_wave[w];
        if (w < wave) off += t;
        total += t;
    }
    __syncthreads();
    return off + inc - v;
}

// Tile index in launch order, and the sum of the totals of the tiles before it: one chained-scan step of a
// workgroup.  `total` is the tile's own sum; the inclusive prefix is published for the tiles after it.
// Called by one whole wave; lane 0 holds the result.  A bounded wait that runs out marks the scan's own error
// word (later tiles and kernels look at it) and the status record the host reads.
__device__ __forceinline__ int64_t chain_wave(ScanWorkspace* ws, IngestStatus* st, int64_t tile, int64_t total, int lane) {
    if (lane == 0 && tile > 0)
        __hip_atomic_store(&ws->status[tile], kStTotal | (uint64_t)total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int64_t excl = tile > 0 ? lookback_exclusive(ws, &ws->error, tile, lane) : 0;
    if (lane == 0) {
        __hip_atomic_store(&ws->status[tile], kStPrefix | (uint64_t)(excl + total), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (__hip_atomic_load(&ws->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicOr(&st->internal, kInternalScan);
    }
    return excl;
}

template <int TILE>
__global__ void __launch_bounds__(kThreads) k_fast_keys(const IngestArgs a, uint64_t* __restrict__ key, uint32_t* __restrict__ val,
                                                        uint32_t* __restrict__ hist1, uint32_t* __restrict__ hist2, int bits,
                                                        ScanWorkspace* seg_scan, ScanWorkspace* lines_scan, ScanWorkspace* dir_scan,
                                                        int seg_tiles, int plan_tiles) {
    extern __shared__ uint32_t s_hist[];     // [bins]
    const int bins = 1 << bits;
    for (int b = threadIdx.x; b < bins; b += kThreads) s_hist[b] = 0;
    __syncthreads();
    constexpr int kFastItems = TILE / kThreads;
    const int64_t base = (int64_t)blockIdx.x * TILE;
    int32_t v_[kFastItems], e_[kFastItems];
    float t_[kFastItems], tp_[kFastItems];
#pragma unroll
    for (int j = 0; j < kFastItems; ++j) {       // all loads first, clamped to the batch
        const int64_t i = min(base + (int64_t)j * kThreads + threadIdx.x, a.m - 1);
        v_[j] = a.src[i];
        t_[j] = a.ts[i];
        tp_[j] = a.ts[i > 0 ? i - 1 : 0];
        e_[j] = a.eid ? a.eid[i] : 0;
    }
#pragma unroll
    for (int j = 0; j < kFastItems; ++j) {
        const int64_t i = base + (int64_t)j * kThreads + threadIdx.x;
        if (i >= a.m) continue;
        const int32_t v = v_[j];
        const float t = t_[j];
        if ((uint64_t)(uint32_t)v >= (uint64_t)a.num_nodes) report(a.status, TNS_ERANGE, i);
        else if (t != t) report(a.status, TNS_EORDER, i);
        else if (e_[j] < 0) report(a.status, TNS_EINVAL, i);
        if (i > 0 && tp_[j] > t) atomicOr(&a.status->unsorted, 1u);
        uint32_t u = t == 0.0f ? 0u : __float_as_uint(t);
        u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
        key[i] = ((uint64_t)(uint32_t)v << 32) | u;
        val[i] = (uint32_t)i;
        atomicAdd(&s_hist[(uint32_t)v & (uint32_t)(bins - 1)], 1u);
    }
    __syncthreads();
    uint32_t* row1 = hist1 + (size_t)blockIdx.x * bins;
    uint32_t* row2 = hist2 + (size_t)blockIdx.x * bins;
    for (int b = threadIdx.x; b < bins; b += kThreads) {
        row1[b] = s_hist[b];
        row2[b] = 0;                      // filled by the first scatter pass
    }
    if (blockIdx.x == 0) {
        // tickets, error words and tile states of the three chained scans that follow
        for (int i = threadIdx.x; i < seg_tiles + 1; i += kThreads) seg_scan->status[i] = 0;
        for (int i = threadIdx.x; i < plan_tiles + 1; i += kThreads) {
            lines_scan->status[i] = 0;
            dir_scan->status[i] = 0;
        }
        if (threadIdx.x == 0) {
            seg_scan->ticket = 0; seg_scan->error = 0;
            lines_scan->ticket = 0; lines_scan->error = 0; lines_scan->pad[0] = 0;      // pad[0]: plan workgroups that are done
            dir_scan->ticket = 0; dir_scan->error = 0;
        }
    }
}

// One stable radix pass over `bits` bits of the key starting at `shift`.  A wave owns TILE / 8
// consecutive keys of the tile and takes them 64 at a time in order, so "earlier in the tile" is
// (wave, item, lane) order; a key's rank among equal digits is the count of its wave so far plus its rank
// among the lanes of the current item (ballots over the digit's bits).
template <int TILE>
__global__ void __launch_bounds__(kScatThreads) k_fast_scatter(const uint64_t* __restrict__ kin, const uint32_t* __restrict__ vin,
                                                           uint64_t* __restrict__ kout, uint32_t* __restrict__ vout, int64_t m,
                                                           int shift, int bits, int tiles, const uint32_t* __restrict__ hist,
                                                           uint32_t* __restrict__ hist_next, int shift_next) {
    extern __shared__ uint32_t smem[];
    const int bins = 1 << bits;
    uint32_t* s_off = smem;                     // [bins]  position of the tile's first key of each digit
    uint32_t* s_cnt = smem + bins;              // [waves][bins]
    __shared__ int64_t s_wave[kScatThreads / kWave];
    const int t = threadIdx.x, lane = t & (kWave - 1), wave = t / kWave;
    const int tile = blockIdx.x;
    const uint32_t mask = (uint32_t)(bins - 1);

    // keys with this digit in earlier tiles, and in all tiles: thread t owns `per` consecutive digits and reads
    // their counts of every tile (16-byte loads when it owns four or more)
    const int per = bins >= kScatThreads ? bins / kScatThreads : 1;
    int64_t mine = 0;
    if (per >= 4) {
        for (int k = 0; k < per; k += 4) {
            const int b = t * per + k;
            uint4 before = make_uint4(0, 0, 0, 0), all = make_uint4(0, 0, 0, 0);
            // eight rows are requested before the first is added up: the rows come from the L2 and a thread
            // that waited for each in turn would spend the whole pass here
            for (int r0 = 0; r0 < tiles; r0 += 8) {
                uint4 c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = min(r0 + u, tiles - 1);
                    c[u] = *reinterpret_cast<const uint4*>(hist + (size_t)r * bins + b);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = r0 + u;
                    if (r < tiles) { all.x += c[u].x; all.y += c[u].y; all.z += c[u].z; all.w += c[u].w; }
                    if (r < tile) { before.x += c[u].x; before.y += c[u].y; before.z += c[u].z; before.w += c[u].w; }
                }
            }
            s_off[b] = before.x; s_off[b + 1] = before.y; s_off[b + 2] = before.z; s_off[b + 3] = before.w;
            s_cnt[b] = all.x; s_cnt[b + 1] = all.y; s_cnt[b + 2] = all.z; s_cnt[b + 3] = all.w;   // parked in the first
            mine += (int64_t)all.x + all.y + all.z + all.w;                                        // wave's row for now
        }
    } else {
        for (int k = 0; k < per; ++k) {
            const int b = t * per + k;
            if (b >= bins) break;
            uint32_t before = 0, all = 0;
            for (int r0 = 0; r0 < tiles; r0 += 8) {
                uint32_t c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) c[u] = hist[(size_t)min(r0 + u, tiles - 1) * bins + b];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (r0 + u < tiles) all += c[u];
                    if (r0 + u < tile) before += c[u];
                }
            }
            s_off[b] = before;
            s_cnt[b] = all;
            mine += all;
        }
    }
    int64_t total;
    int64_t run = block_exclusive_scan<kScatThreads / kWave>(mine, s_wave, total);       // keys with a smaller digit than this thread's first
    for (int k = 0; k < per; ++k) {
        const int b = t * per + k;
        if (b >= bins) break;
        const uint32_t all = s_cnt[b];
        s_off[b] += (uint32_t)run;
        run += all;
    }
    __syncthreads();
    for (int i = t; i < bins * (kScatThreads / kWave); i += kScatThreads) s_cnt[i] = 0;
    __syncthreads();

    constexpr int kScatItems = TILE / kScatThreads;
    const int64_t wbase = (int64_t)tile * TILE + (int64_t)wave * (kScatItems * kWave);
    uint64_t k_[kScatItems];
    uint32_t v_[kScatItems], r_[kScatItems];
    uint32_t* my_cnt = s_cnt + (size_t)wave * bins;
#pragma unroll
    for (int j = 0; j < kScatItems; ++j) {       // all loads of the tile first
        const int64_t i = min(wbase + (int64_t)j * kWave + lane, m - 1);   // clamped: no load sits in a branch
        k_[j] = kin[i];
        v_[j] = vin[i];
    }
#pragma unroll
    for (int j = 0; j < kScatItems; ++j) {
        const int64_t i = wbase + (int64_t)j * kWave + lane;
        const bool valid = i < m;
        const uint32_t d = (uint32_t)(k_[j] >> shift) & mask;
        uint64_t same = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t bal = __ballot(bit);
            same &= bit ? bal : ~bal;
        }
        const int leader = same ? __builtin_ctzll(same) : 0;
        uint32_t prev = 0;
        if (valid && lane == leader) {
            prev = my_cnt[d];
            my_cnt[d] = prev + (uint32_t)__popcll(same);
        }
        prev = (uint32_t)__shfl((int)prev, leader, kWave);
        r_[j] = prev + (uint32_t)__popcll(same & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    // a wave's keys of a digit follow those of the earlier waves
    for (int b = t; b < bins; b += kScatThreads) {
        uint32_t acc = 0;
#pragma unroll
        for (int w = 0; w < kScatThreads / kWave; ++w) {
            const uint32_t c = s_cnt[(size_t)w * bins + b];
            s_cnt[(size_t)w * bins + b] = acc;
            acc += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kScatItems; ++j) {
        const int64_t i = wbase + (int64_t)j * kWave + lane;
        if (i >= m) continue;
        const uint32_t d = (uint32_t)(k_[j] >> shift) & mask;
        const uint32_t pos = s_off[d] + my_cnt[d] + r_[j];
        if ((int64_t)pos < m) {                 // always true for consistent histograms; keeps a bad one in bounds
            kout[pos] = k_[j];
            vout[pos] = v_[j];
            if (hist_next) atomicAdd(&hist_next[(size_t)(pos / TILE) * bins + ((uint32_t)(k_[j] >> shift_next) & mask)], 1u);
        }
    }
}

// Sorted keys -> segment heads, head_excl[p] = number of heads before position p, seg_start[s] = first
// position of segment s (and m after the last), status->num_segments.
__global__ void __launch_bounds__(kThreads) k_fast_segments(const uint64_t* __restrict__ key, int64_t m, int64_t* __restrict__ head_excl,
                                                            int32_t* __restrict__ seg_start, ScanWorkspace* ws, IngestStatus* st) {
    __shared__ int64_t s_wave[kThreads / kWave];
    __shared__ int64_t s_tile, s_excl;
    if (threadIdx.x == 0) s_tile = (int64_t)atomicAdd(&ws->ticket, 1u);
    __syncthreads();
    const int64_t tile = s_tile;
    const int64_t p0 = (tile * kThreads + threadIdx.x) * kSegItems;
    int h[kSegItems];
    int64_t mine = 0;
#pragma unroll
    for (int j = 0; j < kSegItems; ++j) {
        const int64_t p = p0 + j;
        h[j] = (p < m && is_head(key, p)) ? 1 : 0;
        mine += h[j];
    }
    int64_t total;
    int64_t run = block_exclusive_scan(mine, s_wave, total);
    if (threadIdx.x < kWave) {
        const int64_t excl = chain_wave(ws, st, tile, total, threadIdx.x);
        if (threadIdx.x == 0) s_excl = excl;
    }
    __syncthreads();
    run += s_excl;
#pragma unroll
    for (int j = 0; j < kSegItems; ++j) {
        const int64_t p = p0 + j;
        if (p >= m) break;
        head_excl[p] = run;
        if (h[j]) seg_start[run] = (int32_t)p;
        run += h[j];
        if (p == m - 1) {
            seg_start[run] = (int32_t)m;
            st->num_segments = run;
        }
    }
}

// The per-segment plan and, in the same launch, every segment's offset into the edge-line and directory pools.
__global__ void __launch_bounds__(kPlanThreads) k_fast_plan(const IngestArgs a, const uint64_t* __restrict__ key,
                                                            const uint32_t* __restrict__ val, const int32_t* __restrict__ seg_start,
                                                            SegPlan* __restrict__ plan, int64_t* __restrict__ lines_base,
                                                            int64_t* __restrict__ dir_base, const ScanWorkspace* seg_scan,
                                                            ScanWorkspace* lines_scan, ScanWorkspace* dir_scan, int plan_tiles) {
    constexpr int kWaves = kPlanThreads / kWave;
    __shared__ int64_t s_wave[kWaves];
    __shared__ int64_t s_tile, s_excl_lines, s_excl_dir;
    if (threadIdx.x == 0) s_tile = (int64_t)atomicAdd(&lines_scan->ticket, 1u);
    __syncthreads();
    const int64_t tile = s_tile;
    // a time-out of the segment numbering leaves seg_start incomplete: nothing may be read through it
    const bool ok = seg_scan->error == 0;
    const int64_t nseg = ok ? a.status->num_segments : 0;
    const int64_t s = tile * kPlanThreads + threadIdx.x;
    int64_t lines = 0, dirs = 0, blocks = 0, slots = 0;
    if (s < nseg) {
        SegPlan P{};
        plan_segment(a, key, val, seg_start[s], seg_start[s + 1], P, lines, dirs, blocks, slots);
        plan[s] = P;
    }
    int64_t tot_lines, tot_dir;
    const int64_t in_lines = block_exclusive_scan<kWaves>(lines, s_wave, tot_lines);
    const int64_t in_dir = block_exclusive_scan<kWaves>(dirs, s_wave, tot_dir);
    // the two look-backs run side by side in the first two waves
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (wave < 2) {
        const int64_t excl = chain_wave(wave == 0 ? lines_scan : dir_scan, a.status, tile, wave == 0 ? tot_lines : tot_dir, lane);
        if (lane == 0) *(wave == 0 ? &s_excl_lines : &s_excl_dir) = excl;
    }
    __syncthreads();
    if (s < a.m) {
        lines_base[s] = s_excl_lines + in_lines;
        dir_base[s] = s_excl_dir + in_dir;
    }
    if (tile == plan_tiles - 1 && threadIdx.x == 0) {
        a.status->total_lines = s_excl_lines + tot_lines;
        a.status->total_dir = s_excl_dir + tot_dir;
    }
    add_block_totals<kWaves>(a.status, blocks, slots);
    if (a.host_status) {
        // The workgroup that finishes last hands the record to the host.  Every workgroup's updates of the record
        // have been performed when it counts itself in (the barrier waits for the threads' memory operations, the
        // fence orders thread 0's own); the copy reads past the caches of this compute unit.
        __syncthreads();
        if (threadIdx.x == 0) {
            __threadfence();
            const uint32_t before = atomicAdd(&lines_scan->pad[0], 1u);
            if (before == (uint32_t)plan_tiles - 1u) {
                __threadfence();
                const unsigned long long* src = reinterpret_cast<const unsigned long long*>(a.status);
                unsigned long long* dst = reinterpret_cast<unsigned long long*>(a.host_status);
                for (int i = 0; i < (int)(sizeof(IngestStatus) / 8); ++i)
                    dst[i] = __hip_atomic_load(&src[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __threadfence_system();
                __hip_atomic_store(a.host_seq, a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        }
    }
}

// ---- deletion, statistics ------------------------------------------------------------------

__global__ void __launch_bounds__(kThreads) k_delete_edges(NodeLine* nodes, BlockRec* dir, uint32_t* lines, int64_t node_base,
                                                           const int32_t* __restrict__ src, const int32_t* __restrict__ eid, int64_t n,
                                                           IngestStatus* st) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    NodeLine* N = &nodes[node_base + src[i]];
    const int32_t e = eid[i];
    const int32_t nb = N->nblocks;
    unsigned long long hits = 0;
    for (int32_t b = 0; b < nb; ++b) {
        BlockRec* r = nb <= kInlineBlocks ? &N->rec[b] : &dir[(int64_t)N->dir_line * kDirAlign + b];
        const int64_t off = rec_off(*r);
        const int32_t size = rec_size(*r);
        bool here = false;
        for (int32_t k = 0; k < size; ++k) {
            uint32_t* w = &lines[slot_word(off + k) + 2];
            // only one of several requests for the same edge gets the hit
            if (*w == (uint32_t)e && atomicCAS(w, (uint32_t)e, ~(uint32_t)e) == (uint32_t)e) {
                here = true;
                ++hits;
            }
        }
        if (here) atomicOr(&r->size_hi, 0x80000000u);
    }
    if (hits) {
        atomicOr(reinterpret_cast<unsigned int*>(&N->flags), 2u);
        atomicAdd(&st->counter, hits);
    }
}

__global__ void __launch_bounds__(kThreads) k_delete_nodes(NodeLine* nodes, int64_t node_base, const int32_t* __restrict__ ids, int64_t n,
                                                           int32_t deleted) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    unsigned int* f = reinterpret_cast<unsigned int*>(&nodes[node_base + ids[i]].flags);
    if (deleted) atomicOr(f, 1u); else atomicAnd(f, ~1u);
}

__global__ void __launch_bounds__(kThreads) k_max_list_len(const NodeLine* __restrict__ nodes, int64_t first, int64_t count,
                                                           IngestStatus* st) {
    int64_t mx = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += (int64_t)gridDim.x * kThreads)
        mx = max(mx, (int64_t)nodes[first + i].nblocks);
    for (int d = 32; d >= 1; d >>= 1) mx = max(mx, (int64_t)__shfl_xor((long long)mx, d, kWave));
    if ((threadIdx.x & (kWave - 1)) == 0 && mx > 0) atomicMax(&st->counter, (unsigned long long)mx);
}

// ---- workspace -----------------------------------------------------------------------------

size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

struct Carve {
    uint64_t *keyA, *keyB;
    uint32_t *valA, *valB, *hist;
    int64_t *head_excl, *lines_base, *dir_base, *sums;
    int32_t* seg_start;
    SegPlan* plan;
    int64_t chunk;
    int nblk;
    // short pipeline (batches of at most kFastMaxBatch edges)
    uint32_t* tile_hist[2];        // [tiles][bins] per radix pass
    ScanWorkspace *seg_scan, *lines_scan, *dir_scan;
    int fast_tiles, seg_tiles, plan_tiles;
    size_t bytes;
};

Carve carve(void* ws, int64_t m) {
    Carve c{};
    // sort chunks: at least 2048 keys and at most 1024 chunks
    c.chunk = std::max<int64_t>(2048, ((m + 1023) / 1024 + kThreads - 1) / kThreads * kThreads);
    c.nblk = (int)std::max<int64_t>(1, (m + c.chunk - 1) / c.chunk);
    unsigned char* p = static_cast<unsigned char*>(ws);
    size_t o = 0;
    auto take = [&](size_t bytes) { unsigned char* r = p ? p + o : nullptr; o += align256(bytes); return r; };
    const size_t mm = (size_t)std::max<int64_t>(m, 1);
    c.keyA = reinterpret_cast<uint64_t*>(take(mm * 8));
    c.keyB = reinterpret_cast<uint64_t*>(take(mm * 8));
    c.valA = reinterpret_cast<uint32_t*>(take(mm * 4));
    c.valB = reinterpret_cast<uint32_t*>(take(mm * 4));
    c.hist = reinterpret_cast<uint32_t*>(take((size_t)256 * c.nblk * 4));
    c.head_excl = reinterpret_cast<int64_t*>(take(mm * 8));
    c.lines_base = reinterpret_cast<int64_t*>(take(mm * 8));
    c.dir_base = reinterpret_cast<int64_t*>(take(mm * 8));
    c.sums = reinterpret_cast<int64_t*>(take(((mm + kScanTile - 1) / kScanTile + 1) * 8));
    c.seg_start = reinterpret_cast<int32_t*>(take((mm + 1) * 4));
    c.plan = reinterpret_cast<SegPlan*>(take(mm * sizeof(SegPlan)));
    if (m <= kFastMaxBatch) {
        c.fast_tiles = (int)((mm + fast_tile_keys(m) - 1) / fast_tile_keys(m));
        c.seg_tiles = (int)((mm + kThreads * kSegItems - 1) / (kThreads * kSegItems));
        c.plan_tiles = (int)((mm + kPlanThreads - 1) / kPlanThreads);
        for (int p2 = 0; p2 < 2; ++p2)
            c.tile_hist[p2] = reinterpret_cast<uint32_t*>(take((size_t)c.fast_tiles * (size_t(1) << kFastMaxBits) * 4));
        c.seg_scan = reinterpret_cast<ScanWorkspace*>(take(sizeof(ScanWorkspace) + (size_t)(c.seg_tiles + 1) * 8));
        c.lines_scan = reinterpret_cast<ScanWorkspace*>(take(sizeof(ScanWorkspace) + (size_t)(c.plan_tiles + 1) * 8));
        c.dir_scan = reinterpret_cast<ScanWorkspace*>(take(sizeof(ScanWorkspace) + (size_t)(c.plan_tiles + 1) * 8));
    }
    c.bytes = o;
    return c;
}

int src_passes(int64_t num_nodes) {
    int bits = 0;
    while (bits < 32 && (int64_t(1) << bits) < num_nodes) ++bits;
    return (bits + 7) / 8;
}

unsigned grid_for(int64_t n) { return (unsigned)std::max<int64_t>(1, (n + kThreads - 1) / kThreads); }

}  // namespace

size_t ingest_workspace_bytes(int64_t m) { return carve(nullptr, m).bytes; }

hipError_t ingest_status_reset(IngestStatus* status, hipStream_t stream) {
    hipLaunchKernelGGL(k_status_reset, dim3(1), dim3(64), 0, stream, status);
    return hipGetLastError();
}

hipError_t ingest_plan(const IngestArgs& a, hipStream_t stream) {
    if (a.m <= 0 || a.m > kMaxDeviceBatch) return hipErrorInvalidValue;
    const Carve c = carve(a.workspace, a.m);
    const int64_t m = a.m;
    hipLaunchKernelGGL(k_status_reset, dim3(1), dim3(64), 0, stream, a.status);
    hipLaunchKernelGGL(k_keys, dim3(grid_for(m)), dim3(kThreads), 0, stream, a, c.keyA, c.valA);
    // least significant digit first: 4 passes over the time bits (an even number, so a skipped
    // group leaves the data where it is), then the passes over the source id
    uint64_t *kin = c.keyA, *kout = c.keyB;
    uint32_t *vin = c.valA, *vout = c.valB;
    const int passes = 4 + src_passes(a.num_nodes);
    for (int p = 0; p < passes; ++p) {
        const int skippable = p < 4 ? 1 : 0;
        hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)c.nblk), dim3(kThreads), 0, stream, kin, m, 8 * p, c.chunk, c.nblk, c.hist,
                           a.status, skippable);
        hipLaunchKernelGGL(k_radix_scan, dim3(1), dim3(1024), 0, stream, c.hist, (int64_t)256 * c.nblk, a.status, skippable);
        hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)c.nblk), dim3(kThreads), 0, stream, kin, vin, kout, vout, m, 8 * p,
                           c.chunk, c.nblk, c.hist, a.status, skippable);
        std::swap(kin, kout);
        std::swap(vin, vout);
    }
    // kin / vin now name the sorted arrays
    hipLaunchKernelGGL(k_heads, dim3(grid_for(m)), dim3(kThreads), 0, stream, kin, m, c.head_excl);
    hipError_t e = exclusive_scan64(c.head_excl, c.head_excl, m, c.sums, &a.status->num_segments, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_seg_start, dim3(grid_for(m)), dim3(kThreads), 0, stream, kin, m, c.head_excl, c.seg_start);
    hipLaunchKernelGGL(k_plan, dim3(grid_for(m)), dim3(kThreads), 0, stream, a, kin, vin, c.seg_start, c.plan, c.lines_base,
                       c.dir_base);
    e = exclusive_scan64(c.lines_base, c.lines_base, m, c.sums, &a.status->total_lines, stream);
    if (e != hipSuccess) return e;
    return exclusive_scan64(c.dir_base, c.dir_base, m, c.sums, &a.status->total_dir, stream);
}

// Bits per digit of the short pipeline's two radix passes, or 0 if the batch does not qualify.
int fast_digit_bits(int64_t m, int64_t num_nodes) {
    if (m > kFastMaxBatch) return 0;
    int bits = 0;
    while (bits < 32 && (int64_t(1) << bits) < num_nodes) ++bits;
    if (bits > 2 * kFastMaxBits) return 0;
    return std::max(1, (bits + 1) / 2);
}

bool ingest_fast_ok(int64_t m, int64_t num_nodes) { return fast_digit_bits(m, num_nodes) > 0; }

hipError_t ingest_plan_fast(const IngestArgs& a, hipStream_t stream) {
    const int bits = fast_digit_bits(a.m, a.num_nodes);
    if (a.m <= 0 || bits <= 0) return hipErrorInvalidValue;
    const Carve c = carve(a.workspace, a.m);
    const int bins = 1 << bits;
    const size_t lds = (size_t)bins * 4 * (1 + kScatThreads / kWave);
#define TNS_FAST_SORT(TILE)                                                                                                          \
    do {                                                                                                                             \
        hipLaunchKernelGGL((k_fast_keys<TILE>), dim3((unsigned)c.fast_tiles), dim3(kThreads), (size_t)bins * 4, stream, a, c.keyA,  \
                           c.valA, c.tile_hist[0], c.tile_hist[1], bits, c.seg_scan, c.lines_scan, c.dir_scan, c.seg_tiles,          \
                           c.plan_tiles);                                                                                            \
        hipLaunchKernelGGL((k_fast_scatter<TILE>), dim3((unsigned)c.fast_tiles), dim3(kScatThreads), lds, stream, c.keyA, c.valA,    \
                           c.keyB, c.valB, a.m, 32, bits, c.fast_tiles, c.tile_hist[0], c.tile_hist[1], 32 + bits);                  \
        hipLaunchKernelGGL((k_fast_scatter<TILE>), dim3((unsigned)c.fast_tiles), dim3(kScatThreads), lds, stream, c.keyB, c.valB,    \
                           c.keyA, c.valA, a.m, 32 + bits, bits, c.fast_tiles, c.tile_hist[1], (uint32_t*)nullptr, 0);               \
    } while (0)
    switch (fast_tile_keys(a.m)) {
        case 1024: TNS_FAST_SORT(1024); break;
        case 2048: TNS_FAST_SORT(2048); break;
        default: TNS_FAST_SORT(kFastTileMax); break;
    }
#undef TNS_FAST_SORT
    hipLaunchKernelGGL(k_fast_segments, dim3((unsigned)c.seg_tiles), dim3(kThreads), 0, stream, c.keyA, a.m, c.head_excl, c.seg_start,
                       c.seg_scan, a.status);
    hipLaunchKernelGGL(k_fast_plan, dim3((unsigned)c.plan_tiles), dim3(kPlanThreads), 0, stream, a, c.keyA, c.valA, c.seg_start, c.plan,
                       c.lines_base, c.dir_base, c.seg_scan, c.lines_scan, c.dir_scan, c.plan_tiles);
    return hipGetLastError();
}

hipError_t ingest_apply(const IngestArgs& a, int64_t num_segments, bool fast, hipStream_t stream) {
    if (a.m <= 0 || num_segments <= 0 || num_segments > a.m) return hipErrorInvalidValue;
    const Carve c = carve(a.workspace, a.m);
    const bool in_b = !fast && (src_passes(a.num_nodes) & 1) != 0;
    const uint64_t* key = in_b ? c.keyB : c.keyA;
    const uint32_t* val = in_b ? c.valB : c.valA;
    hipLaunchKernelGGL(k_apply_edges, dim3(grid_for(a.m)), dim3(kThreads), 0, stream, a, key, val, c.head_excl, c.seg_start, c.plan,
                       c.lines_base, 1);
    hipLaunchKernelGGL(k_apply_nodes, dim3(grid_for(num_segments)), dim3(kThreads), 0, stream, a, val, c.seg_start, c.plan,
                       c.lines_base, c.dir_base, num_segments, key);
    return hipGetLastError();
}

hipError_t ingest_delete_edges(NodeLine* nodes, BlockRec* dir, uint32_t* lines, int64_t node_base, const int32_t* src,
                               const int32_t* eid, int64_t n, IngestStatus* status, hipStream_t stream) {
    hipLaunchKernelGGL(k_status_reset, dim3(1), dim3(64), 0, stream, status);
    if (n > 0)
        hipLaunchKernelGGL(k_delete_edges, dim3(grid_for(n)), dim3(kThreads), 0, stream, nodes, dir, lines, node_base, src, eid, n,
                           status);
    return hipGetLastError();
}

hipError_t ingest_delete_nodes(NodeLine* nodes, int64_t node_base, const int32_t* ids, int64_t n, int32_t deleted,
                               hipStream_t stream) {
    if (n > 0) hipLaunchKernelGGL(k_delete_nodes, dim3(grid_for(n)), dim3(kThreads), 0, stream, nodes, node_base, ids, n, deleted);
    return hipGetLastError();
}

hipError_t ingest_max_list_len(const NodeLine* nodes, int64_t first, int64_t count, IngestStatus* status, hipStream_t stream) {
    hipLaunchKernelGGL(k_status_reset, dim3(1), dim3(64), 0, stream, status);
    if (count > 0) {
        const unsigned grid = (unsigned)std::min<int64_t>(4096, (count + kThreads - 1) / kThreads);
        hipLaunchKernelGGL(k_max_list_len, dim3(grid), dim3(kThreads), 0, stream, nodes, first, count, status);
    }
    return hipGetLastError();
}

}  // namespace tns
