// Device-side building blocks shared by the sampling kernels (tns_kernels.hip, tns_kernels_prefix.hip):
// the chained scan over workgroup tiles, the per-lane block walk of Algorithm 1, the cooperative
// gather and the coalesced stores.  Included by .hip files only; everything has internal linkage.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "tns_chain.h"
#include "tns_kernels.h"

namespace tns {
namespace {

constexpr int kWave = 64;
constexpr int kXcds = 8;

// Workgroup -> tile mapping that gives each XCD (own L2) one contiguous range of tiles; the
// hardware hands consecutive workgroup ids to the XCDs round-robin.
__device__ __forceinline__ int64_t xcd_tile(int64_t bid, int64_t nb) {
    const int64_t q = nb / kXcds, r = nb % kXcds;
    const int64_t xcd = bid % kXcds, idx = bid / kXcds;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

__device__ __forceinline__ uint32_t div_by(uint32_t s, uint32_t f, uint32_t magic) {
    // floor(s / f) for s < 2^16 with magic = ceil(2^32 / f) (f >= 2)
    return f == 1 ? s : __umulhi(s, magic);
}

// Rank in [0, c) for slot j of query qid: splitmix64 output function on the counter
// seed + G * (qid * f + j + 1), top 32 bits scaled by multiply-shift.
__device__ __forceinline__ uint64_t pick_rank(uint64_t seed, int64_t qid, int32_t f, int32_t j, uint64_t c) {
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * ((uint64_t)qid * (uint64_t)f + (uint64_t)j + 1ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return ((z >> 32) * c) >> 32;
}

__device__ __forceinline__ int32_t wave_inclusive_scan(int32_t v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t u = __shfl_up(v, d, kWave);
        if (lane >= d) v += u;
    }
    return v;
}

constexpr int kCoopGroup = 16;        // lanes per query in the cooperative search (recent policy, fan-out <= 16)
constexpr int kGatherChunk = 10;      // gather iterations whose loads are issued together (8 and 5 measured slower)

// Unsigned index type of the same width as the LDS position entries: with a 32-bit index the edge
// load is addressed as base + 32-bit offset, one register per address.
template <typename pos_t> struct index_of { using type = uint64_t; };
template <> struct index_of<int32_t> { using type = uint32_t; };

// State of one lane's walk over the blocks of its target node, newest block first
// (Algorithm 1).  `t` numbers the blocks in visiting order.
template <int POLICY, bool INCL, typename pos_t>
struct Walk {
    float tb, te;                 // window [tb, te) or [tb, te]
    int32_t f;
    pos_t* s_pos;                 // this lane's f slots in LDS: word index of each selected edge
    const uint32_t* __restrict__ edges;   // edge lines as 4-byte words
    int32_t k = 0;                // slots filled so far (newest candidates first)
    int64_t c = 0;                // uniform: candidates seen in all overlapping blocks
    int32_t t_first = -1, t_last = -1, hi_first = 0, lo_last = 0;   // uniform: first/last overlapping block
    int32_t n_blocks = 0, n_probes = 0;                              // counted for the byte model
    // recent: search left to the wave.  When the window end falls inside a block, the lane only
    // narrows the search to at most `group` slots [d_lo, d_lo + d_n) of that block (edges before
    // d_lo are known to qualify); the wave then reads those timestamps side by side and counts,
    // right before it gathers from the same lines.
    int32_t group = 0;            // 0: the lane does every search itself
    int64_t d_off = -1;           // slot index of that block's first edge, -1: nothing left to the wave
    int32_t d_lo = 0, d_n = 0;

    // first index i in [0, n) with ts[i] >= x (STRICT=false) or ts[i] > x (STRICT=true)
    template <bool STRICT>
    __device__ __forceinline__ int32_t first_not_before(int64_t off, int32_t n, float x) {
        int32_t lo = 0, hi = n;
        while (lo < hi) {
            const int32_t mid = lo + ((hi - lo) >> 1);
            const float t = __uint_as_float(edges[slot_word(off + mid)]);   // Edge::ts is the first word
            ++n_probes;
            const bool ge = STRICT ? (t > x) : (t >= x);
            if (ge) hi = mid; else lo = mid + 1;
        }
        return lo;
    }

    // Examine one block; returns false when no older block can contribute.
    __device__ __forceinline__ bool step(const BlockRec& r, int32_t t) {
        ++n_blocks;
        if (INCL ? (te < r.t_min) : (te <= r.t_min)) return true;   // block lies after the window: next older
        if (tb > r.t_max) return false;                             // block lies before the window: stop
        const int32_t size = rec_size(r);
        const int64_t off = rec_off(r);
        // candidate range [lo, hi) of the block; t_min / t_max settle most cases without a search
        int32_t hi = size;
        const bool all_before_end = INCL ? (te >= r.t_max) : (te > r.t_max);
        const bool tomb = rec_tombstones(r);   // some edges of the block are deleted: they count as absent
        if (POLICY == 0 && group > 0 && !tomb && !all_before_end && !(tb > r.t_min)) {
            // only the newest overlapping block can contain the window end, so nothing is recorded yet
            int32_t lo = 0;
            while (hi - lo > group) {
                const int32_t mid = lo + ((hi - lo) >> 1);
                const float tm = __uint_as_float(edges[slot_word(off + mid)]);
                ++n_probes;
                const bool ge = INCL ? (tm > te) : (tm >= te);
                if (ge) hi = mid; else lo = mid + 1;
            }
            d_off = off; d_lo = lo; d_n = hi - lo;
            // the byte model counts what a binary search over the window would still read, not the
            // d_n timestamps the cooperating lanes fetch side by side
            n_probes += 32 - __clz(d_n);
            return true;            // older blocks supply the remaining slots
        }
        if (!all_before_end) hi = first_not_before<INCL>(off, size, te);
        int32_t lo = 0;
        if (tb > r.t_min) lo = first_not_before<false>(off, hi, tb);
        return record(off, lo, hi, tomb, t);
    }

    // Candidates [lo, hi) of the block whose edges start at slot `off` (visiting order t): records the
    // newest ones while slots are free and counts all of them for the uniform policy.  Returns false
    // when no older block can contribute.
    __device__ __forceinline__ bool record(int64_t off, int32_t lo, int32_t hi, bool tomb, int32_t t) {
        int32_t cnt = hi - lo;
        if (tomb) {
            // slow path: look at every candidate's validity (the edge id word), newest first
            cnt = 0;
            for (int32_t i = hi - 1; i >= lo; --i) {
                const int32_t id = (int32_t)edges[slot_word(off + i) + 2];
                ++n_probes;
                if (id < 0) continue;
                if (k < f) s_pos[k++] = (pos_t)slot_word(off + i);
                ++cnt;
                if (POLICY == 0 && k >= f) break;
            }
            if (POLICY == 1 && cnt > 0) {
                if (t_first < 0) { t_first = t; hi_first = hi; }
                t_last = t; lo_last = lo;
                c += cnt;
            }
        } else if (cnt > 0) {
            const int32_t take = min(f - k, cnt);
            for (int32_t j = 0; j < take; ++j) s_pos[k + j] = (pos_t)slot_word(off + hi - 1 - j);
            k += take > 0 ? take : 0;
            if (POLICY == 1) {
                if (t_first < 0) { t_first = t; hi_first = hi; }
                t_last = t; lo_last = lo;
                c += cnt;
            }
        }
        if (lo > 0) return false;                  // everything older is before the window
        if (POLICY == 0 && k >= f) return false;   // recent: the newest f are found
        return true;
    }

    // Uniform with more candidates than slots: f independent picks, rank counted from the
    // oldest candidate, stored as the negated distance from the newest one until resolved.
    __device__ __forceinline__ void draw(uint64_t seed, int64_t qid) {
        for (int32_t j = 0; j < f; ++j) {
            const int64_t from_newest = c - 1 - (int64_t)pick_rank(seed, qid, f, j, (uint64_t)c);
            s_pos[j] = (pos_t)(-(from_newest + 1));
        }
    }

    // Second visit of an overlapping block: turn the ranks that fall into it into positions.
    __device__ __forceinline__ void resolve(const BlockRec& r, int32_t t, int64_t& cum) {
        ++n_blocks;
        const int32_t hi = (t == t_first) ? hi_first : rec_size(r);
        const int32_t lo = (t == t_last) ? lo_last : 0;
        int64_t cnt = hi - lo;
        const int64_t off = rec_off(r);
        if (rec_tombstones(r)) {
            // ranks count valid edges only: walk them newest first
            cnt = 0;
            for (int32_t i = hi - 1; i >= lo; --i) {
                if ((int32_t)edges[slot_word(off + i) + 2] < 0) continue;
                for (int32_t j = 0; j < f; ++j) {
                    const int64_t sv = (int64_t)s_pos[j];
                    if (sv < 0 && -(sv + 1) - cum == cnt) s_pos[j] = (pos_t)slot_word(off + i);
                }
                ++cnt;
            }
        } else {
            for (int32_t j = 0; j < f; ++j) {
                const int64_t sv = (int64_t)s_pos[j];
                if (sv < 0) {
                    const int64_t rr = -(sv + 1) - cum;
                    if (rr < cnt) s_pos[j] = (pos_t)slot_word(off + hi - 1 - rr);
                }
            }
        }
        cum += cnt;
    }
};

// Ordering between LDS writes and reads of the SAME wave (rows are wave-private): the hardware
// executes a wave's LDS operations in order, so only the compiler must not reorder them.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also orders global memory: on
// gfx9 that is a wait for EVERY outstanding vector memory operation of the wave, stores included, and a
// store is only done when the L2 has taken it (microseconds under load).  Here the wave waits for its
// LDS operations and meets the others; its stores stay in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}


// Word index of the edge in slot j of a query: the first hq slots come from the block whose
// search the wave finished (newest first), the others from the positions the lane recorded.
// The wave's cooperative gather: its 64*f slots in flat order, lane l handles slot it*64 + l, so
// consecutive lanes read consecutive edges of one query (12-byte loads within one or two lines)
// and every store instruction covers 256 consecutive bytes of an output array.  The loads of up to
// kGatherChunk iterations are issued together, into registers, before anything is stored: the
// wave pays the memory latency once per batch instead of once per slot.
struct GatherRegs {
    int32_t nbr[kGatherChunk], eid[kGatherChunk];     // eid < 0: empty slot (edge ids are non-negative)
    float ts[kGatherChunk];
};

// BRANCHY: each load sits in its own branch instead (uniform policy: every slot of a query lies in another
// line and the variant below measured slower there, C5 step 35.4 against 31.2 ms).
template <typename pos_t, bool BRANCHY = false>
__device__ __forceinline__ void gather_load(GatherRegs& g, const SampleArgs& p, uint32_t f_magic, int32_t stride,
                                            const pos_t* __restrict__ w_pos, int lane, int32_t it0, int32_t k) {
    const int32_t f = p.fanout;
    // The loads are unconditional (an empty slot reads the first edge of the array and drops it) and all
    // issued before the first result is looked at: loads inside divergent branches make the compiler lose
    // count of the memory operations in flight, and it then waits for ALL of them, stores included, before
    // every store that follows.
    if (BRANCHY) {
#pragma unroll
        for (int i = 0; i < kGatherChunk; ++i) {
            g.nbr[i] = -1; g.eid[i] = -1; g.ts[i] = 0.0f;
            if (it0 + i < f) {
                const uint32_t s = (uint32_t)((it0 + i) * kWave + lane);
                const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
                const int32_t j = (int32_t)(s - ql * (uint32_t)f);
                const int32_t kq = __shfl(k, (int)ql, kWave);
                if (j < kq) {
                    const auto pos = (typename index_of<pos_t>::type)w_pos[ql * stride + j];
                    const Edge e = *reinterpret_cast<const Edge*>(p.edges + pos);
                    g.nbr[i] = e.nbr; g.eid[i] = e.eid; g.ts[i] = e.ts;
                }
            }
        }
        return;
    }
    bool filled[kGatherChunk];
    Edge raw[kGatherChunk];
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        filled[i] = false;
        raw[i].ts = 0.0f; raw[i].nbr = -1; raw[i].eid = -1;
        if (it0 + i < f) {          // uniform over the wave
            const uint32_t s = (uint32_t)((it0 + i) * kWave + lane);
            const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
            const int32_t j = (int32_t)(s - ql * (uint32_t)f);
            const int32_t kq = __shfl(k, (int)ql, kWave);
            filled[i] = j < kq;
            // an empty slot reads what the first filled slot of the instruction reads (one request for both;
            // a fixed address instead would make one memory channel everybody's)
            const uint64_t m = __ballot(filled[i]);
            const pos_t own = filled[i] ? w_pos[ql * stride + j] : (pos_t)0;
            const pos_t other = sizeof(pos_t) == 8 ? (pos_t)shfl64((int64_t)own, m ? __builtin_ctzll(m) : 0)
                                                   : (pos_t)__shfl((int)own, m ? __builtin_ctzll(m) : 0, kWave);
            const auto pos = (typename index_of<pos_t>::type)(filled[i] ? own : other);
            raw[i] = *reinterpret_cast<const Edge*>(p.edges + pos);
        }
    }
    // every load of the batch has returned before the first store is issued: the stores that follow then
    // go out back to back without waiting for one another
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0) only
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        g.nbr[i] = filled[i] ? raw[i].nbr : -1;
        g.eid[i] = filled[i] ? raw[i].eid : -1;
        g.ts[i] = filled[i] ? raw[i].ts : 0.0f;
    }
}

// padded rows: slots of queries below Q, empty slots get the sentinels
__device__ __forceinline__ void store_padded(const GatherRegs& g, const SampleArgs& p, uint32_t f_magic, int lane,
                                             int32_t it0, int64_t q0, int64_t Q) {
    if (!p.out_nbr) return;      // dense-only run: the padded rows are not materialised
    const int32_t f = p.fanout;
    const int64_t out0 = q0 * f;
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        if (it0 + i < f) {
            const uint32_t s = (uint32_t)((it0 + i) * kWave + lane);
            const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
            if (q0 + (int64_t)ql < Q) {
                __builtin_nontemporal_store(g.nbr[i], &p.out_nbr[out0 + s]);
                __builtin_nontemporal_store(g.eid[i], &p.out_eid[out0 + s]);
                __builtin_nontemporal_store(g.ts[i], &p.out_ts[out0 + s]);
            }
        }
    }
}

// dense copy: `row` = where the lane's own query starts; consecutive lanes write consecutive entries
__device__ __forceinline__ void store_dense(const GatherRegs& g, const SampleArgs& p, uint32_t f_magic, int lane,
                                            int32_t it0, int64_t row) {
    const int32_t f = p.fanout;
#pragma unroll
    for (int i = 0; i < kGatherChunk; ++i) {
        if (it0 + i < f) {
            const uint32_t s = (uint32_t)((it0 + i) * kWave + lane);
            const uint32_t ql = div_by(s, (uint32_t)f, f_magic);
            const int32_t j = (int32_t)(s - ql * (uint32_t)f);
            const int64_t rowq = shfl64(row, (int)ql);
            if (g.eid[i] >= 0) {
                p.cmp_nbr[rowq + j] = g.nbr[i];
                p.cmp_eid[rowq + j] = g.eid[i];
                p.cmp_ts[rowq + j] = g.ts[i];
            }
        }
    }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ BlockRec as_rec(const uint4& u) {
    BlockRec r;
    r.t_min = __uint_as_float(u.x);
    r.t_max = __uint_as_float(u.y);
    r.off_lo = u.z;
    r.size_hi = u.w;
    return r;
}

}  // namespace
}  // namespace tns
