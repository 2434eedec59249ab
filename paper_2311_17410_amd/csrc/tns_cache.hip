// Vectorised dynamic feature cache (section 4.3 of the paper) on gfx950: C ABI of
// include/tns_cache.h and its kernels.  Everything a fetch does is queued on the caller's stream:
// lookup, row gather, score update, selection of the victims (radix select over the scores),
// insertion of the missed rows.  No host round trip, no allocation.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdint>
#include <new>

#include "../../include/tns_cache.h"
#include "tns_internal.h"

using tns::DeviceGuard;
using tns::fail;
using tns::fail_hip;

namespace {

constexpr int kWave = 64;
constexpr int kScanTile = 1024;           // elements per workgroup in the scans
constexpr int kNoIndex = INT_MAX;
constexpr int kStripes = 64;

// Device-side scalars of one fetch.
struct Ctl {
    uint32_t prefix, mask;                // radix select: decided high bits of the threshold key (final, after four passes)
    int32_t remaining;                    // how many entries are still to be taken among keys equal to the threshold
    int32_t m;                            // entries replaced by this update
    int32_t n_unique;                     // distinct missed ids of the batch
    // state after each pass of the radix select (index p = after p passes; 0 = nothing decided) and the histogram
    // each pass fills: a pass's digit is picked by the kernel that follows it, in every workgroup's prologue
    uint32_t sel_prefix[5], sel_mask[5];
    int32_t sel_rem[5];
    int32_t hist[4][256];
};

struct CacheState {
    int32_t* slot_of;    // [num_ids]   slot of a cached id, -1 otherwise
    int32_t* first_idx;  // [num_ids]   scratch: first batch position of a missed id (kNoIndex between fetches)
    int32_t* id_of;      // [capacity]  id held by a slot, -1 if empty
    int32_t* score;      // [capacity]  recent score (LRU) / access count (LFU)
    int32_t* touched;    // [capacity]  LRU: accessed by the current batch
    float* rows;         // [capacity * dim]
    unsigned long long* counters;  // [kStripes][3]: hits, misses, replaced (striped: one hot word would serialise the batch)
    int64_t* ring;       // FIFO position
};

__global__ void __launch_bounds__(256) k_fill_i32(int32_t* p, int64_t n, int32_t v) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// slot_of from id_of (after a restore)
__global__ void __launch_bounds__(256) k_rebuild_map(const int32_t* __restrict__ id_of, int64_t capacity, int64_t num_ids,
                                                     int32_t* __restrict__ slot_of) {
    const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (s < capacity) {
        const int32_t id = id_of[s];
        if (id >= 0 && id < num_ids) slot_of[id] = (int32_t)s;
    }
}

// Lookup of the batch against the cache as it is before the update; accesses are recorded.  A thread takes
// kLookupUnroll ids, one grid width apart, and runs each dependent step for all of them before the next.
constexpr int kLookupUnroll = 4;
__global__ void __launch_bounds__(256) k_lookup(CacheState c, int policy, int64_t num_ids, int64_t B,
                                                const int32_t* __restrict__ ids, int32_t* __restrict__ slots,
                                                uint8_t* __restrict__ hit, Ctl* ctl) {
    if (blockIdx.x == 0) {          // scalars of this update
        if (threadIdx.x == 0) { ctl->prefix = 0; ctl->mask = 0; ctl->remaining = 0; ctl->m = 0; ctl->n_unique = 0; }
#pragma unroll
        for (int p4 = 0; p4 < 4; ++p4) ctl->hist[p4][threadIdx.x] = 0;
    }
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t b0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int32_t id[kLookupUnroll], s[kLookupUnroll];
#pragma unroll
    for (int u = 0; u < kLookupUnroll; ++u) id[u] = ids[min(b0 + (int64_t)u * stride, B - 1)];
#pragma unroll
    for (int u = 0; u < kLookupUnroll; ++u) {
        const bool in_range = id[u] >= 0 && id[u] < num_ids;
        s[u] = c.slot_of[in_range ? id[u] : 0];
        if (!in_range) s[u] = -2;                         // -2: id out of range
    }
    unsigned long long h = 0, m = 0;
#pragma unroll
    for (int u = 0; u < kLookupUnroll; ++u) {
        const int64_t b = b0 + (int64_t)u * stride;
        int is_hit = 0, is_miss = 0;
        if (b < B) {
            if (s[u] >= 0) {
                is_hit = 1;
                if (policy == TNS_CACHE_LRU) c.touched[s[u]] = 1;
                else if (policy == TNS_CACHE_LFU) atomicAdd(&c.score[s[u]], 1);
            } else if (s[u] == -1) {
                is_miss = 1;
                atomicMin(&c.first_idx[id[u]], (int32_t)b);   // first occurrence of a missed id
            }
            slots[b] = s[u];
            if (hit) hit[b] = (uint8_t)is_hit;
        }
        h += __popcll(__ballot(is_hit));
        m += __popcll(__ballot(is_miss));
    }
    if ((threadIdx.x & (kWave - 1)) == 0) {
        unsigned long long* mine = c.counters + (size_t)((blockIdx.x * 4 + (threadIdx.x >> 6)) % kStripes) * 3;
        if (h) atomicAdd(&mine[0], h);
        if (m) atomicAdd(&mine[1], m);
    }
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// out[b] = cached row or row of the backing store; VEC floats per thread, rows stay coalesced
// The slot comes from the id map directly (the threads of a row read the same two words), so the gather does not
// wait for the lookup kernel, which records the accesses for the update beside it.  A thread moves kGatherUnroll
// pieces, one grid width apart, and runs each dependent step (id, slot, row, store) for all of them before the next:
// the kernel is a copy, and a copy on this machine is bound by how much each compute unit has in flight.
constexpr int kGatherUnroll = 8;
template <int VEC>
__global__ void __launch_bounds__(256) k_gather(const float* __restrict__ rows, const float* __restrict__ store, int32_t dim,
                                                int64_t B, int64_t num_ids, const int32_t* __restrict__ ids,
                                                const int32_t* __restrict__ slot_of, float* __restrict__ out) {
    const int32_t per_row = dim / VEC;
    const int64_t total = B * per_row;
    const int64_t stride = (int64_t)gridDim.x * 256;
    const int64_t t0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t b[kGatherUnroll];
    int32_t col[kGatherUnroll], id[kGatherUnroll], s[kGatherUnroll];
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
        const int64_t t = min(t0 + (int64_t)u * stride, total - 1);      // clamped: no load sits in a branch
        b[u] = t / per_row;
        col[u] = (int32_t)(t - b[u] * per_row) * VEC;
        id[u] = ids[b[u]];
    }
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
        const bool in_range = id[u] >= 0 && id[u] < num_ids;
        s[u] = slot_of[in_range ? id[u] : 0];
        if (!in_range) s[u] = -2;                                         // -1: not cached, -2: id out of range
    }
    // the output and the rows of the backing store are touched once (non-temporal); the cached rows are
    // what should stay in the L2
    if (VEC == 4) {
        f32x4 v[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u) {
            const float* src = s[u] >= 0 ? rows + (int64_t)s[u] * dim + col[u] : store + (int64_t)(s[u] == -1 ? id[u] : 0) * dim + col[u];
            v[u] = s[u] >= 0 ? *reinterpret_cast<const f32x4*>(src) : __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src));
            if (s[u] == -2) v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (t0 + (int64_t)u * stride < total) __builtin_nontemporal_store(v[u], reinterpret_cast<f32x4*>(out + b[u] * dim + col[u]));
    } else {
        float v[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u) {
            const float* src = s[u] >= 0 ? rows + (int64_t)s[u] * dim + col[u] : store + (int64_t)(s[u] == -1 ? id[u] : 0) * dim + col[u];
            v[u] = s[u] >= 0 ? *src : __builtin_nontemporal_load(src);
            if (s[u] == -2) v[u] = 0.f;
        }
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (t0 + (int64_t)u * stride < total) __builtin_nontemporal_store(v[u], out + b[u] * dim + col[u]);
    }
}

// LRU: every score is decremented, accessed entries are reset to 0
__global__ void __launch_bounds__(256) k_lru_scores(int32_t* __restrict__ score, int32_t* __restrict__ touched, int64_t capacity) {
    const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (s < capacity) {
        score[s] = touched[s] ? 0 : score[s] - 1;
        touched[s] = 0;
    }
}

// ---- compaction of flagged elements in three launches -------------------------------------------
// A flag functor gives each element a packed 64-bit count (one or two counters); (1) per-tile sums,
// (2) exclusive scan of the tile sums by one workgroup, (3) per tile: the flags again, a local scan,
// and the functor's emit() with the number of flagged elements before each one.  No flag array.

__device__ __forceinline__ int32_t wave_inclusive_scan(int32_t v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int32_t u = __shfl_up(v, d, kWave);
        if (lane >= d) v += u;
    }
    return v;
}
__device__ __forceinline__ int64_t wave_inclusive_scan64(int64_t v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int64_t u = (int64_t)__shfl_up((long long)v, d, kWave);
        if (lane >= d) v += u;
    }
    return v;
}

constexpr int kPerThread = kScanTile / 256;

template <class F>
__global__ void __launch_bounds__(256) k_flag_tile_sums(const F f, int64_t n, int64_t* __restrict__ sums) {
    __shared__ int64_t s_w[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kPerThread;
    int64_t v = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
        if (base + i < n) v += f.count(base + i);
    const int lane = threadIdx.x & 63;
    v = wave_inclusive_scan64(v, lane);
    if (lane == 63) s_w[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

// one workgroup: exclusive scan of the tile sums in place; the functor receives the total
template <class F>
__global__ void __launch_bounds__(1024) k_flag_scan_sums(const F f, int64_t* __restrict__ sums, int64_t num_tiles) {
    __shared__ int64_t s_w[16];
    __shared__ int64_t s_carry;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < num_tiles; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int64_t v = i < num_tiles ? sums[i] : 0;
        const int64_t inc = wave_inclusive_scan64(v, lane);
        if (lane == 63) s_w[wave] = inc;
        __syncthreads();
        int64_t wave_off = 0, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int64_t t = s_w[w];
            if (w < wave) wave_off += t;
            all += t;
        }
        const int64_t carry = s_carry;
        if (i < num_tiles) sums[i] = carry + wave_off + (inc - v);
        __syncthreads();
        if (threadIdx.x == 0) s_carry = carry + all;
        __syncthreads();
    }
    if (threadIdx.x == 0) f.total(s_carry);
}

// FOLD: `sums` holds the raw tile sums and every workgroup adds up those of the tiles before it by itself (at most
// kFoldTiles of them, read from the L2); the last one also hands the total to the functor.  This saves the
// one-workgroup scan kernel between the two, which is slow beside a kernel that saturates the memory system.
constexpr int64_t kFoldTiles = 2048;
template <class F, bool FOLD>
__device__ __forceinline__ void flag_collect_body(const F& f, int64_t n, const int64_t* __restrict__ sums, int64_t bid, int64_t nblocks) {
    __shared__ int64_t s_w[4], s_t[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = bid * kScanTile + (int64_t)threadIdx.x * kPerThread;
    int64_t tile_off = 0;
    if (FOLD) {
        int64_t part = 0;
        for (int64_t t0 = 0; t0 < bid; t0 += 256 * 4) {
            int64_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t t = t0 + u * 256 + threadIdx.x;
                v[u] = sums[min(t, bid)];          // clamped: no load sits in a branch
                if (t >= bid) v[u] = 0;
            }
            part += v[0] + v[1] + v[2] + v[3];
        }
        part = wave_inclusive_scan64(part, lane);
        if (lane == 63) s_t[wave] = part;
    }
    int64_t c[kPerThread], sum = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        c[i] = base + i < n ? f.count(base + i) : 0;
        sum += c[i];
    }
    const int64_t inc = wave_inclusive_scan64(sum, lane);
    if (lane == 63) s_w[wave] = inc;
    __syncthreads();
    if (FOLD) tile_off = s_t[0] + s_t[1] + s_t[2] + s_t[3];
    else tile_off = sums[bid];
    int64_t before = tile_off + inc - sum;
    for (int w = 0; w < wave; ++w) before += s_w[w];
    if (FOLD && bid == nblocks - 1 && threadIdx.x == 0) f.total(tile_off + s_w[0] + s_w[1] + s_w[2] + s_w[3]);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        if (c[i]) f.emit(base + i, before);
        before += c[i];
    }
}

template <class F, bool FOLD>
__global__ void __launch_bounds__(256) k_flag_collect(const F f, int64_t n, const int64_t* __restrict__ sums) {
    flag_collect_body<F, FOLD>(f, n, sums, blockIdx.x, gridDim.x);
}

// Distinct missed ids in the order of their first occurrence (the flag: a missed row that is the first
// of its id), up to max_replace of them; the total fixes how many entries this update replaces.
struct NewIds {
    const int32_t* first_idx;
    const int32_t* ids;
    const int32_t* slots;
    int32_t max_replace;
    int32_t* new_ids;
    Ctl* ctl;
    __device__ int64_t count(int64_t b) const { return slots[b] == -1 && first_idx[ids[b]] == (int32_t)b ? 1 : 0; }
    __device__ void emit(int64_t b, int64_t before) const {
        if (before < max_replace) new_ids[before] = ids[b];
    }
    __device__ void total(int64_t n_unique) const {
        const int32_t m = (int32_t)(n_unique < max_replace ? n_unique : max_replace);
        ctl->n_unique = (int32_t)n_unique;
        ctl->m = m;
        ctl->remaining = m;
    }
};


// ---- victims: the m entries with the lowest (score, slot) --------------------------------------

__device__ __forceinline__ uint32_t score_key(int32_t score) { return (uint32_t)score ^ 0x80000000u; }   // unsigned order = signed order

// Radix select of the m-th smallest key, 8 bits per pass, most significant first.  A pass is one launch that
// histograms the digit over the entries whose decided high bits match; the digit in which the remaining-th
// smallest key falls is picked by the NEXT kernel, by every workgroup for itself in its prologue (a scan over
// 256 bins), so a pass needs no launch of its own for the pick.  Workgroup 0 also stores the state for whoever
// reads it later.  Called by all 256 threads of a workgroup; returns the state after `pass` passes.
struct SelState { uint32_t prefix, mask; int32_t rem; };
__device__ __forceinline__ SelState select_pick(Ctl* ctl, int pass /* 1..4 */, bool store) {
    __shared__ int32_t s_w[4];
    __shared__ SelState s_out;
    SelState prev;
    if (pass == 1) { prev.prefix = 0; prev.mask = 0; prev.rem = ctl->m; }
    else { prev.prefix = ctl->sel_prefix[pass - 1]; prev.mask = ctl->sel_mask[pass - 1]; prev.rem = ctl->sel_rem[pass - 1]; }
    const int shift = 32 - 8 * pass;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int32_t h = ctl->hist[pass - 1][threadIdx.x];
    int32_t inc = wave_inclusive_scan(h, lane);
    if (lane == 63) s_w[wave] = inc;
    __syncthreads();
    for (int w = 0; w < wave; ++w) inc += s_w[w];
    // the first bin whose inclusive count reaches rem; bin 255 if none does
    const bool mine = (inc >= prev.rem && inc - h < prev.rem) || (threadIdx.x == 255 && inc < prev.rem);
    if (mine) {
        s_out.prefix = prev.prefix | ((uint32_t)threadIdx.x << shift);
        s_out.mask = prev.mask | (255u << shift);
        s_out.rem = prev.rem - (inc - h);             // entries to take among keys equal to the threshold so far
    }
    __syncthreads();
    const SelState out = s_out;
    if (store && threadIdx.x == 0) {
        ctl->sel_prefix[pass] = out.prefix; ctl->sel_mask[pass] = out.mask; ctl->sel_rem[pass] = out.rem;
        if (pass == 4) { ctl->prefix = out.prefix; ctl->mask = out.mask; ctl->remaining = out.rem; }
    }
    __syncthreads();
    return out;
}

// Histogram of pass `pass` (0..3).  LRU_UPDATE (pass 0 under LRU): the scores are brought up to date on the way
// (every score decremented, entries accessed by the batch reset to 0); that pass does not know yet whether
// anything will be replaced and histograms regardless.  `bid` / `nb`: this workgroup's index and the number of
// workgroups that share the pass (the kernel may hold other work in its other workgroups).
template <bool LRU_UPDATE>
__device__ __forceinline__ void select_hist_body(int32_t* __restrict__ score, int32_t* __restrict__ touched, int64_t capacity,
                                                 int pass, Ctl* ctl, int64_t bid, int64_t nb) {
    __shared__ int32_t s_h[256];
    uint32_t prefix = 0, mask = 0;
    if (pass > 0) {
        if (ctl->m <= 0) return;
        const SelState st = select_pick(ctl, pass, bid == 0);
        prefix = st.prefix;
        mask = st.mask;
    }
    const int shift = 24 - 8 * pass;
    s_h[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t s = bid * 256 + threadIdx.x; s < capacity; s += nb * 256) {
        int32_t sc = score[s];
        if (LRU_UPDATE) {
            sc = touched[s] ? 0 : sc - 1;
            score[s] = sc;
            touched[s] = 0;
        }
        const uint32_t k = score_key(sc);
        if ((k & mask) == prefix) atomicAdd(&s_h[(k >> shift) & 255u], 1);
    }
    __syncthreads();
    if (s_h[threadIdx.x]) atomicAdd(&ctl->hist[pass][threadIdx.x], s_h[threadIdx.x]);
}

template <bool LRU_UPDATE>
__global__ void __launch_bounds__(256) k_select_hist(int32_t* __restrict__ score, int32_t* __restrict__ touched, int64_t capacity,
                                                     int pass, Ctl* ctl) {
    select_hist_body<LRU_UPDATE>(score, touched, capacity, pass, ctl, blockIdx.x, gridDim.x);
}

// The victims in ascending slot order: every entry below the threshold key and the first `remaining`
// entries equal to it.  Packed count: entries below in the high word, equal entries in the low word.
struct Victims {
    const int32_t* score;
    const Ctl* ctl;
    int32_t* victims;
    __device__ int64_t count_with(int64_t s, uint32_t t) const {
        const uint32_t k = score_key(score[s]);
        return k < t ? (int64_t(1) << 32) : (k == t ? 1 : 0);
    }
    __device__ int64_t count(int64_t s) const { return ctl->m <= 0 ? 0 : count_with(s, ctl->prefix); }
    __device__ void emit(int64_t s, int64_t before) const {
        const int64_t below_before = before >> 32, eq_before = before & 0xffffffffll, rem = ctl->remaining;
        const bool below = score_key(score[s]) < ctl->prefix;
        if (below || eq_before < rem) victims[below_before + (eq_before < rem ? eq_before : rem)] = (int32_t)s;
    }
    __device__ void total(int64_t) const {}
};

// Tile sums of the victims' compaction; the prologue picks the last digit of the radix select (the threshold is
// final from here on: workgroup 0 stores it for the collect kernel).
__global__ void __launch_bounds__(256) k_victims_tile_sums(const Victims f, Ctl* ctl, int64_t n, int64_t* __restrict__ sums) {
    __shared__ int64_t s_w[4];
    int64_t v = 0;
    if (ctl->m > 0) {
        const SelState st = select_pick(ctl, 4, blockIdx.x == 0);
        const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kPerThread;
#pragma unroll
        for (int i = 0; i < kPerThread; ++i)
            if (base + i < n) v += f.count_with(base + i, st.prefix);
    }
    const int lane = threadIdx.x & 63;
    v = wave_inclusive_scan64(v, lane);
    if (lane == 63) s_w[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) sums[blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}


// Two independent pieces of the update in one launch (the chain of short launches is what the update costs):
// workgroups [0, tiles) collect the distinct missed ids (which also fixes m), the other `hb` workgroups run pass 0
// of the radix select over the scores, which depends on the lookup only.
template <bool LRU_UPDATE>
__global__ void __launch_bounds__(256) k_newids_collect_hist0(const NewIds f, int64_t n, const int64_t* __restrict__ sums, int64_t tiles,
                                                              int32_t* __restrict__ score, int32_t* __restrict__ touched,
                                                              int64_t capacity, Ctl* ctl, int64_t hb) {
    if ((int64_t)blockIdx.x < tiles) flag_collect_body<NewIds, true>(f, n, sums, blockIdx.x, tiles);
    else select_hist_body<LRU_UPDATE>(score, touched, capacity, 0, ctl, (int64_t)blockIdx.x - tiles, hb);
}

__global__ void __launch_bounds__(256) k_fifo_victims(int64_t capacity, int32_t max_replace, int64_t* ring, const Ctl* ctl,
                                                      int32_t* __restrict__ victims) {
    const int32_t i = blockIdx.x * 256 + threadIdx.x;
    const int32_t m = ctl->m;
    const int64_t r = *ring;
    if (i < m) victims[i] = (int32_t)((r + i) % capacity);
}
__global__ void k_fifo_advance(int64_t capacity, int64_t* ring, const Ctl* ctl) { *ring = (*ring + ctl->m) % capacity; }

// one wave per replaced entry: maps, score, row copy from the backing store
__device__ __forceinline__ void insert_body(const CacheState& c, int policy, int32_t dim, const float* __restrict__ store,
                                            const int32_t* __restrict__ new_ids, const int32_t* __restrict__ victims, const Ctl* ctl,
                                            int64_t bid) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t i = bid * 4 + (threadIdx.x >> 6);
    if (i >= ctl->m) return;
    const int32_t s = victims[i], id = new_ids[i];
    if (lane == 0) {
        const int32_t old = c.id_of[s];
        if (old >= 0) c.slot_of[old] = -1;
        c.id_of[s] = id;
        c.slot_of[id] = s;
        c.score[s] = policy == TNS_CACHE_LFU ? 1 : 0;
        if (i == 0) atomicAdd(&c.counters[2], (unsigned long long)ctl->m);
    }
    const float* __restrict__ src = store + (int64_t)id * dim;
    float* __restrict__ dst = c.rows + (int64_t)s * dim;
    for (int32_t k = lane; k < dim; k += kWave) dst[k] = src[k];
}

// The insertion (workgroups [0, insert_blocks)) and the clearing of the batch's first-occurrence marks (the rest),
// which touch different arrays, in one launch at the end of the fetch.
__global__ void __launch_bounds__(256) k_insert_clear(CacheState c, int policy, int32_t dim, const float* __restrict__ store,
                                                      const int32_t* __restrict__ new_ids, const int32_t* __restrict__ victims,
                                                      const Ctl* ctl, int64_t insert_blocks, int64_t B,
                                                      const int32_t* __restrict__ ids, const int32_t* __restrict__ slots) {
    if ((int64_t)blockIdx.x < insert_blocks) {
        insert_body(c, policy, dim, store, new_ids, victims, ctl, blockIdx.x);
    } else {
        const int64_t b = ((int64_t)blockIdx.x - insert_blocks) * 256 + threadIdx.x;
        if (b < B && slots[b] == -1) c.first_idx[ids[b]] = kNoIndex;
    }
}

inline unsigned blocks_for(int64_t n, int per = 256) { return (unsigned)std::max<int64_t>(1, (n + per - 1) / per); }
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// flagged elements of [0, n) through the functor (see above); sums = scratch for ceil(n/1024) + 1 int64
template <class F>
void compact_flagged(const F& f, int64_t n, int64_t* sums, hipStream_t stream) {
    const int64_t tiles = (n + kScanTile - 1) / kScanTile;
    if (tiles > 0 && tiles <= kFoldTiles) {
        hipLaunchKernelGGL((k_flag_tile_sums<F>), dim3((unsigned)tiles), dim3(256), 0, stream, f, n, sums);
        hipLaunchKernelGGL((k_flag_collect<F, true>), dim3((unsigned)tiles), dim3(256), 0, stream, f, n, sums);
        return;
    }
    if (tiles > 0) hipLaunchKernelGGL((k_flag_tile_sums<F>), dim3((unsigned)tiles), dim3(256), 0, stream, f, n, sums);
    hipLaunchKernelGGL((k_flag_scan_sums<F>), dim3(1), dim3(1024), 0, stream, f, sums, tiles);
    if (tiles > 0) hipLaunchKernelGGL((k_flag_collect<F, false>), dim3((unsigned)tiles), dim3(256), 0, stream, f, n, sums);
}

}  // namespace

struct tns_cache {
    tns_cache_config cfg;
    CacheState st{};
    int32_t max_replace = 0;
    // the update (scores, victims) runs beside the row gather on a stream of the cache's own,
    // forked from and joined back into the caller's stream with these events
    hipStream_t side = nullptr;
    hipEvent_t forked = nullptr, joined = nullptr;
};

namespace {
struct Workspace {
    Ctl* ctl;
    int32_t *slots, *new_ids, *victims;
    int64_t* sums;
    size_t bytes;
};
Workspace carve(const tns_cache* c, int64_t B, void* base) {
    Workspace w{};
    unsigned char* p = static_cast<unsigned char*>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* r = p ? p + off : nullptr; off += align256(bytes); return r; };
    const int64_t cap = c->cfg.capacity;
    w.ctl = reinterpret_cast<Ctl*>(take(sizeof(Ctl)));
    w.slots = reinterpret_cast<int32_t*>(take((size_t)B * 4));
    w.new_ids = reinterpret_cast<int32_t*>(take((size_t)std::max(c->max_replace, 1) * 4));
    w.victims = reinterpret_cast<int32_t*>(take((size_t)std::max(c->max_replace, 1) * 4));
    w.sums = reinterpret_cast<int64_t*>(take((size_t)(std::max(B, cap) / kScanTile + 2) * 8));
    w.bytes = off;
    return w;
}
}  // namespace

extern "C" {

int tns_cache_create(const tns_cache_config* cfg, tns_cache** out) {
    tns::clear_error();
    if (!cfg || !out) return fail(TNS_EINVAL, "null config or output pointer");
    if (cfg->num_ids < 1 || cfg->num_ids > (int64_t)INT32_MAX) return fail(TNS_EINVAL, "num_ids must be in [1, 2^31-1]");
    if (cfg->capacity < 1 || cfg->capacity > (int64_t)INT32_MAX / 2) return fail(TNS_EINVAL, "capacity must be in [1, 2^30]");
    if (cfg->dim < 1 || cfg->dim > (1 << 20)) return fail(TNS_EINVAL, "dim must be in [1, 2^20]");
    if (cfg->policy < 0 || cfg->policy > 2) return fail(TNS_EINVAL, "unknown policy");
    if (!(cfg->lambda > 0.0f) || cfg->lambda > 1.0f) return fail(TNS_EINVAL, "lambda must be in (0, 1]");
    if (cfg->device < 0) return fail(TNS_EINVAL, "negative device ordinal");
    DeviceGuard guard(cfg->device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the cache's device");
    tns_cache* c = new (std::nothrow) tns_cache();
    if (!c) return fail(TNS_ENOMEM, "host allocation failed");
    c->cfg = *cfg;
    c->max_replace = (int32_t)std::floor(cfg->lambda * (float)cfg->capacity);
    const int64_t N = cfg->num_ids, C = cfg->capacity;
    struct Alloc { void** p; size_t bytes; };
    const Alloc allocs[] = {{(void**)&c->st.slot_of, (size_t)N * 4}, {(void**)&c->st.first_idx, (size_t)N * 4},
                            {(void**)&c->st.id_of, (size_t)C * 4},   {(void**)&c->st.score, (size_t)C * 4},
                            {(void**)&c->st.touched, (size_t)C * 4}, {(void**)&c->st.rows, (size_t)C * cfg->dim * 4},
                            {(void**)&c->st.counters, kStripes * 3 * 8},        {(void**)&c->st.ring, 8}};
    for (const Alloc& a : allocs) {
        const hipError_t e = hipMalloc(a.p, a.bytes);
        if (e != hipSuccess) {
            tns_cache_destroy(c);
            return fail_hip(e, "allocating the cache");
        }
    }
    hipError_t es = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (es == hipSuccess) es = hipEventCreateWithFlags(&c->forked, hipEventDisableTiming);
    if (es == hipSuccess) es = hipEventCreateWithFlags(&c->joined, hipEventDisableTiming);
    if (es != hipSuccess) {
        tns_cache_destroy(c);
        return fail_hip(es, "creating the cache's stream and events");
    }
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(N)), dim3(256), 0, nullptr, c->st.slot_of, N, -1);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(N)), dim3(256), 0, nullptr, c->st.first_idx, N, kNoIndex);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(C)), dim3(256), 0, nullptr, c->st.id_of, C, -1);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(C)), dim3(256), 0, nullptr, c->st.score, C, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(C)), dim3(256), 0, nullptr, c->st.touched, C, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(kStripes * 6)), dim3(256), 0, nullptr, reinterpret_cast<int32_t*>(c->st.counters), kStripes * 6, 0);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(256), 0, nullptr, reinterpret_cast<int32_t*>(c->st.ring), 2, 0);
    hipError_t e = hipMemsetAsync(c->st.rows, 0, (size_t)C * cfg->dim * 4, nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) {
        tns_cache_destroy(c);
        return fail_hip(e, "initialising the cache");
    }
    *out = c;
    return TNS_OK;
}

int tns_cache_workspace(const tns_cache* cache, int64_t B, size_t* bytes) {
    tns::clear_error();
    if (!cache || !bytes || B < 0) return fail(TNS_EINVAL, "null cache/pointer or negative B");
    *bytes = carve(cache, B, nullptr).bytes;
    return TNS_OK;
}

int tns_cache_fetch(tns_cache* cache, int64_t B, const int32_t* d_ids, const float* store, float* d_out, uint8_t* d_hit,
                    void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    tns::clear_error();
    if (!cache) return fail(TNS_EINVAL, "null cache");
    if (B < 0) return fail(TNS_EINVAL, "negative B");
    if (B == 0) return TNS_OK;
    if (B > (int64_t)INT32_MAX) return fail(TNS_ESIZE, "more than 2^31-1 ids in one batch");
    if (!d_ids || !store || !d_out) return fail(TNS_EINVAL, "null ids, store or output");
    if (!d_workspace) return fail(TNS_EINVAL, "null workspace");
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255) return fail(TNS_EINVAL, "workspace must be 256-byte aligned");
    const Workspace w = carve(cache, B, d_workspace);
    if (workspace_bytes < w.bytes) return fail(TNS_ESIZE, "workspace smaller than tns_cache_workspace()");
    DeviceGuard guard(cache->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the cache's device");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const CacheState& st = cache->st;
    const int policy = cache->cfg.policy;
    const int32_t dim = cache->cfg.dim;
    const int64_t C = cache->cfg.capacity, N = cache->cfg.num_ids;
    const int32_t maxrep = cache->max_replace;

    // Two chains that only meet at the insertion.  The caller's stream gathers the rows (bound by memory bandwidth;
    // each row's threads look the slot up themselves).  The cache's own stream runs the lookup proper (hit flags,
    // counters, recorded accesses, first occurrence of every missed id) and the update (scores, distinct misses,
    // victims: many short kernels over the score vector).  Both only read the maps and rows; the insertion changes
    // them and waits for both.
    const bool select = maxrep > 0 && policy != TNS_CACHE_FIFO;
    hipStream_t us = cache->side;
    {
        hipError_t ef = hipEventRecord(cache->forked, stream);
        if (ef == hipSuccess) ef = hipStreamWaitEvent(us, cache->forked, 0);
        if (ef != hipSuccess) return fail_hip(ef, "forking the cache update");
    }
    const bool vec4 = dim % 4 == 0 && ((reinterpret_cast<uintptr_t>(store) | reinterpret_cast<uintptr_t>(d_out)) & 15) == 0;
    if (vec4)
        hipLaunchKernelGGL(k_gather<4>, dim3(blocks_for((B * (dim / 4) + kGatherUnroll - 1) / kGatherUnroll)), dim3(256), 0, stream, st.rows, store, dim, B, N, d_ids,
                           st.slot_of, d_out);
    else
        hipLaunchKernelGGL(k_gather<1>, dim3(blocks_for((B * dim + kGatherUnroll - 1) / kGatherUnroll)), dim3(256), 0, stream, st.rows, store, dim, B, N, d_ids,
                           st.slot_of, d_out);

    hipLaunchKernelGGL(k_lookup, dim3(blocks_for((B + kLookupUnroll - 1) / kLookupUnroll)), dim3(256), 0, us, st, policy, N, B, d_ids,
                       w.slots, d_hit, w.ctl);
    // LRU: every score is decremented and the accessed entries are reset; done on the way by the first
    // pass of the victim selection when there is one
    if (policy == TNS_CACHE_LRU && !select)
        hipLaunchKernelGGL(k_lru_scores, dim3(blocks_for(C)), dim3(256), 0, us, st.score, st.touched, C);
    if (maxrep > 0) {
        const NewIds nf{st.first_idx, d_ids, w.slots, maxrep, w.new_ids, w.ctl};
        // few workgroups for the histograms: they are added to one global one with atomics
        const unsigned hb = (unsigned)std::min<int64_t>(blocks_for(C), 256);
        const int64_t tiles_b = (B + kScanTile - 1) / kScanTile;
        const bool lru = policy == TNS_CACHE_LRU;
        if (select && tiles_b <= kFoldTiles) {
            // distinct missed ids: tile sums, then the collect kernel, which shares its launch with pass 0 of the selection
            hipLaunchKernelGGL((k_flag_tile_sums<NewIds>), dim3((unsigned)tiles_b), dim3(256), 0, us, nf, B, w.sums);
            if (lru)
                hipLaunchKernelGGL((k_newids_collect_hist0<true>), dim3((unsigned)tiles_b + hb), dim3(256), 0, us, nf, B, w.sums, tiles_b,
                                   st.score, st.touched, C, w.ctl, (int64_t)hb);
            else
                hipLaunchKernelGGL((k_newids_collect_hist0<false>), dim3((unsigned)tiles_b + hb), dim3(256), 0, us, nf, B, w.sums, tiles_b,
                                   st.score, st.touched, C, w.ctl, (int64_t)hb);
        } else {
            compact_flagged(nf, B, w.sums, us);
            if (select) {
                if (lru) hipLaunchKernelGGL(k_select_hist<true>, dim3(hb), dim3(256), 0, us, st.score, st.touched, C, 0, w.ctl);
                else hipLaunchKernelGGL(k_select_hist<false>, dim3(hb), dim3(256), 0, us, st.score, st.touched, C, 0, w.ctl);
            }
        }
        if (policy == TNS_CACHE_FIFO) {
            hipLaunchKernelGGL(k_fifo_victims, dim3(blocks_for(maxrep)), dim3(256), 0, us, C, maxrep, st.ring, w.ctl, w.victims);
            hipLaunchKernelGGL(k_fifo_advance, dim3(1), dim3(1), 0, us, C, st.ring, w.ctl);
        } else {
            // passes 1-3: each picks the digit of the pass before it in its prologue
            for (int pass = 1; pass < 4; ++pass)
                hipLaunchKernelGGL(k_select_hist<false>, dim3(hb), dim3(256), 0, us, st.score, st.touched, C, pass, w.ctl);
            // victims in slot order; the tile-sum kernel picks the last digit first
            const Victims vf{st.score, w.ctl, w.victims};
            const int64_t tiles_c = (C + kScanTile - 1) / kScanTile;
            hipLaunchKernelGGL(k_victims_tile_sums, dim3((unsigned)std::max<int64_t>(tiles_c, 1)), dim3(256), 0, us, vf, w.ctl, C, w.sums);
            if (tiles_c <= kFoldTiles) {
                hipLaunchKernelGGL((k_flag_collect<Victims, true>), dim3((unsigned)std::max<int64_t>(tiles_c, 1)), dim3(256), 0, us, vf, C, w.sums);
            } else {
                hipLaunchKernelGGL((k_flag_scan_sums<Victims>), dim3(1), dim3(1024), 0, us, vf, w.sums, tiles_c);
                hipLaunchKernelGGL((k_flag_collect<Victims, false>), dim3((unsigned)tiles_c), dim3(256), 0, us, vf, C, w.sums);
            }
        }
    }
    {
        hipError_t ej = hipEventRecord(cache->joined, us);
        if (ej == hipSuccess) ej = hipStreamWaitEvent(stream, cache->joined, 0);
        if (ej != hipSuccess) return fail_hip(ej, "joining the cache update");
    }
    // the insertion, and the clearing of this batch's first-occurrence marks for the next one, in one launch
    {
        const int64_t ib = maxrep > 0 ? (int64_t)blocks_for(maxrep, 4) : 0;
        hipLaunchKernelGGL(k_insert_clear, dim3((unsigned)(ib + blocks_for(B))), dim3(256), 0, stream, st, policy, dim, store, w.new_ids,
                           w.victims, w.ctl, ib, B, d_ids, w.slots);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e, "launching the cache kernels");
    return TNS_OK;
}

int tns_cache_stats(tns_cache* cache, void* hip_stream, int64_t* hits, int64_t* misses, int64_t* replaced) {
    tns::clear_error();
    if (!cache) return fail(TNS_EINVAL, "null cache");
    DeviceGuard guard(cache->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the cache's device");
    unsigned long long all[kStripes * 3], h[3] = {0, 0, 0};
    hipError_t e = hipMemcpyAsync(all, cache->st.counters, sizeof(all), hipMemcpyDeviceToHost, static_cast<hipStream_t>(hip_stream));
    if (e == hipSuccess) e = hipStreamSynchronize(static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "reading the cache counters");
    for (int i = 0; i < kStripes; ++i)
        for (int k = 0; k < 3; ++k) h[k] += all[i * 3 + k];
    if (hits) *hits = (int64_t)h[0];
    if (misses) *misses = (int64_t)h[1];
    if (replaced) *replaced = (int64_t)h[2];
    return TNS_OK;
}

int tns_cache_save(tns_cache* cache, void* hip_stream, int32_t* h_id_of, int32_t* h_score, float* h_rows, int64_t* h_ring) {
    tns::clear_error();
    if (!cache || !h_id_of || !h_score || !h_rows || !h_ring) return fail(TNS_EINVAL, "null cache or buffer");
    DeviceGuard guard(cache->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the cache's device");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int64_t C = cache->cfg.capacity;
    hipError_t e = hipMemcpyAsync(h_id_of, cache->st.id_of, (size_t)C * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipMemcpyAsync(h_score, cache->st.score, (size_t)C * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipMemcpyAsync(h_rows, cache->st.rows, (size_t)C * cache->cfg.dim * 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipMemcpyAsync(h_ring, cache->st.ring, 8, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail_hip(e, "saving the cache");
    return TNS_OK;
}

int tns_cache_restore(tns_cache* cache, void* hip_stream, const int32_t* h_id_of, const int32_t* h_score, const float* h_rows,
                      int64_t ring) {
    tns::clear_error();
    if (!cache || !h_id_of || !h_score || !h_rows) return fail(TNS_EINVAL, "null cache or buffer");
    const int64_t C = cache->cfg.capacity, N = cache->cfg.num_ids;
    if (ring < 0 || ring >= C) return fail(TNS_EINVAL, "ring position outside [0, capacity)");
    for (int64_t s = 0; s < C; ++s)
        if (h_id_of[s] < -1 || h_id_of[s] >= N) return fail(TNS_ERANGE, "saved id outside [-1, num_ids)");
    DeviceGuard guard(cache->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the cache's device");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMemcpyAsync(cache->st.id_of, h_id_of, (size_t)C * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(cache->st.score, h_score, (size_t)C * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(cache->st.rows, h_rows, (size_t)C * cache->cfg.dim * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemcpyAsync(cache->st.ring, &ring, 8, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return fail_hip(e, "restoring the cache");
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(N)), dim3(256), 0, s, cache->st.slot_of, N, -1);
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(C)), dim3(256), 0, s, cache->st.touched, C, 0);
    hipLaunchKernelGGL(k_rebuild_map, dim3(blocks_for(C)), dim3(256), 0, s, cache->st.id_of, C, N, cache->st.slot_of);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail_hip(e, "restoring the cache");
    return TNS_OK;
}

int tns_cache_destroy(tns_cache* cache) {
    tns::clear_error();
    if (!cache) return TNS_OK;
    {
        DeviceGuard guard(cache->cfg.device);
        void* ptrs[] = {cache->st.slot_of, cache->st.first_idx, cache->st.id_of, cache->st.score,
                        cache->st.touched, cache->st.rows,      cache->st.counters, cache->st.ring};
        for (void* p : ptrs)
            if (p) (void)hipFree(p);
        if (cache->forked) (void)hipEventDestroy(cache->forked);
        if (cache->joined) (void)hipEventDestroy(cache->joined);
        if (cache->side) (void)hipStreamDestroy(cache->side);
    }
    delete cache;
    return TNS_OK;
}

}  // extern "C"
