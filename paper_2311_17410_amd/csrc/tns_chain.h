// Single-pass chained scan over workgroup tiles (decoupled look-back): the piece shared by the sampling
// kernels (padding removal fused into sampling) and the device-side store builder (segment numbering and
// pool offsets in one launch each).  Included by .hip files only; everything has internal linkage.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace tns {
namespace {

constexpr int kChainWave = 64;

// ---- single-pass chained scan over workgroup tiles (padding removal fused into sampling) ----
//
// Workspace layout: word 0 = tile ticket, word 1 = error flag, then one 64-bit status per tile:
// bits 62-63 = state (0 not ready, 1 tile total, 2 inclusive prefix), bits 0-61 = value.
// Tiles take their index from the ticket, so a tile only ever waits for tiles that have
// already started; the wait is bounded and sets the error flag if the bound is ever hit.
constexpr uint64_t kStTotal = 1ull << 62, kStPrefix = 2ull << 62, kStMask = 3ull << 62;
constexpr int kSpinLimit = 1 << 22;

struct ScanWorkspace {
    uint32_t ticket;
    uint32_t error;
    uint32_t pad[62];
    uint64_t status[1];   // [number of tiles]
};

__device__ __forceinline__ int64_t shfl64(int64_t v, int src) {
    const int lo = __shfl((int)(uint32_t)(v & 0xffffffffll), src, kChainWave);
    const int hi = __shfl((int)(v >> 32), src, kChainWave);
    return ((int64_t)hi << 32) | (uint32_t)lo;
}

// Sum of the totals of all tiles before `tile` (called by one whole wave).
__device__ __forceinline__ int64_t lookback_exclusive(ScanWorkspace* ws, uint32_t* err_flag, int64_t tile, int lane) {
    int64_t excl = 0;
    int64_t idx = tile - 1;
    int spins = 0;
    bool fresh = true;              // new window: every lane reads its tile's state
    uint64_t st = 0;
    while (true) {
        const int64_t t = idx - lane;
        // a lane re-reads only while its tile is not ready
        if (fresh || (st & kStMask) == 0) {
            st = kStPrefix;         // before the first tile: prefix 0
            if (t >= 0) st = __hip_atomic_load(&ws->status[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        fresh = false;
        const uint64_t state = st & kStMask;
        const uint64_t is_prefix = __ballot(state == kStPrefix);
        const uint64_t not_ready = __ballot(state == 0);
        const int first = is_prefix ? __builtin_ctzll(is_prefix) : kChainWave;             // nearest tile with a full prefix
        const uint64_t needed = first >= kChainWave - 1 ? ~0ull : ((2ull << first) - 1);    // lanes 0..first
        if (not_ready & needed) {
            if (++spins > kSpinLimit) {
                // reported before this tile publishes anything, so that whoever builds on its (wrong)
                // prefix can see the flag
                if (lane == 0) atomicExch(err_flag, 1u);
                __threadfence();
                return excl;
            }
            __builtin_amdgcn_s_sleep(16);      // ~0.4 us between polls: late tiles are late by microseconds
            continue;
        }
        int64_t v = (lane <= first) ? (int64_t)(st & ~kStMask) : 0;
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kChainWave);
        excl += v;
        if (first < kChainWave) return excl;
        idx -= kChainWave;
        fresh = true;
    }
}

}  // namespace
}  // namespace tns
