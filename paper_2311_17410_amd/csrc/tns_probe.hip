// Streaming kernels of known traffic: what this GPU's memory system sustains for plain reads, writes
// and copies.  The bench times them next to the sampling step (the practical ceiling of the box) and
// counter runs use them to calibrate the byte counters (a launch that moves exactly `bytes`).
#include <hip/hip_runtime.h>

#include "../../include/tns.h"
#include "tns_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kUnroll = 8;     // 16-byte vectors per thread: 32 KiB per workgroup, all loads issued before the first store

template <bool NT>
__device__ __forceinline__ u32x4 ld(const u32x4* p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT>
__device__ __forceinline__ void st(u32x4 v, u32x4* p) {
    if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}

// MODE 0: copy, 1: read only (the sum is stored only if it equals a value the data never has), 2: write only
template <int MODE, bool NT>
__global__ void __launch_bounds__(kThreads) tns_probe_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                             int64_t n_vec, unsigned sentinel) {
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
    u32x4 v[kUnroll];
    if (MODE != 2) {
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            const int64_t k = base + (int64_t)i * kThreads;
            v[i] = u32x4{0u, 0u, 0u, 0u};
            if (k < n_vec) v[i] = ld<NT>(src + k);
        }
    } else {
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) v[i] = u32x4{sentinel, (unsigned)i, threadIdx.x, blockIdx.x};
    }
    if (MODE == 1) {
        unsigned acc = 0;
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
        if (acc == sentinel && dst) dst[base % n_vec] = v[0];
    } else {
#pragma unroll
        for (int i = 0; i < kUnroll; ++i) {
            const int64_t k = base + (int64_t)i * kThreads;
            if (k < n_vec) st<NT>(v[i], dst + k);
        }
    }
}

// Reads rv vectors of src and writes wv vectors of dst, the shorter stream spread evenly over the longer one:
// workgroup g of G takes the g-th share of each stream (two divisions per workgroup, none per vector), loads its
// share of src, then stores its share of dst.
template <bool NT>
__global__ void __launch_bounds__(kThreads) tns_probe_mix_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, int64_t rv,
                                                                 int64_t wv, unsigned sentinel) {
    const int64_t g = blockIdx.x, G = gridDim.x;
    const int64_t r_lo = g * rv / G, r_hi = (g + 1) * rv / G;        // g, G < 2^31 and rv, wv < 2^31: the products fit
    const int64_t w_lo = g * wv / G, w_hi = (g + 1) * wv / G;
    u32x4 v[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
        const int64_t k = r_lo + (int64_t)i * kThreads + threadIdx.x;
        v[i] = u32x4{sentinel, (unsigned)i, threadIdx.x, blockIdx.x};
        if (k < r_hi) v[i] = ld<NT>(src + k);
    }
    unsigned acc = 0;
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) acc ^= v[i].x;
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
        const int64_t k = w_lo + (int64_t)i * kThreads + threadIdx.x;
        if (k < w_hi) {
            v[i].w ^= acc;          // every store depends on every load of the thread
            st<NT>(v[i], dst + k);
        }
    }
}

}  // namespace

extern "C" int tns_hbm_probe_mix(int32_t nontemporal, void* d_dst, size_t write_bytes, const void* d_src, size_t read_bytes,
                                 void* hip_stream) {
    tns::clear_error();
    if (!d_dst || !d_src) return tns::fail(TNS_EINVAL, "null buffer");
    if (read_bytes % 16 || write_bytes % 16 || read_bytes < 16 || write_bytes < 16 ||
        (reinterpret_cast<uintptr_t>(d_dst) | reinterpret_cast<uintptr_t>(d_src)) % 16)
        return tns::fail(TNS_EINVAL, "sizes and addresses must be positive multiples of 16 bytes");
    const int64_t rv = (int64_t)(read_bytes / 16), wv = (int64_t)(write_bytes / 16), n = rv > wv ? rv : wv;
    const int64_t grid = (n + kThreads * kUnroll - 1) / (kThreads * kUnroll);      // a workgroup's share of either stream fits its registers
    if (n >= (int64_t(1) << 31)) return tns::fail(TNS_ESIZE, "at most 32 GiB per stream: split the buffers");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (nontemporal)
        hipLaunchKernelGGL((tns_probe_mix_kernel<true>), dim3((unsigned)grid), dim3(kThreads), 0, s, static_cast<u32x4*>(d_dst),
                           static_cast<const u32x4*>(d_src), rv, wv, 0x9e3779b9u);
    else
        hipLaunchKernelGGL((tns_probe_mix_kernel<false>), dim3((unsigned)grid), dim3(kThreads), 0, s, static_cast<u32x4*>(d_dst),
                           static_cast<const u32x4*>(d_src), rv, wv, 0x9e3779b9u);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return tns::fail_hip(e, "launching a probe kernel");
    return TNS_OK;
}

extern "C" int tns_hbm_probe(int32_t mode, int32_t nontemporal, void* d_dst, const void* d_src, size_t bytes, void* hip_stream) {
    tns::clear_error();
    if (mode < 0 || mode > 2) return tns::fail(TNS_EINVAL, "mode must be 0 (copy), 1 (read) or 2 (write)");
    if ((mode != 1 && !d_dst) || (mode != 2 && !d_src)) return tns::fail(TNS_EINVAL, "null buffer");
    if (bytes % 16 || (reinterpret_cast<uintptr_t>(d_dst) | reinterpret_cast<uintptr_t>(d_src)) % 16)
        return tns::fail(TNS_EINVAL, "size and addresses must be multiples of 16 bytes");
    const int64_t n_vec = (int64_t)(bytes / 16);
    if (n_vec == 0) return TNS_OK;
    const int64_t grid = (n_vec + kThreads * kUnroll - 1) / (kThreads * kUnroll);
    if (grid > 0x7fffffffLL) return tns::fail(TNS_ESIZE, "more than 2^31 workgroups: split the buffer");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    u32x4* dst = static_cast<u32x4*>(d_dst);
    const u32x4* src = static_cast<const u32x4*>(d_src);
    const unsigned sentinel = 0x9e3779b9u;
#define TNS_PROBE(M, N) hipLaunchKernelGGL((tns_probe_kernel<M, N>), dim3((unsigned)grid), dim3(kThreads), 0, s, dst, src, n_vec, sentinel)
    if (mode == 0) { if (nontemporal) TNS_PROBE(0, true); else TNS_PROBE(0, false); }
    else if (mode == 1) { if (nontemporal) TNS_PROBE(1, true); else TNS_PROBE(1, false); }
    else { if (nontemporal) TNS_PROBE(2, true); else TNS_PROBE(2, false); }
#undef TNS_PROBE
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return tns::fail_hip(e, "launching a probe kernel");
    return TNS_OK;
}
