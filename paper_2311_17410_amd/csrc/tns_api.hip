// C ABI of the library (include/tns.h): plan lifetime, ingestion, commit, run, statistics.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/tns.h"
#include "tns_ingest.h"
#include "tns_internal.h"
#include "tns_kernels.h"
#include "tns_pstore.h"
#include "tns_store.h"
#include "tns_test_hooks.h"

namespace tns {
thread_local std::string g_err;

int fail(int code, const std::string& msg) {
    g_err = msg;
    return code;
}

int fail_hip(hipError_t e, const char* what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? TNS_ENOMEM : TNS_EHIP;
}
void clear_error() { g_err.clear(); }
}  // namespace tns

using tns::fail;
using tns::fail_hip;
using tns::g_err;
using tns::DeviceGuard;

namespace {

template <class T>
struct DeviceArray {
    T* ptr = nullptr;
    int64_t cap = 0;   // elements allocated
    int64_t used = 0;  // elements valid on the device
    bool on_host = false;   // page-locked host memory the device reads directly, instead of device memory

    hipError_t alloc(T** p, int64_t n) const {
        const size_t bytes = (size_t)n * sizeof(T);
        return on_host ? hipHostMalloc(reinterpret_cast<void**>(p), bytes, hipHostMallocMapped | hipHostMallocPortable)
                       : hipMalloc(reinterpret_cast<void**>(p), bytes);
    }
    void release() {
        if (ptr) (void)(on_host ? hipHostFree(ptr) : hipFree(ptr));
        ptr = nullptr;
        cap = used = 0;
    }
};

// State of a plan whose store is built on the device (TNS_FLAG_DEVICE_INGEST): no host copy.
struct DeviceStore {
    DeviceArray<tns::NodeAux> aux;
    DeviceArray<unsigned char> ws;              // scratch of the ingestion kernels, grown on demand
    tns::IngestStatus* d_status = nullptr;
    tns::IngestStatus* h_status = nullptr;      // page-locked landing place of the status read-backs, followed by a
                                                // sequence word; the device can write both (mapped, coherent)
    tns::IngestStatus* h_status_dev = nullptr;  // the same memory as the device addresses it
    unsigned long long seq = 0;                 // batches planned by the short pipeline
    std::vector<tns::InstanceTotals> totals;   // per instance: edges, blocks, slots, running edge id, deleted
};

}  // namespace

struct tns_plan {
    tns_config cfg;
    std::unique_ptr<tns::Store> store;          // host builder (null for a device-built store)
    std::unique_ptr<DeviceStore> dev;           // device builder (null otherwise)
    std::unique_ptr<tns::PrefixStore> pstore;   // host builder of the prefix layout (TNS_FLAG_PREFIX_LAYOUT; null otherwise)
    DeviceArray<tns::StoreLine> d_lines;        // prefix layout: node lines and edge lines in one array
    DeviceArray<tns::NodeLine> d_nodes;
    DeviceArray<tns::BlockRec> d_dir;
    DeviceArray<uint32_t> d_dir_cum;            // per directory record: the node's edges in older blocks
    DeviceArray<tns::EdgeLine> d_edges;
    bool committed = false;
    bool deleted_edges = false;                 // some edge has been deleted: blocks with deleted edges are scanned candidate by candidate
};

namespace {

// Ensures room for `need` elements.  Growing reallocates; the host copy is complete, so the
// whole array is simply marked for upload instead of being copied device to device.
template <class T, class P>
int ensure_capacity(DeviceArray<T>& d, int64_t need, P& host, const char* what) {
    if (need <= d.cap) return TNS_OK;
    int64_t cap = need + need / 4 + 1024;
    T* p = nullptr;
    hipError_t e = d.alloc(&p, cap);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        cap = need;
        e = d.alloc(&p, cap);
    }
    if (e != hipSuccess) return fail_hip(e, what);
    d.release();
    d.ptr = p;
    d.cap = cap;
    d.used = 0;
    host.mark_all();
    return TNS_OK;
}

template <class T, class P>
int upload_dirty(DeviceArray<T>& d, const P& host, hipStream_t stream, const char* what) {
    hipError_t first = hipSuccess;
    host.for_each_dirty([&](int64_t start, int64_t count, const T* src) {
        if (first != hipSuccess) return;
        first = hipMemcpyAsync(d.ptr + start, src, (size_t)count * sizeof(T), hipMemcpyDefault, stream);
    });
    if (first != hipSuccess) return fail_hip(first, what);
    d.used = host.size();
    return TNS_OK;
}

// Device-built store: room for `need` elements, keeping the first `used` ones (device-to-device copy).
template <class T>
int grow_device(DeviceArray<T>& d, int64_t need, hipStream_t stream, const char* what) {
    if (need <= d.cap) return TNS_OK;
    int64_t cap = need + need / 2 + 1024;
    T* p = nullptr;
    hipError_t e = d.alloc(&p, cap);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        cap = need;
        e = d.alloc(&p, cap);
    }
    if (e != hipSuccess) return fail_hip(e, what);
    if (d.ptr && d.used > 0) {
        e = hipMemcpyAsync(p, d.ptr, (size_t)d.used * sizeof(T), hipMemcpyDeviceToDevice, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) {
            (void)(d.on_host ? hipHostFree(p) : hipFree(p));
            return fail_hip(e, what);
        }
    }
    const int64_t used = d.used;
    d.release();
    d.ptr = p;
    d.cap = cap;
    d.used = used;
    return TNS_OK;
}

// Device-built store: first use allocates the (empty) node table, the builder state and the status record.
int ensure_device_store(tns_plan* plan, hipStream_t stream) {
    DeviceStore& ds = *plan->dev;
    if (ds.d_status) return TNS_OK;
    const int64_t total_nodes = std::max<int64_t>((int64_t)plan->cfg.num_instances * plan->cfg.num_nodes, 1);
    int rc;
    if ((rc = grow_device(plan->d_nodes, total_nodes, stream, "allocating node table"))) return rc;
    if ((rc = grow_device(ds.aux, total_nodes, stream, "allocating the builder state"))) return rc;
    if ((rc = grow_device(plan->d_dir, 1024, stream, "allocating the block directory"))) return rc;
    if ((rc = grow_device(plan->d_dir_cum, 1024, stream, "allocating the block directory"))) return rc;
    if ((rc = grow_device(plan->d_edges, 1024, stream, "allocating edge data"))) return rc;
    hipError_t e = hipMemsetAsync(plan->d_nodes.ptr, 0, (size_t)total_nodes * sizeof(tns::NodeLine), stream);
    if (e == hipSuccess) e = hipMemsetAsync(ds.aux.ptr, 0, (size_t)total_nodes * sizeof(tns::NodeAux), stream);
    tns::IngestStatus* st = nullptr;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&st), sizeof(tns::IngestStatus));
    if (e == hipSuccess && !ds.h_status) {
        e = hipHostMalloc(reinterpret_cast<void**>(&ds.h_status), 2 * sizeof(tns::IngestStatus), hipHostMallocMapped | hipHostMallocCoherent);
        if (e == hipSuccess) {
            std::memset(ds.h_status, 0, 2 * sizeof(tns::IngestStatus));
            e = hipHostGetDevicePointer(reinterpret_cast<void**>(&ds.h_status_dev), ds.h_status, 0);
        }
    }
    if (e == hipSuccess) e = hipMemsetAsync(st, 0, sizeof(tns::IngestStatus), stream);
    if (e == hipSuccess) e = tns::ingest_status_reset(st, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        if (st) (void)hipFree(st);
        return fail_hip(e, "initialising the device store");
    }
    plan->d_nodes.used = total_nodes;
    ds.aux.used = total_nodes;
    ds.d_status = st;
    plan->committed = true;
    return TNS_OK;
}

// Waits for the stream and returns the builder's status record.  A set `internal` word (a pool found too small by
// an apply kernel, or a chained scan whose bounded wait ran out) is an error of the library, reported here by
// whichever call reads the record next; the record is then made clean again.
int read_status(tns_plan* plan, hipStream_t stream, tns::IngestStatus& out, const char* what) {
    DeviceStore& ds = *plan->dev;
    hipError_t e = hipMemcpyAsync(ds.h_status, ds.d_status, sizeof(out), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail_hip(e, what);
    out = *ds.h_status;
    if (out.internal) {
        const uint32_t bits = out.internal;
        e = hipMemsetAsync(ds.d_status, 0, sizeof(out), stream);
        if (e == hipSuccess) e = tns::ingest_status_reset(ds.d_status, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail_hip(e, what);
        return fail(TNS_EHIP, bits & 8u ? "a chained scan of the ingestion kernels timed out (internal error); the batch was not applied"
                                        : "ingestion kernels of an earlier batch ran out of pool space (internal error)");
    }
    return TNS_OK;
}

// Copies a host array into a temporary device buffer (deletion requests).
template <class T>
struct DeviceTemp {
    T* ptr = nullptr;
    ~DeviceTemp() { if (ptr) (void)hipFree(ptr); }
    hipError_t upload(const T* host, int64_t n, hipStream_t stream) {
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&ptr), (size_t)std::max<int64_t>(n, 1) * sizeof(T));
        if (e == hipSuccess && n > 0) e = hipMemcpyAsync(ptr, host, (size_t)n * sizeof(T), hipMemcpyHostToDevice, stream);
        return e;
    }
};

}  // namespace

// ---- entry point for callers that cannot allocate: the workspace is a static device array ----
//
// Each GPU the library runs on holds its own copy of the array for the life of the process.  Host code never
// uses the array's name as an address: the per-device address comes from hipGetSymbolAddress, once.
constexpr int64_t kStaticMaxQueries = int64_t(1) << 24;
constexpr size_t kStaticScratchBytes = (size_t(2) << 20) + 512;   // = tns_workspace() for 2^24 queries
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Address of `scratch` on device `dev` (which must be the current device).
static int static_scratch_of(int dev, void** out) {
    if (dev < 0 || dev >= kMaxDevices) return fail(TNS_EINVAL, "device ordinal beyond the static scratch table");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail_hip(e == hipSuccess ? hipErrorInvalidSymbol : e, "locating the static scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TNS_OK;
}

extern "C" {

int tns_plan_create(const tns_config* cfg, tns_plan** out) {
    g_err.clear();
    if (!cfg || !out) return fail(TNS_EINVAL, "null config or output pointer");
    if (cfg->num_nodes < 0 || cfg->num_nodes > (int64_t)INT32_MAX) return fail(TNS_EINVAL, "num_nodes must be in [0, 2^31-1]");
    if (cfg->num_instances < 1) return fail(TNS_EINVAL, "num_instances must be >= 1");
    if (cfg->fanout < 1 || cfg->fanout > TNS_MAX_FANOUT) return fail(TNS_EINVAL, "fanout must be in [1, 64]");
    if (cfg->policy != TNS_POLICY_RECENT && cfg->policy != TNS_POLICY_UNIFORM) return fail(TNS_EINVAL, "unknown policy");
    if (cfg->block_threshold < 1) return fail(TNS_EINVAL, "block_threshold (tau) must be >= 1");
    if (cfg->sizing < 0 || cfg->sizing > 2) return fail(TNS_EINVAL, "unknown sizing method");
    if (cfg->inclusive_end != 0 && cfg->inclusive_end != 1) return fail(TNS_EINVAL, "inclusive_end must be 0 or 1");
    if (cfg->device < 0) return fail(TNS_EINVAL, "negative device ordinal");
    constexpr int32_t kKnownFlags = TNS_FLAG_NO_XCD_REMAP | TNS_FLAG_NO_NODE_SLAB | TNS_FLAG_EDGES_ON_HOST |
                                    TNS_FLAG_ALL_ON_HOST | TNS_FLAG_DEVICE_INGEST | TNS_FLAG_WIDE_POSITIONS | TNS_TEST_FLAG_LOST_TILE |
                                    TNS_FLAG_PREFIX_LAYOUT;
    if (cfg->flags & ~kKnownFlags) return fail(TNS_EINVAL, "unknown bit in flags");
    if ((cfg->flags & TNS_FLAG_EDGES_ON_HOST) && (cfg->flags & TNS_FLAG_ALL_ON_HOST))
        return fail(TNS_EINVAL, "TNS_FLAG_EDGES_ON_HOST and TNS_FLAG_ALL_ON_HOST exclude each other");
    if ((cfg->flags & TNS_FLAG_DEVICE_INGEST) &&
        (cfg->flags & (TNS_FLAG_EDGES_ON_HOST | TNS_FLAG_ALL_ON_HOST | TNS_FLAG_NO_NODE_SLAB)))
        return fail(TNS_EINVAL, "TNS_FLAG_DEVICE_INGEST cannot be combined with host placement or TNS_FLAG_NO_NODE_SLAB");
    if ((cfg->flags & TNS_FLAG_PREFIX_LAYOUT) &&
        (cfg->flags & (TNS_FLAG_EDGES_ON_HOST | TNS_FLAG_ALL_ON_HOST | TNS_FLAG_DEVICE_INGEST | TNS_FLAG_NO_NODE_SLAB)))
        return fail(TNS_EINVAL, "TNS_FLAG_PREFIX_LAYOUT cannot be combined with host placement, TNS_FLAG_DEVICE_INGEST or TNS_FLAG_NO_NODE_SLAB");
    try {
        std::unique_ptr<tns_plan> p(new tns_plan());
        p->cfg = *cfg;
        p->d_edges.on_host = (cfg->flags & (TNS_FLAG_EDGES_ON_HOST | TNS_FLAG_ALL_ON_HOST)) != 0;
        p->d_nodes.on_host = p->d_dir.on_host = p->d_dir_cum.on_host = (cfg->flags & TNS_FLAG_ALL_ON_HOST) != 0;
        if (cfg->flags & TNS_FLAG_DEVICE_INGEST) {
            p->dev.reset(new DeviceStore());
            p->dev->totals.resize((size_t)cfg->num_instances);
        } else {
            tns::StoreConfig sc;
            sc.num_nodes = cfg->num_nodes;
            sc.num_instances = cfg->num_instances;
            sc.tau = cfg->block_threshold;
            sc.sizing = cfg->sizing;
            sc.node_slab = !(cfg->flags & TNS_FLAG_NO_NODE_SLAB);
            if (cfg->flags & TNS_FLAG_PREFIX_LAYOUT) p->pstore.reset(new tns::PrefixStore(sc));
            else p->store.reset(new tns::Store(sc));
        }
        *out = p.release();
    } catch (const std::bad_alloc&) {
        return fail(TNS_ENOMEM, "host allocation failed");
    }
    return TNS_OK;
}

int tns_set_sampler(tns_plan* plan, int32_t fanout, int32_t policy, int32_t inclusive_end, uint64_t seed) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (fanout < 1 || fanout > TNS_MAX_FANOUT) return fail(TNS_EINVAL, "fanout must be in [1, 64]");
    if (policy != TNS_POLICY_RECENT && policy != TNS_POLICY_UNIFORM) return fail(TNS_EINVAL, "unknown policy");
    if (inclusive_end != 0 && inclusive_end != 1) return fail(TNS_EINVAL, "inclusive_end must be 0 or 1");
    plan->cfg.fanout = fanout;
    plan->cfg.policy = policy;
    plan->cfg.inclusive_end = inclusive_end;
    plan->cfg.seed = seed;
    return TNS_OK;
}

int tns_add_edges(tns_plan* plan, int32_t instance, const int32_t* src, const int32_t* dst, const float* ts,
                  const int32_t* eid, int64_t m) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (plan->dev) return fail(TNS_ESTATE, "this plan's store is built on the device: use tns_add_edges_device");
    try {
        std::string err;
        const int rc = plan->pstore ? plan->pstore->add_edges(instance, src, dst, ts, eid, m, err)
                                    : plan->store->add_edges(instance, src, dst, ts, eid, m, err);
        if (rc != TNS_OK) g_err = err;
        return rc;
    } catch (const std::bad_alloc&) {
        return fail(TNS_ENOMEM, "host allocation failed during ingestion");
    }
}

int tns_add_edges_device(tns_plan* plan, int32_t instance, const int32_t* d_src, const int32_t* d_dst, const float* d_ts,
                         const int32_t* d_eid, int64_t m, void* hip_stream) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (!plan->dev) return fail(TNS_ESTATE, "tns_add_edges_device needs a plan created with TNS_FLAG_DEVICE_INGEST");
    if (instance < 0 || instance >= plan->cfg.num_instances) return fail(TNS_ERANGE, "instance out of range");
    if (m < 0 || (m > 0 && (!d_src || !d_dst || !d_ts))) return fail(TNS_EINVAL, "null array or negative batch size");
    if (m == 0) return TNS_OK;
    if (m > tns::kMaxDeviceBatch) return fail(TNS_ESIZE, "batch larger than 2^24-1 edges: split it");
    DeviceStore& ds = *plan->dev;
    tns::InstanceTotals& tot = ds.totals[(size_t)instance];
    if (!d_eid && tot.next_eid + m > (int64_t)INT32_MAX) return fail(TNS_ESIZE, "running edge id would exceed 2^31-1");

    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int rc;
    if ((rc = ensure_device_store(plan, stream))) return rc;
    const int64_t ws_need = (int64_t)tns::ingest_workspace_bytes(m);
    if (ws_need > ds.ws.cap) {
        ds.ws.used = 0;   // scratch: nothing to keep
        if ((rc = grow_device(ds.ws, ws_need, stream, "allocating the ingestion workspace"))) return rc;
    }

    tns::IngestArgs a{};
    a.src = d_src;
    a.dst = d_dst;
    a.ts = d_ts;
    a.eid = d_eid;
    a.m = m;
    a.eid_base = tot.next_eid;
    a.nodes = plan->d_nodes.ptr;
    a.aux = ds.aux.ptr;
    a.dir = plan->d_dir.ptr;
    a.dir_cum = plan->d_dir_cum.ptr;
    a.lines = reinterpret_cast<uint32_t*>(plan->d_edges.ptr);
    a.node_base = (int64_t)instance * plan->cfg.num_nodes;
    a.num_nodes = plan->cfg.num_nodes;
    a.used_lines = plan->d_edges.used;
    a.cap_lines = plan->d_edges.cap;
    a.used_dir = plan->d_dir.used;
    a.cap_dir = plan->d_dir.cap;
    a.tau = plan->cfg.block_threshold;
    a.sizing = plan->cfg.sizing;
    a.workspace = ds.ws.ptr;
    a.status = ds.d_status;

    // Batches of stream size take the short planning pipeline, which assumes time order; if the status says the
    // batch was not in time order (nothing has been changed yet) the general pipeline plans it again.
    bool fast = tns::ingest_fast_ok(m, plan->cfg.num_nodes);
    if (fast && ds.h_status_dev) {
        a.host_status = ds.h_status_dev;
        a.host_seq = reinterpret_cast<unsigned long long*>(ds.h_status_dev + 1);
        a.seq = ++ds.seq;
    }
    hipError_t e = fast ? tns::ingest_plan_fast(a, stream) : tns::ingest_plan(a, stream);
    if (e != hipSuccess) return fail_hip(e, "launching the ingestion planning kernels");
    tns::IngestStatus st;
    bool polled = false;
    if (a.host_status) {
        // The plan's last workgroup writes the record into host memory and then the batch's sequence number: picked
        // up here by polling, which is some 20 us sooner than a copy and a wait for the stream.  The wait is bounded;
        // past the bound (or with an internal error in the record) the ordinary read-back takes over.
        const volatile unsigned long long* seq_word = reinterpret_cast<const volatile unsigned long long*>(ds.h_status + 1);
        const auto t0 = std::chrono::steady_clock::now();
        int spins = 0;
        while (*seq_word != a.seq) {
            if ((++spins & 1023) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(2)) break;
        }
        if (*seq_word == a.seq) {
            std::atomic_thread_fence(std::memory_order_acquire);
            st = *ds.h_status;
            polled = st.internal == 0;
        }
    }
    if (!polled && (rc = read_status(plan, stream, st, "waiting for the ingestion plan"))) return rc;
    if (fast && st.unsorted && st.err_word == ~0ull) {
        fast = false;
        if ((e = tns::ingest_plan(a, stream)) != hipSuccess) return fail_hip(e, "launching the ingestion planning kernels");
        if ((rc = read_status(plan, stream, st, "waiting for the ingestion plan"))) return rc;
    }
    if (st.err_word != ~0ull || st.num_segments < 1 || st.num_segments > m || st.total_lines < 0 || st.total_dir < 0) {
        // no apply phase will run: the record is cleaned for the next batch here
        if ((e = tns::ingest_status_reset(ds.d_status, stream)) != hipSuccess) return fail_hip(e, "resetting the ingestion status");
    }
    if (st.err_word != ~0ull) {
        const int code = -(int)(st.err_word & 0xffu);
        const int64_t pos = (int64_t)(st.err_word >> 8);
        switch (code) {
            case TNS_ERANGE: return fail(code, "source node id outside [0, num_nodes) at batch position " + std::to_string(pos));
            case TNS_EINVAL: return fail(code, "negative edge id at batch position " + std::to_string(pos));
            case TNS_EORDER:
                if (pos < m) return fail(code, "NaN timestamp at batch position " + std::to_string(pos));
                return fail(code, "node " + std::to_string(pos - m) + " would receive an edge older than its newest stored edge");
            default: return fail(TNS_EHIP, "unexpected status from the ingestion kernels");
        }
    }
    if (st.num_segments < 1 || st.num_segments > m || st.total_lines < 0 || st.total_dir < 0)
        return fail(TNS_EHIP, "inconsistent plan from the ingestion kernels");
    const int64_t lines_after = plan->d_edges.used + st.total_lines;
    const int64_t dir_after = plan->d_dir.used + st.total_dir;
    if (lines_after > tns::kMaxEdgeOffset / tns::kSlotsPerLine) return fail(TNS_ESIZE, "edge array would exceed 2^39 slots");
    if (dir_after / tns::kDirAlign > (int64_t)UINT32_MAX) return fail(TNS_ESIZE, "block directory would exceed its index range");
    if ((rc = grow_device(plan->d_edges, lines_after, stream, "growing edge data"))) return rc;
    if ((rc = grow_device(plan->d_dir, dir_after, stream, "growing the block directory"))) return rc;
    if ((rc = grow_device(plan->d_dir_cum, dir_after, stream, "growing the block directory"))) return rc;
    a.dir = plan->d_dir.ptr;
    a.dir_cum = plan->d_dir_cum.ptr;
    a.lines = reinterpret_cast<uint32_t*>(plan->d_edges.ptr);
    a.cap_lines = plan->d_edges.cap;
    a.cap_dir = std::min(plan->d_dir.cap, plan->d_dir_cum.cap);

    // The apply kernels are not waited for: the store changes in stream order, and an internal error they might
    // raise (a pool too small, which the sizes above rule out) is reported by the next read of the status record.
    e = tns::ingest_apply(a, st.num_segments, fast, stream);
    if (e != hipSuccess) return fail_hip(e, "launching the ingestion kernels");
    plan->d_edges.used = lines_after;
    plan->d_dir.used = dir_after;
    plan->d_dir_cum.used = dir_after;
    tot.edges += m;
    tot.next_eid += m;
    tot.blocks += (int64_t)st.new_blocks;
    tot.slots += (int64_t)st.new_slots;
    return TNS_OK;
}

int tns_delete_edges(tns_plan* plan, int32_t instance, const int32_t* src, const int32_t* eid, int64_t m,
                     int64_t* num_deleted) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (m < 0 || (m > 0 && (!src || !eid))) return fail(TNS_EINVAL, "null array or negative count");
    if (instance < 0 || instance >= plan->cfg.num_instances) return fail(TNS_ERANGE, "instance out of range");
    for (int64_t i = 0; i < m; ++i) {
        if (src[i] < 0 || src[i] >= plan->cfg.num_nodes) return fail(TNS_ERANGE, "node id outside [0, num_nodes)");
        if (eid[i] < 0) return fail(TNS_EINVAL, "negative edge id");
    }
    if (plan->dev) {
        // device-built store: the requests are copied over and applied by a kernel (default stream)
        DeviceGuard guard(plan->cfg.device);
        if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
        int rc;
        if ((rc = ensure_device_store(plan, nullptr))) return rc;
        DeviceTemp<int32_t> d_src, d_eid;
        hipError_t e = hipDeviceSynchronize();          // ingestion's last kernels may still be running on the caller's stream
        if (e == hipSuccess) e = d_src.upload(src, m, nullptr);
        if (e == hipSuccess) e = d_eid.upload(eid, m, nullptr);
        if (e == hipSuccess)
            e = tns::ingest_delete_edges(plan->d_nodes.ptr, plan->d_dir.ptr, reinterpret_cast<uint32_t*>(plan->d_edges.ptr),
                                         (int64_t)instance * plan->cfg.num_nodes, d_src.ptr, d_eid.ptr, m, plan->dev->d_status,
                                         nullptr);
        if (e != hipSuccess) return fail_hip(e, "deleting edges on the device");
        tns::IngestStatus st;
        if ((rc = read_status(plan, nullptr, st, "waiting for the deletion kernel"))) return rc;
        plan->dev->totals[(size_t)instance].deleted += (int64_t)st.counter;
        if (st.counter) plan->deleted_edges = true;
        if (num_deleted) *num_deleted = (int64_t)st.counter;
        return TNS_OK;
    }
    int64_t hit = 0;
    if (plan->pstore) {
        for (int64_t i = 0; i < m; ++i) hit += plan->pstore->delete_edge(instance, src[i], eid[i]);
    } else {
        tns::Store& s = *plan->store;
        for (int64_t i = 0; i < m; ++i) hit += s.delete_edge(instance, src[i], eid[i]);
    }
    if (hit) plan->deleted_edges = true;
    if (num_deleted) *num_deleted = hit;
    return TNS_OK;
}

int tns_delete_nodes(tns_plan* plan, int32_t instance, const int32_t* nodes, int64_t m, int32_t deleted) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (m < 0 || (m > 0 && !nodes)) return fail(TNS_EINVAL, "null array or negative count");
    if (instance < 0 || instance >= plan->cfg.num_instances) return fail(TNS_ERANGE, "instance out of range");
    for (int64_t i = 0; i < m; ++i)
        if (nodes[i] < 0 || nodes[i] >= plan->cfg.num_nodes) return fail(TNS_ERANGE, "node id outside [0, num_nodes)");
    if (plan->dev) {
        DeviceGuard guard(plan->cfg.device);
        if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
        int rc;
        if ((rc = ensure_device_store(plan, nullptr))) return rc;
        DeviceTemp<int32_t> d_ids;
        hipError_t e = hipDeviceSynchronize();          // ingestion's last kernels may still be running on the caller's stream
        if (e == hipSuccess) e = d_ids.upload(nodes, m, nullptr);
        if (e == hipSuccess)
            e = tns::ingest_delete_nodes(plan->d_nodes.ptr, (int64_t)instance * plan->cfg.num_nodes, d_ids.ptr, m, deleted, nullptr);
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess) return fail_hip(e, "marking nodes on the device");
        return TNS_OK;
    }
    if (plan->pstore) {
        for (int64_t i = 0; i < m; ++i) plan->pstore->set_node_deleted(instance, nodes[i], deleted != 0);
        return TNS_OK;
    }
    tns::Store& s = *plan->store;
    for (int64_t i = 0; i < m; ++i) s.set_node_deleted(instance, nodes[i], deleted != 0);
    return TNS_OK;
}

int tns_commit(tns_plan* plan, void* hip_stream) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    {
        // set-up: find this device's copy of the static scratch array (used by tns_run_static)
        void* unused = nullptr;
        const int rc0 = static_scratch_of(plan->cfg.device, &unused);
        if (rc0) return rc0;
    }
    if (plan->dev) return ensure_device_store(plan, stream);   // nothing to upload: the store lives on the device
    if (plan->pstore) {
        tns::PrefixStore& s = *plan->pstore;
        int rc;
        if ((rc = ensure_capacity(plan->d_lines, std::max<int64_t>(s.lines.size(), 1), s.lines, "allocating the store"))) return rc;
        if ((rc = ensure_capacity(plan->d_dir, std::max<int64_t>(s.dir.size(), 1), s.dir, "allocating the block directory"))) return rc;
        if ((rc = ensure_capacity(plan->d_dir_cum, std::max<int64_t>(s.dir_cum.size(), 1), s.dir_cum, "allocating the block directory"))) return rc;
        if ((rc = upload_dirty(plan->d_lines, s.lines, stream, "uploading the store"))) return rc;
        if ((rc = upload_dirty(plan->d_dir, s.dir, stream, "uploading the block directory"))) return rc;
        if ((rc = upload_dirty(plan->d_dir_cum, s.dir_cum, stream, "uploading the block directory"))) return rc;
        const hipError_t e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail_hip(e, "waiting for the upload");
        s.lines.clear_dirty();
        s.dir.clear_dirty();
        s.dir_cum.clear_dirty();
        plan->committed = true;
        return TNS_OK;
    }
    tns::Store& s = *plan->store;
    int rc;
    // at least one element each, so that the kernels always get valid base pointers
    if ((rc = ensure_capacity(plan->d_nodes, std::max<int64_t>(s.nodes.size(), 1), s.nodes, "allocating node table"))) return rc;
    if ((rc = ensure_capacity(plan->d_dir, std::max<int64_t>(s.dir.size(), 1), s.dir, "allocating the block directory"))) return rc;
    if ((rc = ensure_capacity(plan->d_dir_cum, std::max<int64_t>(s.dir_cum.size(), 1), s.dir_cum, "allocating the block directory"))) return rc;
    if ((rc = ensure_capacity(plan->d_edges, std::max<int64_t>(s.lines.size(), 1), s.lines, "allocating edge data"))) return rc;
    if ((rc = upload_dirty(plan->d_nodes, s.nodes, stream, "uploading node table"))) return rc;
    if ((rc = upload_dirty(plan->d_dir, s.dir, stream, "uploading the block directory"))) return rc;
    if ((rc = upload_dirty(plan->d_dir_cum, s.dir_cum, stream, "uploading the block directory"))) return rc;
    if ((rc = upload_dirty(plan->d_edges, s.lines, stream, "uploading edge data"))) return rc;
    const hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail_hip(e, "waiting for the upload");
    s.nodes.clear_dirty();
    s.dir.clear_dirty();
    s.dir_cum.clear_dirty();
    s.lines.clear_dirty();
    plan->committed = true;
    return TNS_OK;
}

int tns_workspace(const tns_plan* plan, int64_t Q, size_t* bytes) {
    g_err.clear();
    if (!plan || !bytes || Q < 0) return fail(TNS_EINVAL, "null plan/pointer or negative Q");
    *bytes = tns::compact_workspace_bytes(Q);
    return TNS_OK;
}

static int check_compact_args(int64_t Q, const void* rowptr, const void* a, const void* b, const void* c,
                              const void* ws, size_t ws_bytes) {
    const int n_cmp = (a != nullptr) + (b != nullptr) + (c != nullptr);
    if (!rowptr) return fail(TNS_EINVAL, "null d_rowptr");
    if (Q > 0 && n_cmp != 3) return fail(TNS_EINVAL, "pass all four compaction outputs or none");
    if (!ws) return fail(TNS_EINVAL, "compaction needs a workspace");
    if (ws_bytes < tns::compact_workspace_bytes(Q)) return fail(TNS_ESIZE, "workspace smaller than tns_workspace()");
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(TNS_EINVAL, "workspace must be 256-byte aligned");
    return TNS_OK;
}

static int fill_sample_args(tns_plan* plan, int64_t Q, const int32_t* d_targets, const float* d_t_start,
                            const float* d_t_end, const int64_t* d_inst_rowptr, int64_t query_id_base,
                            tns::SampleArgs& a) {
    if (Q < 0) return fail(TNS_EINVAL, "negative Q");
    if (!plan->committed) return fail(TNS_ESTATE, "tns_run before the first tns_commit");
    if (Q > 0 && (!d_targets || !d_t_end)) return fail(TNS_EINVAL, "null query pointer");
    if (plan->cfg.num_instances > 1 && !d_inst_rowptr) return fail(TNS_EINVAL, "d_inst_rowptr is required with several instances");
    if (Q > (int64_t(1) << 36)) return fail(TNS_ESIZE, "more than 2^36 queries in one call: split the batch");
    a = tns::SampleArgs{};
    a.delta = INFINITY;
    a.nodes = plan->d_nodes.ptr;
    a.dir = plan->d_dir.ptr;
    a.dir_cum = plan->d_dir_cum.ptr;
    a.edges = reinterpret_cast<const uint32_t*>(plan->d_edges.ptr);
    if (plan->pstore) {
        a.nodes = nullptr;
        a.edges = reinterpret_cast<const uint32_t*>(plan->d_lines.ptr);
        a.prefix_layout = 1;
    }
    a.targets = d_targets;
    a.t_start = d_t_start;
    a.t_end = d_t_end;
    a.inst_rowptr = plan->cfg.num_instances == 1 ? nullptr : d_inst_rowptr;
    a.Q = Q;
    a.num_nodes = plan->cfg.num_nodes;
    a.num_dir = plan->d_dir.used;
    a.qid_base = query_id_base;
    a.seed = plan->cfg.seed;
    a.num_instances = plan->cfg.num_instances;
    a.fanout = plan->cfg.fanout;
    a.policy = plan->cfg.policy;
    a.inclusive_end = plan->cfg.inclusive_end;
    a.xcd_remap = (plan->cfg.flags & TNS_FLAG_NO_XCD_REMAP) ? 0 : 1;
    a.first_ticket = (plan->cfg.flags & TNS_TEST_FLAG_LOST_TILE) ? 1 : 0;
    const int64_t edge_lines = plan->pstore ? plan->d_lines.used : plan->d_edges.used;
    a.wide_offsets = (edge_lines * 32 >= (int64_t(1) << 31) || (plan->cfg.flags & TNS_FLAG_WIDE_POSITIONS)) ? 1 : 0;   // word indices beyond int32
    return TNS_OK;
}

static int run_compact(tns_plan* plan, int64_t Q, const int32_t* nbr, const int32_t* eid, const float* ts,
                       const int32_t* count, int64_t* rowptr, int32_t* cn, int32_t* ce, float* ct, void* ws,
                       hipStream_t stream) {
    tns::CompactArgs c{};
    c.nbr = nbr;
    c.eid = eid;
    c.ts = ts;
    c.count = count;
    c.rowptr = rowptr;
    c.cmp_nbr = cn;
    c.cmp_eid = ce;
    c.cmp_ts = ct;
    c.Q = Q;
    c.fanout = plan->cfg.fanout;
    c.workspace = ws;
    const hipError_t e = tns::launch_compact(c, stream);
    if (e != hipSuccess) return fail_hip(e, "launching the compaction kernels");
    return TNS_OK;
}

static int run_impl(tns_plan* plan, int64_t Q, const int32_t* d_targets, const float* d_t_start, const float* d_t_end,
                    const int64_t* d_inst_rowptr, int64_t query_id_base, int32_t* d_out_nbr, int32_t* d_out_eid,
                    float* d_out_ts, int32_t* d_out_count, int64_t* d_rowptr, int32_t* d_cmp_nbr, int32_t* d_cmp_eid,
                    float* d_cmp_ts, void* d_workspace, size_t workspace_bytes, bool static_scratch, void* hip_stream) {
    tns::SampleArgs a;
    int rc = fill_sample_args(plan, Q, d_targets, d_t_start, d_t_end, d_inst_rowptr, query_id_base, a);
    if (rc) return rc;
    // compaction is requested by d_rowptr; with Q == 0 the dense arrays are empty and may be null
    const bool want_cmp = d_rowptr != nullptr;
    // dense-only run: all four padded outputs null, the padded rows are never written
    const bool dense_only = want_cmp && !d_out_nbr && !d_out_eid && !d_out_ts && !d_out_count;
    if (Q > 0 && !dense_only && (!d_out_nbr || !d_out_eid || !d_out_ts || !d_out_count)) return fail(TNS_EINVAL, "null output pointer");
    if (!want_cmp && (d_cmp_nbr || d_cmp_eid || d_cmp_ts)) return fail(TNS_EINVAL, "pass all four compaction outputs or none");

    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    if (static_scratch && want_cmp) {
        if (Q > kStaticMaxQueries || tns::compact_workspace_bytes(Q) > kStaticScratchBytes)
            return fail(TNS_ESIZE, "tns_run_static serves at most 2^24 queries per call");
        if ((rc = static_scratch_of(plan->cfg.device, &d_workspace))) return rc;
        workspace_bytes = kStaticScratchBytes;
    }
    if (want_cmp && (rc = check_compact_args(Q, d_rowptr, d_cmp_nbr, d_cmp_eid, d_cmp_ts, d_workspace, workspace_bytes))) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    a.out_nbr = d_out_nbr;
    a.out_eid = d_out_eid;
    a.out_ts = d_out_ts;
    a.out_count = d_out_count;
    // One pass: sampling with the padding removal fused in.  With the edge data in host memory the reads
    // cross the host link and what counts is how many of them are in flight: the plain sampling kernel
    // keeps more waves resident than the fused one, so the two steps are run one after the other
    // (C3, edge data on the host: 29.0 + 0.9 ms against 46.9 ms fused).  A store with deleted edges also takes the
    // two steps: a block with deleted edges is scanned candidate by candidate, a hub query under the uniform policy
    // can then take long, and in the fused kernel every later tile's bounded wait would be running meanwhile.
    const bool fuse = want_cmp && !plan->d_edges.on_host && !plan->deleted_edges;
    if (dense_only && !fuse)
        return fail(TNS_EINVAL, "this plan removes the padding in a step of its own (edge data on the host, or deleted edges) and needs the padded outputs");
    if (fuse) {
        a.scan_ws = d_workspace;
        a.rowptr = d_rowptr;
        a.cmp_nbr = d_cmp_nbr;
        a.cmp_eid = d_cmp_eid;
        a.cmp_ts = d_cmp_ts;
    }
    const hipError_t e = tns::launch_sample(a, stream);
    if (e != hipSuccess) return fail_hip(e, "launching the sampling kernel");
    if (want_cmp && !fuse)
        return run_compact(plan, Q, d_out_nbr, d_out_eid, d_out_ts, d_out_count, d_rowptr, d_cmp_nbr, d_cmp_eid,
                           d_cmp_ts, d_workspace, stream);
    return TNS_OK;
}

int tns_run(tns_plan* plan, int64_t Q, const int32_t* d_targets, const float* d_t_start, const float* d_t_end,
            const int64_t* d_inst_rowptr, int64_t query_id_base, int32_t* d_out_nbr, int32_t* d_out_eid,
            float* d_out_ts, int32_t* d_out_count, int64_t* d_rowptr, int32_t* d_cmp_nbr, int32_t* d_cmp_eid,
            float* d_cmp_ts, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    return run_impl(plan, Q, d_targets, d_t_start, d_t_end, d_inst_rowptr, query_id_base, d_out_nbr, d_out_eid, d_out_ts,
                    d_out_count, d_rowptr, d_cmp_nbr, d_cmp_eid, d_cmp_ts, d_workspace, workspace_bytes, false, hip_stream);
}

int tns_run_static(tns_plan* plan, int64_t Q, const int32_t* d_targets, const float* d_t_start, const float* d_t_end,
                   const int64_t* d_inst_rowptr, int64_t query_id_base, int32_t* d_out_nbr, int32_t* d_out_eid,
                   float* d_out_ts, int32_t* d_out_count, int64_t* d_rowptr, int32_t* d_cmp_nbr, int32_t* d_cmp_eid,
                   float* d_cmp_ts, void* hip_stream) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (!d_rowptr) return fail(TNS_EINVAL, "tns_run_static is the variant with padding removal: d_rowptr is required");
    return run_impl(plan, Q, d_targets, d_t_start, d_t_end, d_inst_rowptr, query_id_base, d_out_nbr, d_out_eid, d_out_ts,
                    d_out_count, d_rowptr, d_cmp_nbr, d_cmp_eid, d_cmp_ts, nullptr, 0, true, hip_stream);
}

int tns_run_status(tns_plan* plan, const void* d_workspace, void* hip_stream, int32_t* timed_out) {
    g_err.clear();
    if (!plan || !timed_out) return fail(TNS_EINVAL, "null plan or output pointer");
    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    void* ws = const_cast<void*>(d_workspace);
    int rc;
    if (!ws && (rc = static_scratch_of(plan->cfg.device, &ws))) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t word = 0;
    hipError_t e = hipMemcpyAsync(&word, static_cast<const uint32_t*>(ws) + 1, sizeof(word), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail_hip(e, "reading the status word");
    *timed_out = word != 0;
    return TNS_OK;
}

namespace {
constexpr int kMaxHops = 8;
// caps[h] = most queries hop h can have; false if the sizes leave the supported range
bool khop_caps(int32_t num_hops, const int32_t* fanouts, int64_t Q, int64_t* caps) {
    int64_t cap = Q;
    for (int h = 0; h < num_hops; ++h) {
        if (fanouts[h] < 1 || fanouts[h] > TNS_MAX_FANOUT) return false;
        caps[h] = cap;
        if (cap > (int64_t(1) << 36) / fanouts[h]) return false;
        cap *= fanouts[h];
    }
    return true;
}
constexpr size_t kStatusBytes = 256;
size_t khop_header_bytes(int32_t num_hops, int32_t num_instances) {
    // per hop: the dense total (next hop's query count) and the instance offsets of the next hop
    const size_t per_hop = (size_t)(num_instances + 2) * sizeof(int64_t);
    return ((size_t)num_hops * per_hop + 255) & ~size_t(255);
}
}  // namespace

int tns_workspace_khop(const tns_plan* plan, int32_t num_hops, const int32_t* fanouts, int64_t Q, size_t* bytes) {
    g_err.clear();
    if (!plan || !fanouts || !bytes || Q < 0) return fail(TNS_EINVAL, "null pointer or negative Q");
    if (num_hops < 1 || num_hops > kMaxHops) return fail(TNS_EINVAL, "num_hops must be in [1, 8]");
    int64_t caps[kMaxHops];
    if (!khop_caps(num_hops, fanouts, Q, caps)) return fail(TNS_ESIZE, "fan-out out of range or more than 2^36 queries in a hop");
    // one chained-scan region per hop, so that a single launch can clear them all before the first hop
    size_t scan = 0;
    for (int h = 0; h < num_hops; ++h) scan += tns::compact_workspace_bytes(caps[h]);
    *bytes = kStatusBytes + scan + khop_header_bytes(num_hops, plan->cfg.num_instances);
    return TNS_OK;
}

int tns_run_khop(tns_plan* plan, int32_t num_hops, const int32_t* fanouts, float delta, int64_t Q,
                 const int32_t* d_targets, const float* d_t_start, const float* d_t_end, const int64_t* d_inst_rowptr,
                 int64_t query_id_base, const tns_hop_buffers* hops, void* d_workspace, size_t workspace_bytes,
                 void* hip_stream) {
    g_err.clear();
    if (!plan || !fanouts || !hops) return fail(TNS_EINVAL, "null plan, fanouts or hops");
    if (num_hops < 1 || num_hops > kMaxHops) return fail(TNS_EINVAL, "num_hops must be in [1, 8]");
    if (std::isnan(delta) || delta < 0) return fail(TNS_EINVAL, "delta must be >= 0 (or +infinity)");
    int64_t caps[kMaxHops];
    if (Q < 0 || !khop_caps(num_hops, fanouts, Q, caps)) return fail(TNS_ESIZE, "fan-out out of range or more than 2^36 queries in a hop");
    size_t need = 0;
    int rc = tns_workspace_khop(plan, num_hops, fanouts, Q, &need);
    if (rc) return rc;
    if (!d_workspace) return fail(TNS_EINVAL, "null workspace");
    if (workspace_bytes < need) return fail(TNS_ESIZE, "workspace smaller than tns_workspace_khop()");
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255) return fail(TNS_EINVAL, "workspace must be 256-byte aligned");
    for (int h = 0; h < num_hops; ++h) {
        const tns_hop_buffers& b = hops[h];
        // the four padded outputs of a hop may be null together: only its dense result is written then
        const bool no_padded = !b.nbr && !b.eid && !b.ts && !b.count;
        if (!b.rowptr || (caps[h] > 0 && (!b.cmp_nbr || !b.cmp_eid || !b.cmp_ts || (!no_padded && (!b.nbr || !b.eid || !b.ts || !b.count)))))
            return fail(TNS_EINVAL, "null buffer in hops[]");
    }
    tns::SampleArgs a;
    if ((rc = fill_sample_args(plan, Q, d_targets, d_t_start, d_t_end, d_inst_rowptr, query_id_base, a))) return rc;

    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int32_t I = plan->cfg.num_instances;
    // workspace: the status word (second 32-bit word, as in tns_run's workspace), one chained-scan region per
    // hop, then per hop the dense total and the instance offsets of the next hop
    unsigned char* scan_ws = static_cast<unsigned char*>(d_workspace) + kStatusBytes;
    size_t scan = 0;
    for (int h = 0; h < num_hops; ++h) scan += tns::compact_workspace_bytes(caps[h]);
    int64_t* header = reinterpret_cast<int64_t*>(scan_ws + scan);
    {
        const hipError_t e = tns::launch_scan_clear(d_workspace, kStatusBytes + scan, stream);
        if (e != hipSuccess) return fail_hip(e, "clearing the chained-scan workspace");
    }
    a.err_flag = static_cast<uint32_t*>(d_workspace) + 1;   // every hop reports a time-out in the same word

    for (int h = 0; h < num_hops; ++h) {
        const tns_hop_buffers& b = hops[h];
        int64_t* total = header + (size_t)h * (I + 2);          // dense total of hop h = query count of hop h+1
        int64_t* next_inst = total + 1;                         // [I + 1]
        a.fanout = fanouts[h];
        a.Q = caps[h];
        a.out_nbr = b.nbr;
        a.out_eid = b.eid;
        a.out_ts = b.ts;
        a.out_count = b.count;
        a.total_out = total;
        a.scan_ws = scan_ws;                                    // sampling with the padding removal fused in
        a.scan_ready = Q > 0 ? 1 : 0;                           // cleared above, together with the other hops' regions
        scan_ws += tns::compact_workspace_bytes(caps[h]);
        a.rowptr = b.rowptr;
        a.cmp_nbr = b.cmp_nbr;
        a.cmp_eid = b.cmp_eid;
        a.cmp_ts = b.cmp_ts;
        hipError_t e = tns::launch_sample(a, stream);
        if (e != hipSuccess) return fail_hip(e, "launching the sampling kernel of a hop");
        if (h + 1 == num_hops) break;
        // queries of the next hop: the dense entries of this one
        if (a.inst_rowptr) {
            e = tns::launch_hop_inst_rowptr(a.inst_rowptr, b.rowptr, I, next_inst, stream);
            if (e != hipSuccess) return fail_hip(e, "launching the instance-offset kernel");
            a.inst_rowptr = next_inst;
        }
        a.targets = b.cmp_nbr;
        a.t_end = b.cmp_ts;
        a.t_start = nullptr;
        a.delta = delta;
        a.Q_dev = total;
        a.qid_base += caps[h];
    }
    return TNS_OK;
}

int tns_compact(tns_plan* plan, int64_t Q, const int32_t* d_out_nbr, const int32_t* d_out_eid, const float* d_out_ts,
                const int32_t* d_out_count, int64_t* d_rowptr, int32_t* d_cmp_nbr, int32_t* d_cmp_eid,
                float* d_cmp_ts, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (Q < 0) return fail(TNS_EINVAL, "negative Q");
    if (Q > 0 && (!d_out_nbr || !d_out_eid || !d_out_ts || !d_out_count)) return fail(TNS_EINVAL, "null input pointer");
    if (Q > (int64_t(1) << 36)) return fail(TNS_ESIZE, "more than 2^36 queries in one call: split the batch");
    int rc = check_compact_args(Q, d_rowptr, d_cmp_nbr, d_cmp_eid, d_cmp_ts, d_workspace, workspace_bytes);
    if (rc) return rc;
    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    return run_compact(plan, Q, d_out_nbr, d_out_eid, d_out_ts, d_out_count, d_rowptr, d_cmp_nbr, d_cmp_eid, d_cmp_ts,
                       d_workspace, static_cast<hipStream_t>(hip_stream));
}

int tns_traffic_model(tns_plan* plan, int64_t Q, const int32_t* d_targets, const float* d_t_start,
                      const float* d_t_end, const int64_t* d_inst_rowptr, int64_t query_id_base,
                      uint64_t* d_counters, void* hip_stream) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (!d_counters) return fail(TNS_EINVAL, "null d_counters");
    tns::SampleArgs a;
    const int rc = fill_sample_args(plan, Q, d_targets, d_t_start, d_t_end, d_inst_rowptr, query_id_base, a);
    if (rc) return rc;
    DeviceGuard guard(plan->cfg.device);
    if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
    a.counters = reinterpret_cast<unsigned long long*>(d_counters);
    const hipError_t e = tns::launch_sample(a, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail_hip(e, "launching the counting kernel");
    return TNS_OK;
}

int tns_stats(const tns_plan* plan, int32_t instance, tns_stats_t* out) {
    g_err.clear();
    if (!plan || !out) return fail(TNS_EINVAL, "null plan or output");
    const int32_t I = plan->cfg.num_instances;
    if (instance < -1 || instance >= I) return fail(TNS_ERANGE, "instance out of range");
    const int32_t i0 = instance < 0 ? 0 : instance, i1 = instance < 0 ? I : instance + 1;
    tns_stats_t r{};
    if (plan->dev) {
        // device-built store: totals are kept on the host, the longest list is reduced on the device
        const DeviceStore& ds = *plan->dev;
        for (int32_t i = i0; i < i1; ++i) {
            const tns::InstanceTotals& t = ds.totals[(size_t)i];
            r.num_blocks += t.blocks;
            r.num_edges += t.edges;
            r.wasted_slots += t.slots - t.edges;
        }
        const int64_t n_nodes = (int64_t)(i1 - i0) * plan->cfg.num_nodes;
        if (ds.d_status && n_nodes > 0) {
            DeviceGuard guard(plan->cfg.device);
            if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
            hipError_t e = hipDeviceSynchronize();      // ingestion's last kernels may still be running on the caller's stream
            if (e == hipSuccess)
                e = tns::ingest_max_list_len(plan->d_nodes.ptr, (int64_t)i0 * plan->cfg.num_nodes, n_nodes, ds.d_status, nullptr);
            tns::IngestStatus st{};
            if (e == hipSuccess) e = hipMemcpy(&st, ds.d_status, sizeof(st), hipMemcpyDeviceToHost);
            if (e != hipSuccess) return fail_hip(e, "reducing the list lengths");
            r.max_list_len = (int64_t)st.counter;
        }
        r.edge_data_bytes = plan->d_edges.used * (int64_t)sizeof(tns::EdgeLine);
        r.avg_list_len = n_nodes ? (double)r.num_blocks / (double)n_nodes : 0.0;
        r.metadata_bytes = n_nodes * (int64_t)sizeof(tns::NodeLine) + plan->d_dir.used * (int64_t)(sizeof(tns::BlockRec) + sizeof(uint32_t));
        *out = r;
        return TNS_OK;
    }
    if (plan->pstore) {
        const tns::PrefixStore& s = *plan->pstore;
        for (int32_t i = i0; i < i1; ++i) {
            const tns::InstanceTotals& t = s.totals(i);
            r.num_blocks += t.blocks;
            r.num_edges += t.edges;
            r.wasted_slots += t.slots - t.edges;
            for (int64_t v = 0; v < s.config().num_nodes; ++v) r.max_list_len = std::max<int64_t>(r.max_list_len, s.num_blocks(s.node_index(i, v)));
        }
        const int64_t n_nodes = (int64_t)(i1 - i0) * s.config().num_nodes;
        r.avg_list_len = n_nodes ? (double)r.num_blocks / (double)n_nodes : 0.0;
        // of a node's line 96 bytes are edge slots and 32 the node entry; extension and block lines are shared
        // by all instances and counted in full
        r.edge_data_bytes = (s.lines.size() - s.total_nodes()) * (int64_t)sizeof(tns::StoreLine) + n_nodes * (int64_t)(tns::kInlineSlots * sizeof(tns::Edge));
        r.metadata_bytes = n_nodes * (int64_t)sizeof(tns::PrefixNodeHdr) + s.dir.size() * (int64_t)(sizeof(tns::BlockRec) + sizeof(uint32_t));
        *out = r;
        return TNS_OK;
    }
    const tns::Store& s = *plan->store;
    for (int32_t i = i0; i < i1; ++i) {
        const tns::InstanceTotals& t = s.totals(i);
        r.num_blocks += t.blocks;
        r.num_edges += t.edges;
        r.wasted_slots += t.slots - t.edges;

        for (int64_t v = 0; v < s.config().num_nodes; ++v) {
            const int64_t nb = s.nodes[s.node_index(i, v)].nblocks;
            if (nb > r.max_list_len) r.max_list_len = nb;
        }
    }
    // edge lines are shared by all instances and counted in full (block slots + line padding + unused line ends)
    r.edge_data_bytes = s.lines.size() * (int64_t)sizeof(tns::EdgeLine);
    const int64_t n_nodes = (int64_t)(i1 - i0) * s.config().num_nodes;
    r.avg_list_len = n_nodes ? (double)r.num_blocks / (double)n_nodes : 0.0;
    // node lines of the instance(s) plus the directory pool (shared by all instances, counted in full)
    r.metadata_bytes = n_nodes * (int64_t)sizeof(tns::NodeLine) + s.dir.size() * (int64_t)(sizeof(tns::BlockRec) + sizeof(uint32_t));
    *out = r;
    return TNS_OK;
}

int64_t tns_node_blocks(const tns_plan* plan, int32_t instance, int32_t node, int64_t max_blocks, int32_t* cap,
                        int32_t* size, float* t_min, float* t_max) {
    g_err.clear();
    if (!plan) return fail(TNS_EINVAL, "null plan");
    if (instance < 0 || instance >= plan->cfg.num_instances || node < 0 || node >= plan->cfg.num_nodes)
        return fail(TNS_ERANGE, "instance or node out of range");
    if (plan->dev) {
        // device-built store: copy the node's entry, its builder state and, for a long list, its directory run
        if (!plan->dev->d_status) return 0;     // nothing stored yet
        DeviceGuard guard(plan->cfg.device);
        if (guard.error() != hipSuccess) return fail_hip(guard.error(), "selecting the plan's device");
        const int64_t nidx = (int64_t)instance * plan->cfg.num_nodes + node;
        tns::NodeLine nd;
        tns::NodeAux ax;
        hipError_t e = hipDeviceSynchronize();          // ingestion's last kernels may still be running on the caller's stream
        if (e == hipSuccess) e = hipMemcpy(&nd, plan->d_nodes.ptr + nidx, sizeof(nd), hipMemcpyDeviceToHost);
        if (e == hipSuccess) e = hipMemcpy(&ax, plan->dev->aux.ptr + nidx, sizeof(ax), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return fail_hip(e, "reading a node entry");
        const int64_t n = nd.nblocks;
        std::vector<tns::BlockRec> recs((size_t)n);
        if (n > tns::kInlineBlocks) {
            e = hipMemcpy(recs.data(), plan->d_dir.ptr + (int64_t)nd.dir_line * tns::kDirAlign, (size_t)n * sizeof(tns::BlockRec),
                          hipMemcpyDeviceToHost);
            if (e != hipSuccess) return fail_hip(e, "reading a directory run");
        } else {
            for (int64_t i = 0; i < n; ++i) recs[(size_t)i] = nd.rec[n - 1 - i];
        }
        for (int64_t i = 0; i < n && i < max_blocks; ++i) {
            const tns::BlockRec& r = recs[(size_t)i];
            if (cap) cap[i] = i == n - 1 ? ax.tail_cap : tns::rec_size(r);
            if (size) size[i] = tns::rec_size(r);
            if (t_min) t_min[i] = r.t_min;
            if (t_max) t_max[i] = r.t_max;
        }
        return n;
    }
    if (plan->pstore) {
        const tns::PrefixStore& s = *plan->pstore;
        const int64_t nidx = s.node_index(instance, node);
        const int64_t n = s.num_blocks(nidx);
        for (int64_t i = 0; i < n && i < max_blocks; ++i)
            s.block_info(nidx, (int32_t)i, cap ? cap + i : nullptr, size ? size + i : nullptr, t_min ? t_min + i : nullptr,
                         t_max ? t_max + i : nullptr);
        return n;
    }
    const tns::Store& s = *plan->store;
    const int64_t nidx = s.node_index(instance, node);
    const int64_t n = s.nodes[nidx].nblocks;
    for (int64_t i = 0; i < n && i < max_blocks; ++i) {
        const tns::BlockRec& r = s.block_of(nidx, (int32_t)i);
        if (cap) cap[i] = s.block_cap(nidx, (int32_t)i);
        if (size) size[i] = tns::rec_size(r);
        if (t_min) t_min[i] = r.t_min;
        if (t_max) t_max[i] = r.t_max;
    }
    return n;
}

int tns_destroy(tns_plan* plan) {
    g_err.clear();
    if (!plan) return TNS_OK;
    if (plan->d_nodes.ptr || plan->d_dir.ptr || plan->d_edges.ptr || plan->d_lines.ptr) {
        DeviceGuard guard(plan->cfg.device);
        plan->d_lines.release();
        plan->d_nodes.release();
        plan->d_dir.release();
        plan->d_dir_cum.release();
        plan->d_edges.release();
        if (plan->dev) {
            plan->dev->aux.release();
            plan->dev->ws.release();
            if (plan->dev->d_status) (void)hipFree(plan->dev->d_status);
            if (plan->dev->h_status) (void)hipHostFree(plan->dev->h_status);
        }
    }
    delete plan;
    return TNS_OK;
}

const char* tns_strerror(int status) {
    switch (status) {
        case TNS_OK: return "ok";
        case TNS_EINVAL: return "invalid argument";
        case TNS_EORDER: return "edges out of chronological order (or NaN timestamp)";
        case TNS_ERANGE: return "node id or instance out of range";
        case TNS_ENOMEM: return "out of memory";
        case TNS_EHIP: return "HIP runtime error";
        case TNS_ESTATE: return "store not committed";
        case TNS_ESIZE: return "size beyond a limit or workspace too small";
        default: return "unknown status";
    }
}

const char* tns_last_error(void) { return g_err.c_str(); }

}  // extern "C"
