// Tree plan: everything both calls derive from parent[] before any arithmetic happens.
// The tree is fixed ahead of time (Sec. 3.1: the structure is found offline; Sec. 4.1
// "Implementation Details": because it is known in advance the step can be captured as a
// graph), so the plan is built once per tree shape and cached.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <vector>

#include "seq_internal.h"

namespace seqtree {

namespace {
// Which XCD does each workgroup of a launch run on?
__global__ void xcd_probe_kernel(int* out) {
    if (threadIdx.x == 0) {
        int id;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
        out[blockIdx.x] = id & 0xF;
    }
}

bool probe_round_robin_xcds() {
    int* dev = nullptr;
    if (hipMalloc(&dev, sizeof(int) * kXcdProbeBlocks) != hipSuccess) return false;
    const bool answer = probe_round_robin_xcds_into(dev);
    (void)hipFree(dev);
    return answer;
}
}  // namespace

// True iff workgroup b runs on the XCD of workgroup b % 8 and those eight are distinct.  Runs a
// small kernel on the null stream and reads its output back (synchronous); `device_ints` is
// device memory for kXcdProbeBlocks ints that the caller lends.
bool probe_round_robin_xcds_into(int* device_ints) {
    std::vector<int> host(kXcdProbeBlocks, -1);
    hipLaunchKernelGGL(xcd_probe_kernel, dim3(kXcdProbeBlocks), dim3(64), 0, 0, device_ints);
    if (hipGetLastError() != hipSuccess ||
        hipMemcpy(host.data(), device_ints, sizeof(int) * kXcdProbeBlocks, hipMemcpyDeviceToHost) != hipSuccess)
        return false;
    for (int b = 0; b < 8; ++b)
        for (int c = 0; c < b; ++c)
            if (host[b] == host[c]) return false;
    for (int b = 8; b < kXcdProbeBlocks; ++b)
        if (host[b] != host[b % 8]) return false;
    return true;
}

bool stream_is_capturing(hipStream_t stream) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(stream, &status) == hipSuccess && status != hipStreamCaptureStatusNone;
}

int validate_parent(const int32_t* parent, int32_t n) {
    if (n < 1 || n > SEQ_MAX_TREE) return SEQ_ERR_SHAPE;
    if (parent[0] != -1) return SEQ_ERR_TREE;
    for (int32_t i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i) return SEQ_ERR_TREE;
    return SEQ_OK;
}

static int words_per_row(int32_t n) { return 2 * ((n + 63) / 64); }

static void build_host(const int32_t* parent, int32_t n, std::vector<int32_t>* depth,
                       std::vector<int32_t>* child_start, std::vector<int32_t>* child_list,
                       std::vector<uint32_t>* anc) {
    const int wpr = words_per_row(n);
    depth->assign(n, 0);
    child_start->assign(n + 1, 0);
    child_list->assign(n > 1 ? n - 1 : 1, 0);
    anc->assign((size_t)n * wpr, 0u);
    for (int32_t i = 1; i < n; ++i) {
        (*depth)[i] = (*depth)[parent[i]] + 1;
        (*child_start)[parent[i] + 1] += 1;
    }
    for (int32_t v = 0; v < n; ++v) (*child_start)[v + 1] += (*child_start)[v];
    std::vector<int32_t> fill(child_start->begin(), child_start->end() - 1);
    for (int32_t i = 1; i < n; ++i) (*child_list)[fill[parent[i]]++] = i;  // ascending id per list
    for (int32_t i = 0; i < n; ++i) {
        uint32_t* row = anc->data() + (size_t)i * wpr;
        if (i > 0) std::memcpy(row, anc->data() + (size_t)parent[i] * wpr, sizeof(uint32_t) * wpr);
        row[i >> 5] |= 1u << (i & 31);
    }
}

namespace {
// Where the library's own device memory comes from.  The host tests swap in plain host memory
// (no GPU involved) to exercise the bookkeeping below: what is kept, what is handed out twice,
// what is refused.
struct DeviceMemory {
    bool (*current_device)(int* device);
    void* (*alloc)(size_t bytes);
    bool (*upload)(void* dst, const void* src, size_t bytes);   // synchronous
    bool (*zero)(void* dst, size_t bytes);                      // synchronous
    void (*release)(void* ptr);
    bool (*capturing)(hipStream_t stream);   // work enqueued on the stream is being recorded, not run
    bool gpu;
};
const DeviceMemory kHipMemory = {
    [](int* device) { return hipGetDevice(device) == hipSuccess; },
    [](size_t bytes) { void* ptr = nullptr; return hipMalloc(&ptr, bytes) == hipSuccess ? ptr : nullptr; },
    [](void* dst, const void* src, size_t bytes) { return hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice) == hipSuccess; },
    [](void* dst, size_t bytes) { return hipMemset(dst, 0, bytes) == hipSuccess && hipDeviceSynchronize() == hipSuccess; },
    [](void* ptr) { (void)hipFree(ptr); },
    [](hipStream_t stream) { return stream_is_capturing(stream); },
    true,
};
const DeviceMemory kHostMemory = {
    [](int* device) { *device = 0; return true; },
    [](size_t bytes) { return std::malloc(bytes); },
    [](void* dst, const void* src, size_t bytes) { std::memcpy(dst, src, bytes); return true; },
    [](void* dst, size_t bytes) { std::memset(dst, 0, bytes); return true; },
    [](void* ptr) { std::free(ptr); },
    [](hipStream_t stream) { return (reinterpret_cast<uintptr_t>(stream) & 1) != 0; },   // odd handles play "capturing"
    false,
};
const DeviceMemory* g_mem = &kHipMemory;

struct CacheEntry {
    int device;
    std::vector<int32_t> parent;
    TreePlan plan;
};
struct StreamSync {
    int device;
    hipStream_t stream;
    SyncArea area;
};
std::mutex g_mutex;
// Plans are never evicted: a captured graph keeps the raw device pointers of the plan it was
// captured with for as long as it lives, and the library cannot know how long that is.  A plan
// is small (140 KB at 1024 nodes, 1 KB at 64), so the cache is bounded by a count and a call
// with one tree too many is refused.
std::deque<CacheEntry> g_cache;
std::deque<StreamSync> g_sync;   // (a deque never moves its elements: handed-out pointers stay valid)

void free_plan(TreePlan& p) {
    if (p.anc_words) g_mem->release(p.anc_words);
    if (p.child_start) g_mem->release(p.child_start);
    if (p.child_list) g_mem->release(p.child_list);
    if (p.internal_nodes) g_mem->release(p.internal_nodes);
    p = TreePlan{};
}
void free_area(SyncArea& a) {
    if (a.verify_slots) g_mem->release(a.verify_slots);
    if (a.attn_counters) g_mem->release(a.attn_counters);
    if (a.draft_exchange) g_mem->release(a.draft_exchange);
    if (a.chain_area) g_mem->release(a.chain_area);
    a = SyncArea{};
}
}  // namespace

int get_tree_plan(const int32_t* parent, int32_t n, hipStream_t stream, TreePlan* out) {
    int device = 0;
    if (!g_mem->current_device(&device)) return SEQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mutex);
    for (auto& e : g_cache) {
        if (e.device == device && (int32_t)e.parent.size() == n &&
            std::memcmp(e.parent.data(), parent, sizeof(int32_t) * n) == 0) {
            *out = e.plan;
            return SEQ_OK;
        }
    }
    if (g_cache.size() >= (size_t)SEQ_MAX_PLANS) return SEQ_ERR_FULL;
    // a new plan means allocations and synchronous copies, which would invalidate a capture
    if (g_mem->capturing(stream)) return SEQ_ERR_CAPTURE;
    std::vector<int32_t> depth, cstart, clist;
    std::vector<uint32_t> anc;
    build_host(parent, n, &depth, &cstart, &clist, &anc);
    CacheEntry e;
    e.device = device;
    e.parent.assign(parent, parent + n);
    e.plan.n = n;
    e.plan.words_per_row = words_per_row(n);
    for (int32_t v = 0; v < n; ++v)
        e.plan.max_children = std::max(e.plan.max_children, cstart[v + 1] - cstart[v]);
    // nodes with children, those with the longest sibling lists (the longest chains of dependent
    // steps in the per-node verification kernel) first
    std::vector<int32_t> internal;
    for (int32_t v = 0; v < n; ++v)
        if (cstart[v + 1] > cstart[v]) internal.push_back(v);
    std::stable_sort(internal.begin(), internal.end(), [&](int32_t a, int32_t b) {
        return cstart[a + 1] - cstart[a] > cstart[b + 1] - cstart[b];
    });
    e.plan.n_internal = (int32_t)internal.size();
    if (internal.empty()) internal.push_back(0);
    e.plan.anc_words = static_cast<uint32_t*>(g_mem->alloc(anc.size() * sizeof(uint32_t)));
    e.plan.internal_nodes = static_cast<int32_t*>(g_mem->alloc(internal.size() * sizeof(int32_t)));
    e.plan.child_start = static_cast<int32_t*>(g_mem->alloc(cstart.size() * sizeof(int32_t)));
    e.plan.child_list = static_cast<int32_t*>(g_mem->alloc(clist.size() * sizeof(int32_t)));
    const bool ok = e.plan.anc_words && e.plan.child_start && e.plan.child_list && e.plan.internal_nodes &&
                    g_mem->upload(e.plan.internal_nodes, internal.data(), internal.size() * sizeof(int32_t)) &&
                    g_mem->upload(e.plan.anc_words, anc.data(), anc.size() * sizeof(uint32_t)) &&
                    g_mem->upload(e.plan.child_start, cstart.data(), cstart.size() * sizeof(int32_t)) &&
                    g_mem->upload(e.plan.child_list, clist.data(), clist.size() * sizeof(int32_t));
    if (!ok) {
        free_plan(e.plan);
        if (g_mem->gpu) (void)hipGetLastError();
        return SEQ_ERR_HIP;
    }
    g_cache.push_back(std::move(e));
    *out = g_cache.back().plan;
    return SEQ_OK;
}

// One area per (device, stream): calls on different streams of a device may then overlap in
// time -- they share nothing but the read-only plans -- and calls on one stream are serialised
// by the stream itself.  A stream that is being captured cannot be given an area (that takes
// allocations and a synchronous clear): if it has none yet, its calls are recorded with the
// area of the first stream the library was called on for this device.
int get_sync_area(hipStream_t stream, SyncArea** out) {
    int device = 0;
    if (!g_mem->current_device(&device)) return SEQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mutex);
    int on_device = 0;
    SyncArea* first = nullptr;
    for (auto& s : g_sync) {
        if (s.device != device) continue;
        if (s.stream == stream) { *out = &s.area; return SEQ_OK; }
        if (!first) first = &s.area;
        ++on_device;
    }
    if (g_mem->capturing(stream)) {
        if (!first) return SEQ_ERR_CAPTURE;
        *out = first;
        return SEQ_OK;
    }
    if (on_device >= SEQ_MAX_STREAMS) return SEQ_ERR_FULL;
    StreamSync s;
    s.device = device;
    s.stream = stream;
    // the exchange slots, then two 64-bit cells: tag epoch and poison flag; arrival counter
    const size_t slot_words = (size_t)2 * kVerifyMaxGroups * kVerifySlotWords;
    const size_t slot_bytes = sizeof(unsigned long long) * (slot_words + 2);
    const size_t ctr_bytes = sizeof(uint32_t) * kAttnMaxCounters;
    // the lists of split rows (8 MiB), then one arrival counter per row
    const size_t draft_words = (size_t)kDraftMaxGroups * 64;
    // ... then the per-sequence cells and exchange slots of batched verification launches
    const size_t batch_slot_words = (size_t)kWalkMaxBatch * 2 * kVerifyMaxGroups * kVerifySlotWords;
    static_assert((SEQ_MAX_TREE + 4 * kVerifyMaxBatch) % 2 == 0, "the slots that follow hold 64-bit words");
    const size_t draft_bytes = sizeof(unsigned long long) * draft_words + sizeof(uint32_t) * SEQ_MAX_TREE +
                               sizeof(uint32_t) * 4 * kVerifyMaxBatch + sizeof(unsigned long long) * batch_slot_words;
    s.area.verify_slots = static_cast<unsigned long long*>(g_mem->alloc(slot_bytes));
    s.area.attn_counters = static_cast<uint32_t*>(g_mem->alloc(ctr_bytes));
    s.area.draft_exchange = static_cast<unsigned long long*>(g_mem->alloc(draft_bytes));
    const size_t chain_bytes = sizeof(unsigned long long) * kChainAreaWords;
    s.area.chain_area = static_cast<unsigned long long*>(g_mem->alloc(chain_bytes));
    const bool ok = s.area.verify_slots && s.area.attn_counters && s.area.draft_exchange && s.area.chain_area &&
                    g_mem->zero(s.area.chain_area, chain_bytes) &&
                    g_mem->zero(s.area.verify_slots, slot_bytes) && g_mem->zero(s.area.attn_counters, ctr_bytes) &&
                    g_mem->zero(s.area.draft_exchange, draft_bytes);
    if (!ok) {
        free_area(s.area);
        if (g_mem->gpu) (void)hipGetLastError();
        return SEQ_ERR_HIP;
    }
    s.area.verify_epoch = reinterpret_cast<uint32_t*>(s.area.verify_slots + slot_words);
    s.area.verify_arrivals = s.area.verify_epoch + 2;
    s.area.draft_arrivals = reinterpret_cast<uint32_t*>(s.area.draft_exchange + draft_words);
    s.area.verify_batch_ctl = s.area.draft_arrivals + SEQ_MAX_TREE;
    s.area.verify_batch_slots = reinterpret_cast<unsigned long long*>(s.area.verify_batch_ctl + 4 * kVerifyMaxBatch);
    // what is measured once per device is copied from the device's first area
    bool known = false;
    for (auto& other : g_sync)
        if (other.device == device) {
            s.area.round_robin_xcds = other.area.round_robin_xcds;
            s.area.compute_units = other.area.compute_units;
            known = true;
            break;
        }
    if (!known && g_mem->gpu) {
        s.area.round_robin_xcds = probe_round_robin_xcds();
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0)
            s.area.compute_units = cus;
    }
    g_sync.push_back(s);
    *out = &g_sync.back().area;
    return SEQ_OK;
}

int release_all() {
    std::lock_guard<std::mutex> lock(g_mutex);
    int current = 0;
    const bool have_dev = g_mem->gpu && hipGetDevice(&current) == hipSuccess;
    for (auto& e : g_cache) {
        if (have_dev) (void)hipSetDevice(e.device);
        free_plan(e.plan);
    }
    g_cache.clear();
    for (auto& s : g_sync) {
        if (have_dev) (void)hipSetDevice(s.device);
        free_area(s.area);
    }
    g_sync.clear();
    if (have_dev) (void)hipSetDevice(current);
    return SEQ_OK;
}

}  // namespace seqtree

extern "C" int seq_tree_plan_host(const int32_t* parent, int32_t n_tree, int32_t* depth,
                                  int32_t* child_start, int32_t* child_list, uint32_t* anc_words) {
    if (!parent) return SEQ_ERR_NULL;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE) return SEQ_ERR_SHAPE;
    int rc = seqtree::validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    std::vector<int32_t> d, cs, cl;
    std::vector<uint32_t> anc;
    seqtree::build_host(parent, n_tree, &d, &cs, &cl, &anc);
    if (depth) std::memcpy(depth, d.data(), sizeof(int32_t) * n_tree);
    if (child_start) std::memcpy(child_start, cs.data(), sizeof(int32_t) * (n_tree + 1));
    if (child_list && n_tree > 1) std::memcpy(child_list, cl.data(), sizeof(int32_t) * (n_tree - 1));
    if (anc_words) std::memcpy(anc_words, anc.data(), sizeof(uint32_t) * anc.size());
    return SEQ_OK;
}

extern "C" int seq_shutdown(void) { return seqtree::release_all(); }

extern "C" const char* seq_strerror(int code) {
    switch (code) {
        case SEQ_OK: return "ok";
        case SEQ_ERR_NULL: return "a required pointer is NULL";
        case SEQ_ERR_SHAPE: return "unsupported or inconsistent sizes";
        case SEQ_ERR_TREE: return "parent[] is not a tree in topological order";
        case SEQ_ERR_DTYPE: return "dtype must be SEQ_BF16 or SEQ_F32";
        case SEQ_ERR_TEMPERATURE: return "temperature must be finite and >= 0";
        case SEQ_ERR_WORKSPACE: return "workspace missing or too small";
        case SEQ_ERR_HIP: return "HIP runtime error";
        case SEQ_ERR_ALGORITHM: return "algorithm must be one of SEQ_VERIFY_*";
        case SEQ_ERR_FULL: return "too many distinct trees or streams: seq_shutdown() releases them";
        case SEQ_ERR_CAPTURE: return "first call for this tree or device made under stream capture: make it once outside";
        case SEQ_ERR_ALIGN: return "an attention tensor is not 16-byte aligned";
        default: return "unknown seqtree error code";
    }
}

extern "C" int seq_version(void) { return 200; }

// Test hooks (not part of the public header).  With host memory switched on the bookkeeping of
// plans and synchronisation areas runs without a GPU; switching discards everything held.
extern "C" void seqtree_internal_use_host_memory(int on) {
    (void)seqtree::release_all();
    seqtree::g_mem = on ? &seqtree::kHostMemory : &seqtree::kHipMemory;
}
extern "C" int seqtree_internal_plan_pointers(const int32_t* parent, int32_t n_tree, void* hip_stream, void** three) {
    seqtree::TreePlan plan;
    int rc = seqtree::validate_parent(parent, n_tree);
    if (rc == SEQ_OK) rc = seqtree::get_tree_plan(parent, n_tree, static_cast<hipStream_t>(hip_stream), &plan);
    if (rc != SEQ_OK) return rc;
    three[0] = plan.anc_words; three[1] = plan.child_start; three[2] = plan.child_list;
    return SEQ_OK;
}
extern "C" int seqtree_internal_sync_area_of(void* hip_stream, void** area) {
    seqtree::SyncArea* a = nullptr;
    const int rc = seqtree::get_sync_area(static_cast<hipStream_t>(hip_stream), &a);
    *area = a;
    return rc;
}

// A plain copy of a known size: the yardstick the benchmark puts beside its kernels when HBM
// traffic counters are collected, so that the counters' unit can be checked against bytes
// that are known exactly (16 bytes per lane, grid-stride, `bytes` a multiple of 16).
__global__ void __launch_bounds__(256) seq_copy_probe_kernel(const uint4* __restrict__ src,
                                                             uint4* __restrict__ dst, size_t count) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256)
        dst[i] = src[i];
}

extern "C" int seqtree_internal_copy_probe(const void* src, void* dst, size_t bytes, void* hip_stream) {
    if (!src || !dst) return SEQ_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return SEQ_ERR_SHAPE;
    const size_t count = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>(8192, (count + 255) / 256);
    hipLaunchKernelGGL(seq_copy_probe_kernel, dim3(blocks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), count);
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
