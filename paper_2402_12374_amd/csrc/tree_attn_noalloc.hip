// seq_tree_attn_noalloc: seq_tree_attn for callers that cannot allocate device memory -- code
// under stream capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels,
// same results; everything the ordinary entry point keeps in the caller's workspace, the plan
// cache and the stream's synchronisation area lives in one static device array instead:
//
//     [ ancestor bitset of the tree | arrival counters of the range merge | partial results ]
//
// The bitset is rebuilt by a small kernel at every call from the parent array, which travels in
// that kernel's arguments (no host-to-device copy, no cache, nothing to upload), and the same
// kernel clears the arrival counters this call will use.
#include <mutex>

#include "seq_internal.h"
#include "tree_attn_kernels.h"

namespace {
constexpr size_t kAncBytes = (size_t)SEQ_MAX_TREE * (2 * (SEQ_MAX_TREE / 64)) * sizeof(uint32_t);   // 128 KiB
constexpr size_t kCounterBytes = (size_t)seqtree::kAttnMaxCounters * sizeof(uint32_t);                // 64 KiB
constexpr size_t kPartialBytes = (size_t)SEQ_NOALLOC_MAX_PARTIAL_BYTES;
constexpr size_t kScratchBytes = kAncBytes + kCounterBytes + kPartialBytes;
static_assert(kAncBytes % 256 == 0 && kCounterBytes % 256 == 0, "every part starts on a 256-byte boundary");
static_assert(kCounterBytes >= sizeof(int) * seqtree::kXcdProbeBlocks, "the placement probe borrows the counters");

}  // namespace

// One copy per GPU the library's code object is loaded on, at an address of its own.  In host
// code this name is only a handle for hipGetSymbolAddress: the address the kernels get is the
// one that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace seqtree {
namespace {

struct DeviceScratch {
    unsigned char* base = nullptr;   // device address of `scratch` on this GPU
    bool share_l2 = false;           // workgroups b and b + 8 share an XCD (measured at set-up)
    bool ready = false;
};
constexpr int kMaxDevices = 64;
DeviceScratch g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

// The tree as a kernel argument: 2 KiB by value, baked into a graph node when captured.
struct ParentArg {
    int16_t parent[SEQ_MAX_TREE];
};

// anc[i] = bitset of i and its ancestors, words_per_row 32-bit words per row; thread i writes row
// i.  parent[j] < j, so the walk from i to the root meets the words of its row in descending
// order: each word is written once, finished, and the words in between are written as zero.
// Also clears the arrival counters of the units the attention launch that follows will use.
__global__ __launch_bounds__(SEQ_MAX_TREE) void noalloc_plan_kernel(const ParentArg tree, int n, int words_per_row,
                                                                    uint32_t* __restrict__ anc,
                                                                    uint32_t* __restrict__ counters, int units) {
    __shared__ int16_t par[SEQ_MAX_TREE];
    const int i = threadIdx.x;
    if (i < n) par[i] = tree.parent[i];
    for (int u = i; u < units; u += SEQ_MAX_TREE) counters[u] = 0u;
    __syncthreads();
    if (i >= n) return;
    uint32_t* const row = anc + (size_t)i * words_per_row;
    int next_unwritten = words_per_row - 1;   // words above it are final
    int word = i >> 5;
    uint32_t bits = 0u;
    for (int j = i; j >= 0; j = par[j]) {     // at most n steps: the host has checked parent[j] < j
        if ((j >> 5) != word) {
            for (; next_unwritten > word; --next_unwritten) row[next_unwritten] = 0u;
            row[word] = bits;
            next_unwritten = word - 1;
            word = j >> 5;
            bits = 0u;
        }
        bits |= 1u << (j & 31);
    }
    for (; next_unwritten > word; --next_unwritten) row[next_unwritten] = 0u;
    row[word] = bits;
    for (int w = word - 1; w >= 0; --w) row[w] = 0u;
}

// Once per device, with that device current: where does this GPU keep its copy of `scratch`,
// and how does it place workgroups on XCDs.
int set_up_device(int device, hipStream_t stream, DeviceScratch** out) {
    if (device < 0 || device >= kMaxDevices) return SEQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    DeviceScratch& d = g_scratch[device];
    if (!d.ready) {
        if (stream_is_capturing(stream)) return SEQ_ERR_CAPTURE;   // the probe below synchronises
        unsigned char* base = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void**>(&base), HIP_SYMBOL(scratch)) != hipSuccess || !base) {
            (void)hipGetLastError();
            return SEQ_ERR_HIP;
        }
        d.base = base;
        // the probe writes kXcdProbeBlocks ints where the counters live; every call clears the
        // counters it uses before it uses them
        d.share_l2 = probe_round_robin_xcds_into(reinterpret_cast<int*>(base + kAncBytes));
        d.ready = true;
    }
    *out = &d;
    return SEQ_OK;
}

}  // namespace
}  // namespace seqtree

using namespace seqtree;

extern "C" int seq_tree_attn_noalloc(const void* q, const void* k_cache, const void* v_cache,
                                     const void* k_tree, const void* v_tree, const int32_t* parent,
                                     int32_t prefix_len, int32_t n_tree, int32_t heads, int32_t kv_heads,
                                     int32_t head_dim, void* out, int32_t prefix_cap, int32_t dtype,
                                     void* hip_stream) {
    if (!q || !k_tree || !v_tree || !parent || !out) return SEQ_ERR_NULL;
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE) return SEQ_ERR_SHAPE;
    if (head_dim != 64 && head_dim != 128) return SEQ_ERR_SHAPE;
    if (heads < 1 || kv_heads < 1 || heads % kv_heads != 0) return SEQ_ERR_SHAPE;
    if (prefix_len < 0 || prefix_len > prefix_cap) return SEQ_ERR_SHAPE;
    if (prefix_len > 0 && (!k_cache || !v_cache)) return SEQ_ERR_NULL;
    if (((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_cache) | reinterpret_cast<uintptr_t>(v_cache) |
          reinterpret_cast<uintptr_t>(k_tree) | reinterpret_cast<uintptr_t>(v_tree) | reinterpret_cast<uintptr_t>(out)) & 15u) != 0)
        return SEQ_ERR_ALIGN;
    int rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;

    // What the call needs of the static array, checked before anything touches the GPU.
    AttnSchedule sched{};
    int units = 0;
    if (dtype == SEQ_BF16) {
        sched = plan_attn_schedule(prefix_len, n_tree, heads, kv_heads, head_dim);
        units = kv_heads * sched.query_blocks;
        if (units > kAttnMaxCounters) return SEQ_ERR_SHAPE;
        if (sched.splits > 1 && sched.workspace_bytes > kPartialBytes) return SEQ_ERR_WORKSPACE;
    }

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return SEQ_ERR_HIP;
    DeviceScratch* dev = nullptr;
    rc = set_up_device(device, stream, &dev);
    if (rc != SEQ_OK) return rc;
    uint32_t* const anc = reinterpret_cast<uint32_t*>(dev->base);
    uint32_t* const counters = reinterpret_cast<uint32_t*>(dev->base + kAncBytes);
    float* const partials = reinterpret_cast<float*>(dev->base + kAncBytes + kCounterBytes);

    TreePlan plan;
    plan.n = n_tree;
    plan.words_per_row = 2 * ((n_tree + 63) / 64);
    plan.anc_words = anc;
    ParentArg tree;
    for (int32_t i = 0; i < n_tree; ++i) tree.parent[i] = (int16_t)parent[i];
    for (int32_t i = n_tree; i < SEQ_MAX_TREE; ++i) tree.parent[i] = -1;
    hipLaunchKernelGGL(noalloc_plan_kernel, dim3(1), dim3(SEQ_MAX_TREE), 0, stream, tree, n_tree,
                       plan.words_per_row, anc, counters, units);
    if (hipGetLastError() != hipSuccess) return SEQ_ERR_HIP;
    if (dtype == SEQ_F32) {
        return launch_tree_attn_rowwise_f32(
            static_cast<const float*>(q), static_cast<const float*>(k_cache),
            static_cast<const float*>(v_cache), static_cast<const float*>(k_tree),
            static_cast<const float*>(v_tree), plan, prefix_len, prefix_cap, n_tree, heads, kv_heads,
            head_dim, static_cast<float*>(out), stream);
    }
    return launch_tree_attn_mfma_bf16(q, k_cache, v_cache, k_tree, v_tree, plan, prefix_len, prefix_cap,
                                      n_tree, heads, kv_heads, head_dim, out, sched, partials, counters,
                                      dev->share_l2, stream);
}
