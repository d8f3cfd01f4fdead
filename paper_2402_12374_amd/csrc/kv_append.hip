// seq_kv_append: after a verification, the K/V rows of the root and of the accepted tree nodes
// become part of the prefix: they are copied behind the prefix_len valid rows of the cache, in
// path order, so that the next step's tree attends to them as ordinary prefix keys.  (Loop glue:
// the paper keeps its KV cache inside the Transformers library and does not describe this step.)
//
// The accepted path is read on the device (it is seq_verify's output), so the call needs no
// host synchronisation; the number of rows appended is written to device memory for the caller's
// next launch.  One workgroup per possible path position (the tree's depth + 1), 16 bytes per
// lane; a few hundred KB at most -- launch-bound.
#include "seq_internal.h"

namespace seqtree {
namespace {

struct AppendParams {
    const uint4* k_tree; const uint4* v_tree;
    uint4* k_cache; uint4* v_cache;
    const int32_t* path;
    int32_t* new_prefix_len;
    int32_t prefix_len, prefix_cap, n_tree, kv_heads;
    int32_t vecs_per_head;     // head_dim * element size / 16
};

__global__ void __launch_bounds__(256) kv_append_kernel(const AppendParams p) {
    const int j = blockIdx.x;                       // position on the path: 0 = the root
    // the path ends at its first -1; position j exists iff entries 0 .. j-1 are all nodes
    int node = 0;
    for (int i = 0; i < j; ++i) {
        node = p.path[i];
        if (node < 0 || node >= p.n_tree) { node = -1; break; }
    }
    if (j == 0 && threadIdx.x == 0 && p.new_prefix_len) {
        int len = 0;
        while (len < p.n_tree - 1 && p.path[len] >= 0 && p.path[len] < p.n_tree) ++len;
        *p.new_prefix_len = min(p.prefix_len + 1 + len, p.prefix_cap);
    }
    const int row = p.prefix_len + j;
    if (node < 0 || node >= p.n_tree || row >= p.prefix_cap) return;
    const int per_node = p.kv_heads * p.vecs_per_head;
    for (int t = threadIdx.x; t < per_node; t += 256) {
        const int g = t / p.vecs_per_head, part = t - g * p.vecs_per_head;
        const size_t src = (size_t)node * per_node + t;
        const size_t dst = ((size_t)g * p.prefix_cap + row) * p.vecs_per_head + part;
        p.k_cache[dst] = p.k_tree[src];
        p.v_cache[dst] = p.v_tree[src];
    }
}

}  // namespace
}  // namespace seqtree

using namespace seqtree;

extern "C" int seq_kv_append(const void* k_tree, const void* v_tree, const int32_t* accepted_path,
                             const int32_t* parent, void* k_cache, void* v_cache, int32_t prefix_len,
                             int32_t n_tree, int32_t kv_heads, int32_t head_dim, int32_t prefix_cap,
                             int32_t dtype, int32_t* new_prefix_len, void* hip_stream) {
    if (!k_tree || !v_tree || !accepted_path || !parent || !k_cache || !v_cache) return SEQ_ERR_NULL;
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE || kv_heads < 1 || (head_dim != 64 && head_dim != 128) ||
        prefix_len < 0 || prefix_cap < 1 || prefix_len > prefix_cap)
        return SEQ_ERR_SHAPE;
    int rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    for (const void* ptr : {k_tree, v_tree, (const void*)k_cache, (const void*)v_cache})
        if (reinterpret_cast<uintptr_t>(ptr) & 15) return SEQ_ERR_SHAPE;
    int depth_max = 0;
    {
        int depth[SEQ_MAX_TREE];
        depth[0] = 0;
        for (int i = 1; i < n_tree; ++i) { depth[i] = depth[parent[i]] + 1; depth_max = depth[i] > depth_max ? depth[i] : depth_max; }
    }
    AppendParams p;
    p.k_tree = static_cast<const uint4*>(k_tree);
    p.v_tree = static_cast<const uint4*>(v_tree);
    p.k_cache = static_cast<uint4*>(k_cache);
    p.v_cache = static_cast<uint4*>(v_cache);
    p.path = accepted_path;
    p.new_prefix_len = new_prefix_len;
    p.prefix_len = prefix_len;
    p.prefix_cap = prefix_cap;
    p.n_tree = n_tree;
    p.kv_heads = kv_heads;
    p.vecs_per_head = head_dim * (dtype == SEQ_BF16 ? 2 : 4) / 16;
    kv_append_kernel<<<depth_max + 1, 256, 0, static_cast<hipStream_t>(hip_stream)>>>(p);
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
