// seq_tree_attn: argument checks (host only, before any GPU call), tree plan lookup, dispatch.
#include <cmath>
#include <cstdint>

#include "seq_internal.h"
#include "tree_attn_kernels.h"

using namespace seqtree;

static int check_attn_shape(int32_t prefix_len, int32_t n_tree, int32_t heads, int32_t kv_heads,
                            int32_t head_dim, int32_t prefix_cap, int32_t dtype) {
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE) return SEQ_ERR_SHAPE;
    if (head_dim != 64 && head_dim != 128) return SEQ_ERR_SHAPE;
    if (heads < 1 || kv_heads < 1 || heads % kv_heads != 0) return SEQ_ERR_SHAPE;
    if (prefix_len < 0 || prefix_len > prefix_cap) return SEQ_ERR_SHAPE;
    return SEQ_OK;
}

static bool aligned16(const void* a, const void* b, const void* c, const void* d, const void* e, const void* f) {
    const uintptr_t all = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c) |
                          reinterpret_cast<uintptr_t>(d) | reinterpret_cast<uintptr_t>(e) | reinterpret_cast<uintptr_t>(f);
    return (all & 15u) == 0;   // (a cache that may be NULL counts as aligned)
}

extern "C" size_t seq_tree_attn_workspace(int32_t prefix_len, int32_t n_tree, int32_t heads,
                                          int32_t kv_heads, int32_t head_dim, int32_t dtype) {
    if (check_attn_shape(prefix_len, n_tree, heads, kv_heads, head_dim, prefix_len, dtype) != SEQ_OK)
        return 256;
    if (dtype == SEQ_F32) return 256;
    return plan_attn_schedule(prefix_len, n_tree, heads, kv_heads, head_dim).workspace_bytes;
}

extern "C" int seq_tree_attn(const void* q, const void* k_cache, const void* v_cache,
                             const void* k_tree, const void* v_tree, const int32_t* parent,
                             int32_t prefix_len, int32_t n_tree, int32_t heads, int32_t kv_heads,
                             int32_t head_dim, void* out, int32_t prefix_cap, int32_t dtype,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!q || !k_tree || !v_tree || !parent || !out) return SEQ_ERR_NULL;
    int rc = check_attn_shape(prefix_len, n_tree, heads, kv_heads, head_dim, prefix_cap, dtype);
    if (rc != SEQ_OK) return rc;
    if (prefix_len > 0 && (!k_cache || !v_cache)) return SEQ_ERR_NULL;
    if (!aligned16(q, k_cache, v_cache, k_tree, v_tree, out)) return SEQ_ERR_ALIGN;
    rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    AttnSchedule sched{};
    if (dtype == SEQ_BF16) {
        sched = plan_attn_schedule(prefix_len, n_tree, heads, kv_heads, head_dim);
        if (sched.splits > 1 && (!workspace || workspace_bytes < sched.workspace_bytes))
            return SEQ_ERR_WORKSPACE;
    }

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TreePlan plan;
    rc = get_tree_plan(parent, n_tree, stream, &plan);
    if (rc != SEQ_OK) return rc;
    if (dtype == SEQ_F32) {
        return launch_tree_attn_rowwise_f32(
            static_cast<const float*>(q), static_cast<const float*>(k_cache),
            static_cast<const float*>(v_cache), static_cast<const float*>(k_tree),
            static_cast<const float*>(v_tree), plan, prefix_len, prefix_cap, n_tree, heads, kv_heads,
            head_dim, static_cast<float*>(out), stream);
    }
    SyncArea* sync = nullptr;
    rc = get_sync_area(stream, &sync);
    if (rc != SEQ_OK) return rc;
    return launch_tree_attn_mfma_bf16(q, k_cache, v_cache, k_tree, v_tree, plan, prefix_len,
                                      prefix_cap, n_tree, heads, kv_heads, head_dim, out, sched,
                                      static_cast<float*>(workspace), sync->attn_counters,
                                      sync->round_robin_xcds, stream);
}

// ---- a batch of sequences that share the tree but not the prefix length ----------------------
// The batch is folded into the heads (query head b * H + h, KV head b * Hk + h / G: a sequence
// only ever meets its own rows); what is new is that a KV head's workgroups take the prefix
// length of their sequence from device memory.  The host cuts the work for the bound it is given.

static int check_batched_shape(int32_t max_prefix_len, int32_t batch, int32_t n_tree, int32_t heads, int32_t kv_heads,
                               int32_t head_dim, int32_t prefix_cap, int32_t dtype) {
    if (batch < 1 || batch > SEQ_MAX_BATCH) return dtype != SEQ_BF16 && dtype != SEQ_F32 ? SEQ_ERR_DTYPE : SEQ_ERR_SHAPE;
    if (heads < 1 || kv_heads < 1 || (long long)batch * heads > (1 << 20)) return SEQ_ERR_SHAPE;
    return check_attn_shape(max_prefix_len, n_tree, batch * heads, batch * kv_heads, head_dim, prefix_cap, dtype);
}

extern "C" size_t seq_tree_attn_batched_workspace(int32_t max_prefix_len, int32_t batch, int32_t n_tree, int32_t heads,
                                                  int32_t kv_heads, int32_t head_dim, int32_t dtype) {
    if (check_batched_shape(max_prefix_len, batch, n_tree, heads, kv_heads, head_dim, max_prefix_len, dtype) != SEQ_OK)
        return 256;
    if (heads % kv_heads != 0) return 256;
    return seq_tree_attn_workspace(max_prefix_len, n_tree, batch * heads, batch * kv_heads, head_dim, dtype);
}

extern "C" int seq_tree_attn_batched(const void* q, const void* k_cache, const void* v_cache,
                                     const void* k_tree, const void* v_tree, const int32_t* parent,
                                     const int32_t* prefix_lens, int32_t max_prefix_len, int32_t batch,
                                     int32_t n_tree, int32_t heads, int32_t kv_heads, int32_t head_dim,
                                     void* out, int32_t prefix_cap, int32_t dtype, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
    if (!q || !k_tree || !v_tree || !parent || !out || !prefix_lens) return SEQ_ERR_NULL;
    int rc = check_batched_shape(max_prefix_len, batch, n_tree, heads, kv_heads, head_dim, prefix_cap, dtype);
    if (rc != SEQ_OK) return rc;
    if (heads % kv_heads != 0) return SEQ_ERR_SHAPE;
    if (max_prefix_len > 0 && (!k_cache || !v_cache)) return SEQ_ERR_NULL;
    if (!aligned16(q, k_cache, v_cache, k_tree, v_tree, out)) return SEQ_ERR_ALIGN;
    rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    const int H = batch * heads, Hk = batch * kv_heads;
    AttnSchedule sched{};
    if (dtype == SEQ_BF16) {
        sched = plan_attn_schedule(max_prefix_len, n_tree, H, Hk, head_dim);
        if (Hk * sched.query_blocks > kAttnMaxCounters) return SEQ_ERR_SHAPE;
        if (sched.splits > 1 && (!workspace || workspace_bytes < sched.workspace_bytes))
            return SEQ_ERR_WORKSPACE;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TreePlan plan;
    rc = get_tree_plan(parent, n_tree, stream, &plan);
    if (rc != SEQ_OK) return rc;
    if (dtype == SEQ_F32) {
        return launch_tree_attn_rowwise_f32(
            static_cast<const float*>(q), static_cast<const float*>(k_cache),
            static_cast<const float*>(v_cache), static_cast<const float*>(k_tree),
            static_cast<const float*>(v_tree), plan, max_prefix_len, prefix_cap, n_tree, H, Hk,
            head_dim, static_cast<float*>(out), stream, prefix_lens, kv_heads);
    }
    SyncArea* sync = nullptr;
    rc = get_sync_area(stream, &sync);
    if (rc != SEQ_OK) return rc;
    return launch_tree_attn_mfma_bf16(q, k_cache, v_cache, k_tree, v_tree, plan, max_prefix_len,
                                      prefix_cap, n_tree, H, Hk, head_dim, out, sched,
                                      static_cast<float*>(workspace), sync->attn_counters,
                                      sync->round_robin_xcds, stream, prefix_lens, kv_heads);
}
