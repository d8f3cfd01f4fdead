// seq_tree_attn: argument checks (host only, before any GPU call), tree plan lookup, dispatch.
#include <cmath>

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
