// Launchers of the tree-attention kernels (internal).
#pragma once

#include "seq_internal.h"

namespace seqtree {

int launch_tree_attn_rowwise_f32(const float* q, const float* k_cache, const float* v_cache,
                                 const float* k_tree, const float* v_tree, const TreePlan& plan,
                                 int P, int cap, int n, int H, int Hk, int D, float* out,
                                 hipStream_t stream, const int32_t* prefix_lens = nullptr,
                                 int seq_kv_heads = 0);

// How the bf16 kernel cuts the work: query rows of one KV head (all G = H/Hk heads of the
// group times n tree tokens) in units of 32 * wq rows (one per workgroup; its 8 wavefronts form
// a wq x 8/wq grid of query blocks x key groups), the key axis in `splits` contiguous ranges of
// 32-key tiles whose partial results are merged by the last workgroup to finish.
struct AttnSchedule {
    int wq;             // query blocks per workgroup: 2, 4 or 8
    int query_blocks;   // units per KV head
    int splits;
    int short_ranges, short_weight, long_weight;   // the first short_ranges ranges have weight short_weight, the others long_weight (equal ranges: 0, 1, 1)
    int long_tiles;     // > 0: long ranges of this many tiles in every unit; 0: each range its weight's share of its unit's tiles
    size_t workspace_bytes;
};
constexpr int kKeyTile = 32;

AttnSchedule plan_attn_schedule(int P, int n, int H, int Hk, int D);

int launch_tree_attn_mfma_bf16(const void* q, const void* k_cache, const void* v_cache,
                               const void* k_tree, const void* v_tree, const TreePlan& plan,
                               int P, int cap, int n, int H, int Hk, int D, void* out,
                               const AttnSchedule& sched, float* workspace, uint32_t* counters,
                               bool units_share_l2, hipStream_t stream,
                               // a batch whose sequences differ in prefix length: DEVICE [sequences], each
                               // held to [0, P]; KV head g belongs to sequence g / seq_kv_heads
                               const int32_t* prefix_lens = nullptr, int seq_kv_heads = 0);

}  // namespace seqtree
