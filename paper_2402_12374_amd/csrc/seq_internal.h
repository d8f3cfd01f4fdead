// Internal declarations shared by the translation units of libseqtree (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "seqtree.h"

namespace seqtree {

// Device-side copy of what both calls derive from parent[]: the ancestor-or-self bitset that
// masks the tree part of the attention scores, and the sibling lists the verification walk
// follows (ascending node id within a list = the order the drafter sampled the children).
struct TreePlan {
    int32_t n = 0;
    int32_t words_per_row = 0;          // 32-bit words per bitset row = 2 * ceil(n / 64)
    uint32_t* anc_words = nullptr;      // [n][words_per_row]
    int32_t* child_start = nullptr;     // [n + 1]
    int32_t* child_list = nullptr;      // [max(n - 1, 1)]
    int32_t* internal_nodes = nullptr;  // [max(n_internal, 1)] nodes that have children, longest sibling list first
    int32_t n_internal = 0;
    int32_t max_children = 0;
};

// Area the kernels use to hand partial results between workgroups, one per (device, stream) the
// library has been called on.  Zeroed once
// when created; the kernels leave it in a reusable state (arrival counters return to zero,
// exchange slots carry ever-increasing tags).
struct SyncArea {
    unsigned long long* verify_slots = nullptr;  // [2][kVerifyMaxGroups][kVerifySlotWords]
    uint32_t* verify_epoch = nullptr;            // [2] tag base of the next verify launch, poison flag
    uint32_t* verify_arrivals = nullptr;         // [1] workgroups of a per-node verify launch that are done
    uint32_t* attn_counters = nullptr;           // [kAttnMaxCounters]
    unsigned long long* draft_exchange = nullptr;  // [kDraftMaxGroups][64] lists of a split row, zero between calls
    uint32_t* draft_arrivals = nullptr;          // [SEQ_MAX_TREE] workgroups of a row that are done
    uint32_t* verify_batch_ctl = nullptr;        // [kVerifyMaxBatch][4] per sequence of a batched launch: tag epoch of the
                                                 // per-node kernel, tag epoch of the walk's teams, arrivals, the teams' poison flag
    unsigned long long* verify_batch_slots = nullptr;  // [kWalkMaxBatch][2][kVerifyMaxGroups][kVerifySlotWords]
    // What the workgroups of a per-node verification launch leave for each other, as words under
    // the tag of their launch: [0] the tag epoch (only ever grows), [1] the word of a team that
    // gave up waiting, [2] the count of workgroups of the launch that are done; from word
    // kChainHeaderWords on the records of up to SEQ_MAX_TREE nodes, then the exchange slots of up
    // to SEQ_MAX_TREE teams.  It lives here and not in the caller's workspace because a tag only
    // proves anything about memory that nothing but these kernels ever writes.
    unsigned long long* chain_area = nullptr;
    // Measured once per device: do workgroups whose ids are congruent mod 8 share an XCD (one
    // L2)?  The attention kernel then keeps all key ranges of a unit on one XCD and can hand
    // partial results over through that L2 without writing it back to memory.
    bool round_robin_xcds = false;
    int compute_units = 256;   // of this device: workgroups of 1024 threads that run at the same time
};

constexpr int kVerifyMaxGroups = 64;
constexpr int kVerifySlotWords = 4;
constexpr int kVerifyTagsPerCall = 4096;
constexpr int kAttnMaxCounters = 16384;
constexpr int kDraftMaxGroups = 16384;
constexpr int kVerifyMaxBatch = 256;
constexpr int kChainHeaderWords = 32;
constexpr int kChainRecordWordsPerNode = 9;     // 5 tagged words per child, 4 per node
constexpr int kChainSlotWordsPerTeam = 256;     // two buffers (by step parity) of 4 x 32 tagged words
constexpr size_t kChainAreaWords = kChainHeaderWords + (size_t)SEQ_MAX_TREE * (kChainRecordWordsPerNode + kChainSlotWordsPerTeam);
constexpr int kWalkMaxBatch = 64;     // teams of the lazy walk that one launch runs side by side

// Looks up (or builds and uploads) the plan for this parent array on the current device.
// Returns SEQ_OK or an error code; *plan receives a copy whose device pointers stay owned by
// the cache.
int get_tree_plan(const int32_t* parent, int32_t n, hipStream_t stream, TreePlan* plan);
int get_sync_area(hipStream_t stream, SyncArea** area);
int release_all();

// Host-side plan construction (no GPU).  Vectors are sized by the callee.
int validate_parent(const int32_t* parent, int32_t n);

constexpr int kXcdProbeBlocks = 1024;
bool probe_round_robin_xcds_into(int* device_ints);
bool stream_is_capturing(hipStream_t stream);

}  // namespace seqtree
