// Device-side pieces shared by the two kernels behind seq_verify (internal): row loads, the
// exponential, wavefront reductions, and the scalar state of Algorithm 2 (Sec. 3.2.1) at one
// tree node.
//
// Residual and draft are never rewritten.  After j rejections at a node, with S the rejected
// tokens (whose p and q registers are set to zero when they are rejected):
//     D_j[x] = q[x] / massQ,   massQ = sum_x q[x]                       (or 1/(V-|S|) off S once
//                                                                        massQ has reached 0)
//     R_j[x] = max(p[x] - A q[x] - B, 0) / W
// where A (resp. B) accumulates W / massQ (resp. W / (V-|S|)) at every rejection and W is the
// vocabulary sum of the numerator.  This is the update R <- norm(max(R - D, 0)) unrolled: the
// nested max(., 0) collapse because the subtracted amounts never decrease.  A rejection thus
// costs one read-only pass over the vocabulary.
#pragma once

#include <cmath>

#include "seq_internal.h"

namespace seqtree {
namespace verify {

constexpr int kThreads = 1024;  // few, fat workgroups
constexpr int kWaves = kThreads / 64;
static_assert(kWaves <= 16, "the first wavefront folds the per-wave partials within one 16-lane row");

struct VerifyParams {
    const void* target;
    const void* draft;
    const int32_t* tokens;
    const float* uniforms;
    const int32_t* child_start;
    const int32_t* child_list;
    int32_t* path;
    int32_t* bonus;
    int32_t* trace;
    unsigned long long* records;   // (top-k baseline) the nodes' draws, in the caller's workspace behind the trace
    unsigned long long* chain_area;   // per-node kernels: header, records, team slots (the library's, see SyncArea)
    unsigned long long* slots;
    uint32_t* epoch;
    uint32_t* poison;       // lazy walk: set after a timed-out wait, later launches refuse to run
    uint32_t* arrivals;
    uint32_t spin_limit;
    int n, V, W;
    float inv_T;
    int with_replacement;   // SpecInfer: the draft distribution is never updated (Algorithm 2 without its blue lines)
    // a batched launch (grid.y = sequences): byte strides between sequences
    size_t batch_logit_bytes, batch_workspace_bytes;
    uint32_t* batch_ctl;    // [sequences][4]: per-node kernel's epoch, walk's epoch, arrivals, walk's poison flag
    unsigned long long* batch_slots;   // [sequences][2][kVerifyMaxGroups][kVerifySlotWords]
    unsigned long long* chain_records; // per-node kernels: this sequence's child records [n][5], then node records [n][4]
    // per-node kernel with a team of W workgroups per node (vocabularies beyond one workgroup's registers)
    unsigned long long* team_slots;    // [teams][2][kTeamSlotWords][kTeamMaxW] tagged words
    const int32_t* internal_nodes;     // [n_internal] nodes that have children, longest sibling list first
    int n_internal;
    int team_xcd;                      // workgroup b runs on XCD b % 8: keep a team on one XCD
};

// A batched launch runs the same code once per sequence (grid.y): every sequence has its own
// logits, tokens, uniforms, outputs, workspace, tag epochs, arrival counter and exchange slots;
// the tree is shared.
__device__ __forceinline__ VerifyParams params_of_sequence(const VerifyParams& in, int b, bool walk_team) {
    VerifyParams p = in;
    p.target = static_cast<const char*>(in.target) + (size_t)b * in.batch_logit_bytes;
    p.draft = in.draft ? static_cast<const char*>(in.draft) + (size_t)b * in.batch_logit_bytes : nullptr;
    p.tokens = in.tokens + (size_t)b * in.n;
    p.uniforms = in.uniforms + (size_t)b * in.n;
    p.path = in.path + (size_t)b * in.n;
    p.bonus = in.bonus + b;
    p.trace = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(in.trace) + (size_t)b * in.batch_workspace_bytes);
    p.records = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(in.records) + (size_t)b * in.batch_workspace_bytes);
    p.chain_records = in.chain_records + (size_t)b * in.n * kChainRecordWordsPerNode;   // (the sequences of a launch hold at most SEQ_MAX_TREE nodes together)
    p.epoch = in.batch_ctl + 4 * b + (walk_team ? 1 : 0);
    p.poison = in.batch_ctl + 4 * b + 3;
    p.arrivals = in.batch_ctl + 4 * b + 2;
    if (walk_team) p.slots = in.batch_slots + (size_t)b * 2 * kVerifyMaxGroups * kVerifySlotWords;
    return p;
}

// verify_chains.hip: every node's sibling chain in parallel, then the walk over the results.
// Vocabularies up to kChainsMaxVocab; dtype SEQ_BF16 or SEQ_F32.
constexpr int kChainsMaxVocab = 32768;
void launch_verify_chains(const VerifyParams& p, int dtype, hipStream_t stream, int batch = 1);
// The same chains for larger vocabularies: a team of p.W = ceil(V / 16384) workgroups of 512
// threads per node that has children (p.internal_nodes), which meet in p.team_slots.
constexpr int kTeamMaxW = 32;
constexpr int kTeamSlotWords = 4;
int team_size_for(int vocab);
void launch_verify_chains_team(const VerifyParams& p, int dtype, hipStream_t stream);
// verify_topk.hip: naive / top-k sampling (Sec. 2.2): one draw from the target per node, then the walk.
void launch_verify_topk(const VerifyParams& p, int dtype, hipStream_t stream, int batch = 1);
void set_topk_mode(int mode);

template <typename LT> __device__ __forceinline__ float load_logit(const LT* row, int x);
template <> __device__ __forceinline__ float load_logit<float>(const float* row, int x) { return row[x]; }
template <> __device__ __forceinline__ float load_logit<uint16_t>(const uint16_t* row, int x) {
    return __uint_as_float((uint32_t)row[x] << 16);
}

// EPT consecutive logits of one row starting at `base` (a multiple of EPT), tempered; tokens past
// the vocabulary read as -inf.  16-byte loads when the row starts and the vocabulary allow it
// (`vec_ok`: every 16-byte group of a row then lies wholly inside or wholly outside it); otherwise
// token by token, in a loop that is kept rolled: it runs for odd vocabularies only and would
// otherwise be most of the kernel's code.
// CH slices of a row -- slice c starts at token base + c * stride -- and, if TWO, the same slices
// of a second row, all requested before the first is touched: one trip to memory for everything
// a thread holds.  (Requests written one slice or one row after the other, each under its own
// condition, come out of the compiler as one trip each: it waits for a load at the end of the
// block that issued it.)  A vector group past the end of the row reads the row's first group
// instead and is replaced by -inf.
template <typename LT, int EPT, int CH, bool TWO>
__device__ __forceinline__ void load_row_slices(const LT* row_a, const LT* row_b, int base, int stride, int V, float inv_T,
                                                bool vec_ok, float* xa, float* xb) {
    constexpr int kPerVec = 16 / (int)sizeof(LT), kVecs = EPT / kPerVec;
    if (vec_ok) {
        uint4 ra[CH][kVecs], rb[CH][kVecs];
        bool inside[CH][kVecs];
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int g = 0; g < kVecs; ++g) {
                const int first = base + c * stride + g * kPerVec;
                inside[c][g] = first + kPerVec <= V;
                const int at = inside[c][g] ? first : 0;
                ra[c][g] = *reinterpret_cast<const uint4*>(row_a + at);
                if (TWO) rb[c][g] = *reinterpret_cast<const uint4*>(row_b + at);
            }
        const uint32_t gone = sizeof(LT) == 4 ? 0xFF800000u : 0xFF80FF80u;   // -inf, or -inf as a bf16 pair
        auto unpack = [&](const uint4& got, bool in, float* x) __attribute__((always_inline)) {
            const uint32_t w[4] = {in ? got.x : gone, in ? got.y : gone, in ? got.z : gone, in ? got.w : gone};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if constexpr (sizeof(LT) == 2) {
                    x[2 * k] = __uint_as_float(w[k] << 16) * inv_T;
                    x[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u) * inv_T;
                } else {
                    x[k] = __uint_as_float(w[k]) * inv_T;
                }
            }
        };
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int g = 0; g < kVecs; ++g) {
                unpack(ra[c][g], inside[c][g], xa + c * EPT + g * kPerVec);
                if (TWO) unpack(rb[c][g], inside[c][g], xb + c * EPT + g * kPerVec);
            }
    } else {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float* const xs[2] = {xa + c * EPT, xb + c * EPT};
            const LT* const rows[2] = {row_a, row_b};
#pragma unroll
            for (int w = 0; w < (TWO ? 2 : 1); ++w) {
#pragma unroll 1
                for (int e = 0; e < EPT; ++e) {
                    const int t = base + c * stride + e;
                    const float val = t < V ? load_logit<LT>(rows[w], t) * inv_T : -INFINITY;
#pragma unroll
                    for (int k = 0; k < EPT; ++k) xs[w][k] = k == e ? val : xs[w][k];   // (static register indices)
                }
            }
        }
    }
}
template <typename LT, int EPT>
__device__ __forceinline__ void load_row_slice(const LT* row, int base, int V, float inv_T, bool vec_ok, float* x) {
    load_row_slices<LT, EPT, 1, false>(row, row, base, 0, V, inv_T, vec_ok, x, x);
}

// e^x on the hardware base-2 exponential, with the rounding error of x * log2(e) carried into
// the result (about 2 ulp for the x <= 0 this file feeds it); e^-inf = 0.
__device__ __forceinline__ float exp_fast(float x) {
    constexpr float kLog2e = 1.44269504088896341f;
    constexpr float kLog2eLo = 1.92596299112661746e-8f;  // log2(e) - float(log2(e))
    constexpr float kLn2 = 0.693147180559945309f;
    const float hi = x * kLog2e;
    const float lo = fmaf(x, kLog2e, -hi) + x * kLog2eLo;
    const float e = __builtin_amdgcn_exp2f(hi);
    return x == -INFINITY ? 0.f : fmaf(e, lo * kLn2, e);
}

__device__ __forceinline__ float prob_of(float scaled_logit, float m, float inv_z) {
    return scaled_logit == -INFINITY ? 0.f : exp_fast(scaled_logit - m) * inv_z;
}

__device__ __forceinline__ float residual_of(float p, float q, float a, float b) {
    return fmaxf(fmaf(-a, q, p) - b, 0.f);
}

// ---- wavefront reductions on the data-parallel-primitive path (no LDS round trips) -----------
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
constexpr int kOpSum = 0, kOpMax = 1;
template <int OP> __device__ __forceinline__ float combine(float a, float b) {
    return OP == kOpSum ? a + b : fmaxf(a, b);
}
// every lane of a 16-lane row ends with the row's result
template <int OP> __device__ __forceinline__ float row_reduce(float v) {
    v = combine<OP>(v, dpp<0xB1>(v));   // quad_perm [1,0,3,2]
    v = combine<OP>(v, dpp<0x4E>(v));   // quad_perm [2,3,0,1]
    v = combine<OP>(v, dpp<0x141>(v));  // row_half_mirror
    v = combine<OP>(v, dpp<0x140>(v));  // row_mirror
    return v;
}
// wave-uniform result; all 64 lanes must be active
template <int OP> __device__ __forceinline__ float wave_reduce(float v) {
    v = row_reduce<OP>(v);
    return combine<OP>(combine<OP>(lane_value(v, 0), lane_value(v, 16)),
                       combine<OP>(lane_value(v, 32), lane_value(v, 48)));
}

// ---- Algorithm 2 at one node: the scalar state and its three moves ---------------------------
struct NodeState {
    double A, B, Wn, massQ, dA, dB;
    float af, bf;
    int n_rej, fallback, sums_valid;
    int fallbacks, degenerate;   // event counts (for the trace)
};

__device__ __forceinline__ void node_begin(NodeState& st) {
    st.A = st.B = 0.0;
    st.Wn = st.massQ = 1.0;
    st.af = st.bf = 0.f;
    st.dA = st.dB = 0.0;
    st.n_rej = 0;
    st.fallback = 0;
    st.sums_valid = 0;
}

// The result of the vocabulary pass that follows a rejection: the mass of the new residual's
// numerator and the draft mass that is left.
__device__ __forceinline__ void node_apply_pass(NodeState& st, double w_new, double q_new) {
    if (w_new > 0.0) { st.Wn = w_new; st.sums_valid = 1; }
    else { st.A -= st.dA; st.B -= st.dB; ++st.degenerate; st.sums_valid = 0; }  // R stays as it was
    st.af = (float)st.A;
    st.bf = (float)st.B;
    st.massQ = q_new;
    if (!st.fallback && !(q_new > 0.0)) { st.fallback = 1; ++st.fallbacks; }
}

// The accept test of one child, u < R[s] / D[s], kept free of divisions: the child is accepted
// iff u * lhs < rhs, both sides products of two floats taken in fp64.  ps, qs: target and draft probability of the child's token; in_s: the token
// was already rejected at this node (an earlier sibling carried it).
struct ChildTest {
    float lhs_w, lhs_q, rhs_r, rhs_m;   // lhs = lhs_w * lhs_q, rhs = rhs_r * rhs_m, products in fp64
    __device__ __forceinline__ bool accepts(float u) const {
        return (double)u * (double)lhs_w * (double)lhs_q < (double)rhs_r * (double)rhs_m;
    }
    // R[s] / D[s] as a float, for the trace (infinite where D[s] = 0 < R[s])
    __device__ __forceinline__ float ratio() const {
        if (lhs_w == 0.f) return rhs_r > 0.f ? INFINITY : 0.f;
        return (rhs_r * rhs_m) / (lhs_w * lhs_q);
    }
};
// What a child's test needs of the state before its rejection.
struct TestState {
    float af, bf, Wn, massQ;
    int n_rej, fallback;
};
__device__ __forceinline__ TestState test_state_of(const NodeState& st) {
    return TestState{st.af, st.bf, (float)st.Wn, (float)st.massQ, st.n_rej, st.fallback};
}
__device__ __forceinline__ ChildTest node_test_child(const TestState& st, float ps, float qs, bool in_s, int V) {
    const int left = V - st.n_rej;  // tokens not yet rejected
    const float r_num = in_s ? 0.f : residual_of(ps, qs, st.af, st.bf);   // R[s] * W
    ChildTest t;
    // D[s]: q/massQ, or 1/left once the draft's support is exhausted, or 0 for a rejected token
    if (in_s || (st.fallback ? left <= 0 : !(qs > 0.f))) {
        t.lhs_w = 0.f; t.lhs_q = 1.f;
        t.rhs_r = r_num > 0.f ? 1.f : 0.f; t.rhs_m = 1.f;    // D[s] = 0: accepted iff R[s] > 0
    } else if (st.fallback) {
        t.lhs_w = st.Wn; t.lhs_q = 1.f;
        t.rhs_r = r_num; t.rhs_m = (float)left;              // vocabularies stay far below 2^24
    } else {
        t.lhs_w = st.Wn; t.lhs_q = qs;
        t.rhs_r = r_num; t.rhs_m = st.massQ;
    }
    return t;
}
__device__ __forceinline__ ChildTest node_test_child(const NodeState& st, float ps, float qs, bool in_s, int V) {
    return node_test_child(test_state_of(st), ps, qs, in_s, V);
}

// Rejection: R <- norm(max(R - D, 0)), then D[s] <- 0 (uniform over what is left once the draft
// has no mass).  Only the coefficients move here; the pass over the vocabulary follows.
__device__ __forceinline__ void node_reject_child(NodeState& st, bool in_s, int V, bool keep_draft = false) {
    const int left = V - st.n_rej;
    st.dA = 0.0;
    st.dB = 0.0;
    if (st.fallback) { if (left > 0) st.dB = (double)((float)st.Wn / (float)left); }
    else st.dA = (double)((float)st.Wn / (float)st.massQ);
    st.A += st.dA;
    st.B += st.dB;
    st.af = (float)st.A;
    st.bf = (float)st.B;
    if (!in_s && !keep_draft) ++st.n_rej;
}

// Inverse CDF over 64 consecutive blocks of the vocabulary, one per lane of a wavefront: which
// block holds the cumulative residual mass u * total?  `sw_f` is the mass of block `lane`
// (0 for lanes past `blocks`).  All lanes return the same answer.
struct BlockPick {
    double total, before;   // total mass; mass of the blocks before the owner
    int owner, forced;      // forced: rounding left no block above the goal; take the last token with mass
};

// Cross-lane moves of doubles and ints without LDS round trips.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_or_zero(double v) {   // lanes the move does not reach read 0
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)bits, CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), CTRL, ROW_MASK, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// inclusive prefix sum over the 64 lanes of a wavefront (all lanes active)
__device__ __forceinline__ double wave_scan(double v) {
    v += dpp_or_zero<0x111, 0xF>(v);   // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);   // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);   // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);   // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ double lane_value(double v, int lane) {   // lane: wave-uniform
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)bits, lane);
    const int hi = __builtin_amdgcn_readlane((int)(bits >> 32), lane);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
template <int CTRL>
__device__ __forceinline__ int dpp_int(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ int wave_min(int v) {   // wave-uniform result; all lanes active
    v = min(v, dpp_int<0xB1>(v));
    v = min(v, dpp_int<0x4E>(v));
    v = min(v, dpp_int<0x141>(v));
    v = min(v, dpp_int<0x140>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
__device__ __forceinline__ int wave_max(int v) { return -wave_min(-v); }

// FRACTION: the goal is x times the total mass of these blocks; otherwise x itself (a cumulative
// mass counted from the first block).  `force_last`: take the last block with mass whatever the goal.
template <bool FRACTION>
__device__ __forceinline__ BlockPick pick_block_impl(double x, bool force_last, float sw_f, int blocks) {
    const double sw = (double)sw_f;
    const double incl = wave_scan(sw);
    BlockPick r;
    r.total = lane_value(incl, 63);
    const double goal = FRACTION ? x * r.total : x;
    const unsigned long long hit = force_last ? 0ull : __ballot(sw > 0.0 && incl > goal);
    const unsigned long long pos = __ballot(sw > 0.0);
    r.forced = 0;
    if (hit) r.owner = __ffsll((long long)hit) - 1;
    else { r.forced = 1; r.owner = pos ? 63 - __clzll((long long)pos) : blocks - 1; }
    r.before = lane_value(incl - sw, __builtin_amdgcn_readfirstlane(r.owner));
    return r;
}
__device__ __forceinline__ BlockPick pick_block(float u0, float sw_f, int blocks) {
    return pick_block_impl<true>((double)u0, false, sw_f, blocks);
}
__device__ __forceinline__ BlockPick pick_block_at(double goal, bool force_last, float sw_f, int blocks) {
    return pick_block_impl<false>(goal, force_last, sw_f, blocks);
}

// Layout of the caller's workspace: the trace first (header, one record per accept test, four
// floats about the bonus draw), then what the per-node kernel leaves for the final walk.
constexpr size_t kTraceBytes =
    sizeof(int32_t) * (SEQ_TRACE_HEADER_INTS + (size_t)SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS + 4);
constexpr size_t kTraceBytesPadded = (kTraceBytes + 255) / 256 * 256;
constexpr int kChildRecordWords = 5;   // tagged words per child: the four factors of the test, events
constexpr int kNodeRecordWords = 4;    // tagged words per node: bonus token, total mass, CDF below / above
constexpr size_t kRecordWords = (size_t)SEQ_MAX_TREE * (kChildRecordWords + kNodeRecordWords);
static_assert(kChildRecordWords + kNodeRecordWords == kChainRecordWordsPerNode, "layout of the per-node kernels' area");
constexpr size_t kVerifyWorkspaceBytes = kTraceBytesPadded + sizeof(unsigned long long) * kRecordWords + 256;
// The per-node kernels' area (library-owned, zeroed when created, written by these kernels only):
// the tag epoch, which every workgroup of a launch reads on entry and the last workgroup of the
// launch to finish moves on -- whatever a word of the area holds was written under a smaller tag
// or by this launch; the word a team member that gave up waiting leaves for the workgroup that
// walks; the count of finished workgroups; the records; the teams' exchange slots: per team two
// buffers (by step parity) of kTeamSlotWords x kTeamMaxW tagged words.
constexpr size_t kTeamSlotWordsPerTeam = (size_t)2 * kTeamSlotWords * kTeamMaxW;
static_assert(kTeamSlotWordsPerTeam == kChainSlotWordsPerTeam, "layout of the per-node kernels' area");
__host__ __device__ __forceinline__ uint32_t* chain_epoch_cell(unsigned long long* area) { return reinterpret_cast<uint32_t*>(area); }
__host__ __device__ __forceinline__ unsigned long long* team_fail_cell(unsigned long long* area) { return area + 1; }
__host__ __device__ __forceinline__ uint32_t* chain_finished_cell(unsigned long long* area) { return reinterpret_cast<uint32_t*>(area + 2); }
__host__ __device__ __forceinline__ unsigned long long* chain_records_of(unsigned long long* area) { return area + kChainHeaderWords; }
__host__ __device__ __forceinline__ unsigned long long* team_slots_of(unsigned long long* area) {
    return area + kChainHeaderWords + (size_t)SEQ_MAX_TREE * kChainRecordWordsPerNode;
}

}  // namespace verify
}  // namespace seqtree
