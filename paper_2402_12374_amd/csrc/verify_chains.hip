// seq_verify for vocabularies that fit one workgroup's registers: Algorithm 2 (Sec. 3.2.1) at
// EVERY node of the tree at once, then the walk from the root (Sec. 2.2) over the results.
//
// What Algorithm 2 does at a node is a chain over its children in sampling order: test child j
// against the residual R_j and draft D_j left by the rejections of children 1..j-1.  Only the
// comparison with the child's uniform depends on the random draw; R_j, D_j and so the threshold
// R_j[x_j] / D_j[x_j] depend on the node's two logit rows and its children's tokens alone.  So
// one workgroup per node computes the thresholds of all its children as if each of them were
// rejected, plus the bonus token that would be drawn (with uniforms[0], by inverse CDF) from
// the residual left after the last child -- or from the target distribution itself at a leaf.
// No workgroup waits for another.  The last workgroup to finish then walks the tree: compare
// uniforms with thresholds, follow the first accepted child, emit the bonus token of the node
// where no child is accepted.
//
// A workgroup keeps its node's two rows in registers (4 x 8 consecutive tokens per thread and
// row, first as tempered logits, then as probabilities), so a rejection is one pass over
// registers, one reduction and two workgroup barriers.  Compared with walking lazily (read only
// the rows of visited nodes, all workgroups sharing the vocabulary of one node at a time) this
// reads every row of the tree, 2 * n * V elements at most, but its critical path is one node's
// chain instead of the sum over the visited nodes, with no exchange between workgroups.
//
// Vocabularies beyond one workgroup's registers (TEAM): a node's two rows are shared by a team of
// W workgroups of 512 threads (two of them fit a compute unit), 16384 consecutive tokens each.
// Every vocabulary-wide number of the chain -- the rows' maxima and normalisers, the residual
// and draft mass after a rejection, the residual mass ahead of the bonus draw -- is then one
// all-to-all of the workgroups' partials through tagged 64-bit slots in the workspace; all
// members fold the same partials in the same order and replicate the scalar step, so they reach
// identical decisions without a leader.  Only nodes that have children get a team: a leaf has
// no accept test, and its row is needed only if the walk ends there, in which case the workgroup
// that walks draws the bonus token from that one row itself.
#include "seq_internal.h"
#include "verify_device.h"

namespace seqtree {
namespace verify {
namespace {

constexpr int kChunk = 8;   // consecutive tokens per thread and chunk: token (c * kThreads + tid) * 8 + e

// A team member: 512 threads with 32 tokens of either row each, two members to a compute unit.
// (1024 threads with 8 tokens each -- a quarter of the unrolled code, twice the members per team --
// was measured slower: 27.4 against 25.5 us for a 64-node tree over 128256 tokens.)
constexpr int kTeamThreads = 512;
constexpr int kTeamChunks = 4;
constexpr int kTeamTokens = kTeamChunks * kChunk * kTeamThreads;
constexpr int kLeafBlock = 64 * kChunk;                  // the leaf draw cuts a row in blocks of one wavefront's load
constexpr int kLeafMaxBlocks = SEQ_MAX_VOCAB / kLeafBlock;
static_assert(kLeafMaxBlocks <= SEQ_MAX_TREE, "the leaf draw keeps its per-block numbers where the records were");
static_assert((long long)kTeamMaxW * kTeamTokens >= SEQ_MAX_VOCAB, "team size limit");

struct ChainShared {
    alignas(16) float part[2][16][4];  // per-wavefront partials, double-buffered by step parity
    float block_mass[64];              // residual mass of (chunk, wavefront) blocks, in token order
    float stat[4];                     // (team) offsets and 1/normalisers of the two rows
    float ctl_a, ctl_b;                // coefficients of the residual for the next pass
    int ctl_zero;                      // token whose probabilities the next pass clears (-1: none)
    int ctl_sum_q;                     // the next pass also sums the draft mass that is left
    int ctl_stop;                      // the child before was accepted: the walk leaves this node through it, nothing after it is needed
    int team_fail;                     // (team) a wait for the other members timed out
    NodeState team_ns;                 // (team) the scalar state of thread 0, kept out of its registers
    TestState before[2];               // the state before the rejection of child j, for its accept test (by parity of j)
    BlockPick pick;
    double pick_goal;                  // cumulative residual mass the bonus draw looks for
    int pick_is_mine;                  // (team) the bonus token lies in this member's part of the row
    int bonus_token;
    float bonus_info[3];               // total mass, CDF just below and just above the bonus token
    int last;
    int w_fail;
    int w_path_len, w_n_dec;
    int w_leaf;                        // (team) the walk ended at this leaf, whose bonus token is still to be drawn; -1: none
    union {
        struct {   // the chain: this node's rows at its children's tokens (tempered logits, then probabilities)
            float child_lt[SEQ_MAX_TREE];
            float child_ld[SEQ_MAX_TREE];
            int child_tok[SEQ_MAX_TREE];
            float child_u[SEQ_MAX_TREE];       // the children's uniforms
            unsigned char child_dup[SEQ_MAX_TREE];
        };
        uint32_t w_node[SEQ_MAX_TREE][kNodeRecordWords];   // the final walk (last workgroup only)
    };
    union {
        float w_rec[SEQ_MAX_TREE][kChildRecordWords];   // the chain: records of my children; the walk: of every node
        struct {   // the draw at a leaf, after the walk: offset and mass of every block of its row
            float leaf_b[kLeafMaxBlocks];
            float leaf_z[kLeafMaxBlocks];
        };
    };
    int w_child_start[SEQ_MAX_TREE + 1];
    int w_child_list[SEQ_MAX_TREE];
    float w_uniform[SEQ_MAX_TREE];
    float w_ratio[SEQ_MAX_TREE];
    int w_path[SEQ_MAX_TREE];
    int w_tested[SEQ_MAX_TREE];
    unsigned char w_accept[SEQ_MAX_TREE];
};
static_assert(sizeof(ChainShared) <= 80 * 1024, "two team members share a compute unit's 160 KB");

// Results travel between workgroups as 64-bit words: a 32-bit payload under the tag of this
// launch, written and read with device-scope atomics (which bypass whatever a compute unit or
// an XCD caches privately).  A reader that finds another tag knows the word has not landed yet;
// no memory fence -- on this chip a write-back of the whole L2 -- is needed anywhere.
__device__ __forceinline__ void put(unsigned long long* dst, uint32_t tag, uint32_t payload) {
    __hip_atomic_store(dst, ((unsigned long long)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void put(unsigned long long* dst, uint32_t tag, float payload) {
    put(dst, tag, __float_as_uint(payload));
}
// Bounded wait for a tagged word.  The writer finished before it was counted as arrived, so
// the first poll normally succeeds.
__device__ __forceinline__ bool get(const unsigned long long* src, uint32_t tag, uint32_t limit, uint32_t* payload) {
    for (uint32_t spins = 0;; ++spins) {
        const unsigned long long w = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(w >> 32) == tag) { *payload = (uint32_t)w; return true; }
        if (spins >= limit) { *payload = 0u; return false; }
        __builtin_amdgcn_s_sleep(1);
    }
}

#ifdef SEQTREE_STAMPS
__device__ long long g_chain_stamps[64];
__device__ int g_chain_stamp_count;
__device__ long long g_chain_wg_times[8 * 1024];   // per workgroup: start, rows in registers, chain done, end; rows loaded, own softmax done
__device__ long long g_chain_last[8];   // the workgroup that walks: arrived, records staged, walk done, outputs written
#define CHAIN_LAST(k) do { if (threadIdx.x == 0) g_chain_last[k] = wall_clock64(); } while (0)
#define CHAIN_STAMP_RESET() do { if (blockIdx.x == 0 && threadIdx.x == 0) g_chain_stamp_count = 0; } while (0)
#define CHAIN_WG_TIME(k) do { if (threadIdx.x == 0 && blockIdx.x < 1024) g_chain_wg_times[8 * blockIdx.x + (k)] = wall_clock64(); } while (0)
#define CHAIN_STAMP(id) do { if (blockIdx.x == 0 && threadIdx.x == 0 && g_chain_stamp_count < 31) { \
    g_chain_stamps[2 * g_chain_stamp_count] = (id); g_chain_stamps[2 * g_chain_stamp_count + 1] = wall_clock64(); ++g_chain_stamp_count; } } while (0)
#else
#define CHAIN_STAMP_RESET() do {} while (0)
#define CHAIN_STAMP(id) do {} while (0)
#define CHAIN_WG_TIME(k) do {} while (0)
#define CHAIN_LAST(k) do {} while (0)
#endif

// All-to-all of K floats among the W members of a team, run by the first wavefront only (all 64
// lanes).  mine[k] is this member's value; afterwards lane w < W holds member w's values in
// got[] (other lanes 0).  `buf` is the team's slot buffer for this step's parity: a member can
// be at most one step ahead of the slowest one, because it cannot finish a step without that
// member's contribution.
template <int K>
__device__ __forceinline__ bool team_exchange(unsigned long long* buf, int rank, int W, uint32_t tag, uint32_t limit,
                                              float mine0, float mine1, float mine2, float mine3,
                                              float& got0, float& got1, float& got2, float& got3) {
    // (plain floats, no arrays: an array that the compiler cannot dissolve into registers goes
    // to a per-thread slice of shared memory, whose address needs the workgroup's size, which
    // the kernel would have to fetch from the dispatch packet -- a trip to host memory)
    static_assert(K >= 1 && K <= kTeamSlotWords, "slot words per step");
    const int lane = threadIdx.x;
    // (the buffer's address is the same for all lanes; pinning it to scalar registers here also
    // keeps the per-lane addresses from being worked out ahead of the chain's loop and held in
    // vector registers, of which a team member has none to spare)
    asm volatile("" : "+s"(buf));
    got0 = got1 = got2 = got3 = 0.f;
    if (lane < K) {
        const float v = lane == 0 ? mine0 : lane == 1 ? mine1 : lane == 2 ? mine2 : mine3;
        put(&buf[lane * kTeamMaxW + rank], tag, v);
    }
    bool done = lane >= W;
    uint32_t spins = 0;
    auto look = [&](int k, float& got) __attribute__((always_inline)) {
        const unsigned long long word = __hip_atomic_load(&buf[k * kTeamMaxW + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(word >> 32) != tag) return false;
        got = __uint_as_float((uint32_t)word);
        return true;
    };
    for (;;) {
        if (!done) {
            bool all = look(0, got0);
            if (K > 1) all &= look(1, got1);
            if (K > 2) all &= look(2, got2);
            if (K > 3) all &= look(3, got3);
            done = all;
        }
        if (__all(done)) return true;
        if (++spins > limit) return false;   // bounded wait: every wavefront leaves this loop
        __builtin_amdgcn_s_sleep(1);
    }
}

// Offset of the exponentials of a stretch of a row whose largest logit is raw_max: minus that
// maximum times the slope, rounded to a multiple of 1/256 (so that offsets add and subtract
// exactly); +inf where the stretch holds nothing but -inf.
__device__ __forceinline__ float offset_of(float raw_max, float slope) {
    return raw_max == -INFINITY ? INFINITY : __builtin_rintf(-raw_max * slope * 256.0f) * (1.0f / 256.0f);
}

// The bonus token at a leaf, x ~ softmax(row / T) by inverse CDF with u0, drawn by one workgroup
// from a row it has not seen yet: one sweep leaves offset and mass of every block of 512 tokens
// in shared memory, the first wavefront finds the block that holds the cumulative mass u0 * total
// and reads that block again.  Result in sh.bonus_token and sh.bonus_info.
// offset and mass of one block of 512 tokens, 8 per lane of one wavefront
__device__ __forceinline__ void leaf_block_stats(const float (&x)[kChunk], float slope, int blk, int lane, ChainShared& sh) {
    float m = x[0];
#pragma unroll
    for (int e = 1; e < kChunk; ++e) m = fmaxf(m, x[e]);
    const float b = offset_of(wave_reduce<kOpMax>(m), slope);
    float z = 0.f;
    if (b != INFINITY) {
#pragma unroll
        for (int e = 0; e < kChunk; ++e) z += __builtin_amdgcn_exp2f(fmaf(x[e], slope, b));
    }
    z = wave_reduce<kOpSum>(z);
    if (lane == 0) { sh.leaf_b[blk] = b; sh.leaf_z[blk] = z; }
}

template <typename LT, int NT>
__device__ void leaf_draw(const LT* row, int V, float slope, float u0, bool vec_ok, ChainShared& sh) {
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int blocks = (V + kLeafBlock - 1) / kLeafBlock;
    // (one workgroup against the memory's latency: sixteen 16-byte loads per lane in flight, still
    // packed; an odd vocabulary takes the slow loads, one block at a time)
    constexpr int kPerVec = 16 / (int)sizeof(LT), kVecs = kChunk / kPerVec;
    constexpr int kDeep = 16 / kVecs;
    for (int first = wave; first < blocks; first += NW * kDeep) {
        if (vec_ok) {
            // (a group past the end reads the row's first group and is replaced by -inf afterwards:
            // loads under a condition would go to memory one at a time)
            uint4 raw[kDeep][kVecs];
            bool inside[kDeep][kVecs];
#pragma unroll
            for (int d = 0; d < kDeep; ++d) {
                const int base = (first + d * NW) * kLeafBlock + lane * kChunk;
#pragma unroll
                for (int c = 0; c < kVecs; ++c) {
                    inside[d][c] = base + (c + 1) * kPerVec <= V;
                    raw[d][c] = *reinterpret_cast<const uint4*>(row + (inside[d][c] ? base + c * kPerVec : 0));
                }
            }
            const uint32_t gone = sizeof(LT) == 2 ? 0xFF80FF80u : 0xFF800000u;   // -inf (as a bf16 pair)
#pragma unroll
            for (int d = 0; d < kDeep; ++d) {
                const int blk = first + d * NW;
                if (blk >= blocks) break;
                float x[kChunk];
#pragma unroll
                for (int c = 0; c < kVecs; ++c) {
                    const bool in = inside[d][c];
                    const uint32_t w[4] = {in ? raw[d][c].x : gone, in ? raw[d][c].y : gone, in ? raw[d][c].z : gone, in ? raw[d][c].w : gone};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if constexpr (sizeof(LT) == 2) {
                            x[2 * k] = __uint_as_float(w[k] << 16);
                            x[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
                        } else {
                            x[c * 4 + k] = __uint_as_float(w[k]);
                        }
                    }
                }
                leaf_block_stats(x, slope, blk, lane, sh);
            }
        } else {
#pragma unroll 1
            for (int d = 0; d < kDeep; ++d) {
                const int blk = first + d * NW;
                if (blk >= blocks) break;
                float x[kChunk];
                load_row_slice<LT, kChunk>(row, blk * kLeafBlock + lane * kChunk, V, 1.0f, false, x);
                leaf_block_stats(x, slope, blk, lane, sh);
            }
        }
    }
    __syncthreads();
    if (wave == 0) {
        // lane l looks after `per` consecutive blocks, so that lane order is token order
        const int per = (blocks + 63) / 64;
        const int lo = min(lane * per, blocks), hi = min(lo + per, blocks);
        float bmin = INFINITY;
        for (int blk = lo; blk < hi; ++blk) bmin = fminf(bmin, sh.leaf_b[blk]);
        const float b_row = -wave_reduce<kOpMax>(-bmin);
        double mine = 0.0;
        for (int blk = lo; blk < hi; ++blk) {
            const float b = sh.leaf_b[blk];
            const float m = b != INFINITY ? sh.leaf_z[blk] * __builtin_amdgcn_exp2f(b_row - b) : 0.f;
            sh.leaf_z[blk] = m;
            mine += (double)m;
        }
        const double incl = wave_scan(mine);
        const double total = lane_value(incl, 63);
        const double goal = (double)u0 * total;
        const unsigned long long hit = __ballot(mine > 0.0 && incl > goal);
        const unsigned long long pos = __ballot(mine > 0.0);
        const int owner_lane = hit ? __ffsll((long long)hit) - 1 : pos ? 63 - __clzll((long long)pos) : 0;
        if (lane == owner_lane) {
            double run = incl - mine, before = run;
            int found = -1, last = -1;
            double last_before = run;
            for (int blk = lo; blk < hi; ++blk) {
                const double m = (double)sh.leaf_z[blk];
                if (hit && found < 0 && m > 0.0 && run + m > goal) { found = blk; before = run; }
                if (m > 0.0) { last = blk; last_before = run; }
                run += m;
            }
            BlockPick b;
            b.total = total;
            b.forced = found < 0;
            b.owner = found >= 0 ? found : max(last, 0);
            b.before = found >= 0 ? before : last_before;
            sh.pick = b;
            sh.pick_goal = goal;
            sh.stat[0] = b_row;
            sh.bonus_token = -1;
        }
    }
    __syncthreads();
    if (wave == 0) {
        const BlockPick b = sh.pick;
        const double goal = sh.pick_goal;
        const int base = b.owner * kLeafBlock + lane * kChunk;
        float x[kChunk];
        load_row_slice<LT, kChunk>(row, base, V, 1.0f, vec_ok, x);
        const float bb = sh.leaf_b[b.owner];
        const float f = bb != INFINITY ? __builtin_amdgcn_exp2f(sh.stat[0] - bb) : 0.f;
        float r[kChunk];
        double mine = 0.0;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            r[e] = bb != INFINITY ? __builtin_amdgcn_exp2f(fmaf(x[e], slope, bb)) * f : 0.f;
            mine += (double)r[e];
        }
        const double incl = wave_scan(mine);
        double run = b.before + incl - mine;
        int found = 0x7FFFFFFF, last_pos = -1;
        double lo = 0.0, hi = 0.0;
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
            const double prev = run;
            run += (double)r[e];
            if (found == 0x7FFFFFFF && !b.forced && run > goal) { found = base + e; lo = prev; hi = run; }
            if (r[e] > 0.f) last_pos = base + e;
        }
        const int wave_found = wave_min(found), wave_last = wave_max(last_pos);
        if (wave_found != 0x7FFFFFFF) {
            if (found == wave_found) {
                sh.bonus_token = found;
                sh.bonus_info[0] = (float)b.total;
                sh.bonus_info[1] = (float)(lo / b.total);
                sh.bonus_info[2] = (float)(hi / b.total);
            }
        } else if (lane == 0) {
            sh.bonus_token = wave_last >= 0 ? wave_last : min(V - 1, b.owner * kLeafBlock);
            sh.bonus_info[0] = (float)b.total;
            sh.bonus_info[1] = 1.f;
            sh.bonus_info[2] = 1.f;
        }
    }
    __syncthreads();
}

// Moving the tag epoch on for the next launch, after every workgroup of this one has read it.
// One sequence per launch: every workgroup reads the epoch before it does anything else, and the
// workgroup that walks runs only after all of them have been counted as arrived, so it can move
// the epoch itself, without waiting for the answer.  Several sequences per launch: a sequence's
// walk may be over before a workgroup of another sequence has started, so every workgroup of
// the launch passes through a count of its own when it is done, and the last one moves the epoch.
template <bool BATCHED>
__device__ __forceinline__ void launch_member_done(const VerifyParams& p, bool walked) {
    if (threadIdx.x != 0) return;
    if constexpr (!BATCHED) {
        if (walked)
            __hip_atomic_fetch_add(chain_epoch_cell(p.chain_area), (uint32_t)kVerifyTagsPerCall, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        uint32_t* const finished = chain_finished_cell(p.chain_area);
        const uint32_t total = gridDim.x * gridDim.y;
        if (__hip_atomic_fetch_add(finished, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == total - 1u) {
            __hip_atomic_store(finished, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_add(chain_epoch_cell(p.chain_area), (uint32_t)kVerifyTagsPerCall, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <typename LT, int CH, bool BATCHED, int TEAM_NT>   // TEAM_NT: threads of a team member, 0: no teams
__global__ __launch_bounds__(TEAM_NT ? TEAM_NT : kThreads, 4) void verify_chains_kernel(const VerifyParams p_in) {
    constexpr bool TEAM = TEAM_NT > 0;
    static_assert(!(TEAM && BATCHED), "teams serve one sequence");
    constexpr int NT = TEAM ? TEAM_NT : kThreads;   // threads of this workgroup
    constexpr int NW = NT / 64;
    const VerifyParams p = BATCHED ? params_of_sequence(p_in, blockIdx.y, false) : p_in;
    __shared__ ChainShared sh;
    constexpr int EPT = CH * kChunk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = p.V;
    // which node, and which part of its rows
    int v = blockIdx.x, rank = 0, team = 0;
    const int W = TEAM ? p.W : 1;
    if constexpr (TEAM) {
        const int b = blockIdx.x;
        if (p.team_xcd) {   // workgroup b runs on XCD b % 8: the members of a team share one
            const int i = b >> 3;
            team = (i / W) * 8 + (b & 7);
            rank = i % W;
        } else {
            team = b / W;
            rank = b % W;
        }
        if (team >= p.n_internal) {   // (the grid is rounded up to whole groups of 8 teams)
            launch_member_done<BATCHED>(p, false);
            return;
        }
        v = p.internal_nodes[team];
    }
    const int row_base = rank * (EPT * NT);   // my first token
    const LT* trow = static_cast<const LT*>(p.target) + (size_t)v * V;
    const LT* drow = static_cast<const LT*>(p.draft) + (size_t)v * V;
    const int c_begin = p.child_start[v], c_end = p.child_start[v + 1];
    const int K = c_end - c_begin;
    unsigned long long* const child_rec = p.chain_records;                                    // [n][kChildRecordWords]
    unsigned long long* const node_rec = p.chain_records + (size_t)p.n * kChildRecordWords;   // [n][kNodeRecordWords]
    // Tag of this launch: every workgroup reads the area's epoch on entry, and the last workgroup
    // of the launch to finish moves it on -- after all have read it.  (A team's exchange number s
    // carries tag + s.)
    uint32_t* const epoch = chain_epoch_cell(p.chain_area);
    const uint32_t tag = __hip_atomic_load(epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
    unsigned long long* const my_slots = TEAM ? p.team_slots + (size_t)team * kTeamSlotWordsPerTeam : nullptr;
    uint32_t step = 0;
    auto slot_buf = [&](uint32_t s) __attribute__((always_inline)) {
        return my_slots + (size_t)(s & 1u) * kTeamSlotWords * kTeamMaxW;
    };
    CHAIN_STAMP_RESET();
    CHAIN_STAMP(0);
    CHAIN_WG_TIME(0);
    const bool vec_ok = (V % (16 / (int)sizeof(LT)) == 0) &&
                        ((reinterpret_cast<uintptr_t>(p.target) | reinterpret_cast<uintptr_t>(p.draft)) & 15) == 0;
    float pr[EPT], qr[EPT];
    if (K > 0) {
        load_row_slices<LT, kChunk, CH, true>(trow, drow, row_base + tid * kChunk, NT * kChunk, V, 1.0f, vec_ok, pr, qr);
    } else {
        load_row_slices<LT, kChunk, CH, false>(trow, trow, row_base + tid * kChunk, NT * kChunk, V, 1.0f, vec_ok, pr, pr);
#pragma unroll
        for (int e = 0; e < EPT; ++e) qr[e] = -INFINITY;   // a leaf has no draft row to read
    }
    // both rows at the children's tokens, in flight together with the rows themselves
    // (up to 64 children: a lane of the first wavefront per child, so that "an earlier sibling has
    // the same token" is a walk over lanes, not over memory)
    if (K > 64) {
        for (int k = tid; k < K; k += NT) {
            const int s = min(max(p.tokens[p.child_list[c_begin + k]], 0), V - 1);
            sh.child_tok[k] = s;
            sh.child_u[k] = p.uniforms[p.child_list[c_begin + k]];
            sh.child_lt[k] = load_logit<LT>(trow, s);
            sh.child_ld[k] = load_logit<LT>(drow, s);
            bool dup = false;
            for (int j = 0; j < k; ++j) dup |= min(max(p.tokens[p.child_list[c_begin + j]], 0), V - 1) == s;
            sh.child_dup[k] = dup ? 1 : 0;
        }
    } else if (tid < 64 && K > 0) {
        const int k = tid;
        const int child = p.child_list[c_begin + min(k, K - 1)];
        const int s = min(max(p.tokens[child], 0), V - 1);  // stay inside the row
        const float u = p.uniforms[child];
        const float lt = load_logit<LT>(trow, s);   // raw: the temperature is in the exponent's slope
        const float ld = load_logit<LT>(drow, s);
        bool dup = false;
        for (int j = 0; j < K - 1; ++j) dup |= j < k && __builtin_amdgcn_readlane(s, j) == s;
        if (k < K) {
            sh.child_tok[k] = s;
            sh.child_u[k] = u;
            sh.child_lt[k] = lt;
            sh.child_ld[k] = ld;
            sh.child_dup[k] = dup ? 1 : 0;
        }
    }
    if (TEAM && tid == 0) sh.team_fail = 0;
#ifdef SEQTREE_STAMPS
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    CHAIN_WG_TIME(4);
#endif

    // ---- softmax of both rows: per wavefront first, then folded by everybody ------------------
    // The bulk of the vocabulary goes through the bare hardware exponential, one fused
    // multiply-add and one v_exp_f32 per token: p ~ 2^(x * slope + b), slope = log2(e) / T.  The
    // product is exact inside the multiply-add, so what matters is b: it stands for minus the
    // wavefront's maximum times slope, and if it were that product rounded to a float, every
    // wavefront would scale its tokens by its own factor 1 +- 1e-6 that the later rescaling knows
    // nothing of -- an error that the accept ratios, which subtract nearly equal numbers when the
    // drafter is good, magnify several times.  So b is rounded to a multiple of 1/256 instead:
    // sums and differences of such offsets are exact, the reference is merely not quite the
    // maximum (values reach 2^(1/256) at most).  The probabilities that decide an accept test
    // (the children's tokens) take the same offsets with a compensated product and exponential.
    constexpr float kLog2e = 1.44269504088896341f;
    const float slope = p.inv_T * kLog2e;
    float mt_wave = -INFINITY, md_wave = -INFINITY;
#pragma unroll
    for (int e = 0; e < EPT; ++e) { mt_wave = fmaxf(mt_wave, pr[e]); md_wave = fmaxf(md_wave, qr[e]); }
    const float bt_wave = offset_of(wave_reduce<kOpMax>(mt_wave), slope);   // +inf: nothing but -inf in my part of the row
    const float bd_wave = offset_of(wave_reduce<kOpMax>(md_wave), slope);
    {
        const float bt = bt_wave == INFINITY ? 0.f : bt_wave;
        const float bd = bd_wave == INFINITY ? 0.f : bd_wave;
        float zt = 0.f, zd = 0.f;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            pr[e] = __builtin_amdgcn_exp2f(fmaf(pr[e], slope, bt));
            qr[e] = __builtin_amdgcn_exp2f(fmaf(qr[e], slope, bd));
            zt += pr[e];
            zd += qr[e];
        }
        zt = wave_reduce<kOpSum>(zt);
        zd = wave_reduce<kOpSum>(zd);
        if (lane == 0) { sh.part[0][wave][0] = bt_wave; sh.part[0][wave][1] = zt; sh.part[0][wave][2] = bd_wave; sh.part[0][wave][3] = zd; }
    }
    __syncthreads();
    CHAIN_STAMP(1);
    CHAIN_WG_TIME(5);
    float bt_row, bd_row, inv_zt, inv_zd;   // offsets of the rows (those of the wavefronts with the largest maxima)
    {
        // every wavefront folds the same per-wavefront partials in the same order: identical results
        // (a team: only the first wavefront, which then trades the workgroup's numbers for the others')
        const int w = lane & 15;
        const bool have = w < NW;
        const float4 part_w = *reinterpret_cast<const float4*>(sh.part[0][w]);   // (rows past NW: never written, never used)
        const float bt_w = have ? part_w.x : INFINITY, zt_w = have ? part_w.y : 0.f;
        const float bd_w = have ? part_w.z : INFINITY, zd_w = have ? part_w.w : 0.f;
        bt_row = -lane_value(row_reduce<kOpMax>(-bt_w), 0);
        bd_row = -lane_value(row_reduce<kOpMax>(-bd_w), 0);
        // (bt_row - bt_w is an exact multiple of 1/256, at most 0: the hardware exponential of it
        // is the same number wherever it is taken)
        float zt = lane_value(row_reduce<kOpSum>(bt_w != INFINITY ? zt_w * __builtin_amdgcn_exp2f(bt_row - bt_w) : 0.f), 0);
        float zd = lane_value(row_reduce<kOpSum>(bd_w != INFINITY ? zd_w * __builtin_amdgcn_exp2f(bd_row - bd_w) : 0.f), 0);
        if constexpr (TEAM) {
            ++step;
            if (wave == 0) {
                float got_bt, got_zt, got_bd, got_zd;
                CHAIN_WG_TIME(6);
                const bool ok = team_exchange<4>(slot_buf(step), rank, W, tag + step, p.spin_limit, bt_row, zt, bd_row, zd,
                                                 got_bt, got_zt, got_bd, got_zd);
                CHAIN_WG_TIME(7);
                const bool member = lane < W;
                bt_row = -wave_reduce<kOpMax>(member ? -got_bt : -INFINITY);
                bd_row = -wave_reduce<kOpMax>(member ? -got_bd : -INFINITY);
                zt = wave_reduce<kOpSum>(member && got_bt != INFINITY ? got_zt * __builtin_amdgcn_exp2f(bt_row - got_bt) : 0.f);
                zd = wave_reduce<kOpSum>(member && got_bd != INFINITY ? got_zd * __builtin_amdgcn_exp2f(bd_row - got_bd) : 0.f);
                if (lane == 0) {
                    sh.stat[0] = bt_row; sh.stat[1] = bd_row; sh.stat[2] = 1.0f / zt; sh.stat[3] = 1.0f / zd;
                    if (!ok) sh.team_fail = 1;
                }
            }
            __syncthreads();
            bt_row = sh.stat[0]; bd_row = sh.stat[1]; inv_zt = sh.stat[2]; inv_zd = sh.stat[3];
        } else {
            inv_zt = 1.0f / zt;
            inv_zd = 1.0f / zd;
        }
        const float ft = bt_wave == INFINITY ? 0.f : __builtin_amdgcn_exp2f(bt_row - bt_wave) * inv_zt;
        const float fd = bd_wave == INFINITY ? 0.f : __builtin_amdgcn_exp2f(bd_row - bd_wave) * inv_zd;
#pragma unroll
        for (int e = 0; e < EPT; ++e) { pr[e] *= ft; qr[e] *= fd; }
    }
    // the children's logits become probabilities in the first wavefront, whose first lane is
    // their only reader: no barrier needed
    if (wave == 0) {
        auto exact_prob = [&](float raw, float b_row, float inv_z) __attribute__((always_inline)) {
            // 2^(raw * slope + b_row) / z with the rounding errors of the product and of the sum
            // carried into the result
            if (raw == -INFINITY || b_row == INFINITY) return 0.f;
            const float hi = raw * slope;
            const float lo = fmaf(raw, slope, -hi);
            const float sum = hi + b_row;
            const float bb = sum - hi;
            const float err = (hi - (sum - bb)) + (b_row - bb);
            const float e2 = __builtin_amdgcn_exp2f(sum);
            return fmaf(e2, (lo + err) * 0.693147180559945309f, e2) * inv_z;
        };
        for (int k = lane; k < K; k += 64) {
            sh.child_lt[k] = exact_prob(sh.child_lt[k], bt_row, inv_zt);
            sh.child_ld[k] = exact_prob(sh.child_ld[k], bd_row, inv_zd);
        }
    }
    CHAIN_STAMP(2);
    CHAIN_WG_TIME(1);

    // ---- the chain: children in order, each taken as rejected ---------------------------------
    // Two wavefronts share the scalar work (in a team: of every member, all taking the same steps
    // on the same numbers).  The first owns the state: at the top of iteration j its thread 0
    // applies the pass that followed child j-1, rejects child j and publishes the coefficients
    // of the next pass -- the only thing everybody waits for.  The second works out, at the same
    // time, the accept test of child j-1 from the state the first left before rejecting it, and
    // writes that child's record.  The uniforms are inputs: if that test accepts, the walk will
    // leave this node through child j-1 and never look at the later children or at this node's
    // bonus token, so the chain ends here (the step the first wavefront took beside it is
    // dropped).  Iteration K only closes child K-1.
    //
    // The draft mass left after a rejection is the mass before it minus the rejected token's: as
    // long as a twentieth of the mass is left, thread 0 takes that difference (in fp64; its error
    // is that of the initial normalisation, 1e-7 absolute) and the pass skips the sum over q.  Once
    // less is left the pass sums q again, which is also what finds the mass exactly zero.
    // (a team member has fewer registers to spare: its thread 0 keeps the state in shared memory)
    NodeState ns_regs;
    NodeState& ns = TEAM ? sh.team_ns : ns_regs;
    bool stopped = false;
    bool failed = TEAM && __builtin_amdgcn_readfirstlane(sh.team_fail) != 0;
    uint32_t events = 0;
    double q_predicted = 1.0;
    bool q_summed = true;
    if (tid == 0) { node_begin(ns); ns.fallbacks = 0; ns.degenerate = 0; sh.ctl_stop = 0; }
    int par = 1;
    for (int j = 0, j_end = failed ? -1 : K; j <= j_end; ++j) {
        if (TEAM && j > 0) ++step;
        if (wave == 0) {
            // what the step needs of child j, asked for together with the partials
            const int tok_j = j < K ? sh.child_tok[j] : 0;
            const float qs_j = j < K ? sh.child_ld[j] : 0.f;
            const bool dup_j = j < K && sh.child_dup[j] != 0;
            // lanes 0..15 read the per-wavefront partials (the other rows repeat them)
            const bool have = (lane & 15) < NW;
            const float2 part_w = *reinterpret_cast<const float2*>(sh.part[par ^ 1][lane & 15]);
            float w_new = lane_value(row_reduce<kOpSum>(have ? part_w.x : 0.f), 0);
            float q_new = lane_value(row_reduce<kOpSum>(have ? part_w.y : 0.f), 0);
            if constexpr (TEAM) {
                if (j > 0) {   // the pass that followed child j-1: everybody's share of the two masses
                    float got_w, got_q, unused2, unused3;
                    const bool ok = team_exchange<2>(slot_buf(step), rank, W, tag + step, p.spin_limit, w_new, q_new, 0.f, 0.f,
                                                     got_w, got_q, unused2, unused3);
                    w_new = wave_reduce<kOpSum>(got_w);
                    q_new = wave_reduce<kOpSum>(got_q);
                    if (!ok && lane == 0) sh.team_fail = 1;
                }
            }
            if (tid == 0) {
                if (j > 0) {
                    const int fb = ns.fallbacks, dg = ns.degenerate;
                    node_apply_pass(ns, (double)w_new, q_summed ? (double)q_new : q_predicted);
                    events = (uint32_t)(ns.fallbacks - fb) | ((uint32_t)(ns.degenerate - dg) << 1);
                }
                if (j < K) {
                    sh.before[j & 1] = test_state_of(ns);
                    // (SpecInfer: the draft distribution stays what it was -- nothing is struck out)
                    const bool in_s = !p.with_replacement && dup_j;
                    const bool strike = !in_s && !p.with_replacement;
                    node_reject_child(ns, in_s, V, p.with_replacement != 0);
                    sh.ctl_zero = strike ? tok_j : -1;
                    q_predicted = ns.massQ - (strike ? (double)qs_j : 0.0);
                    q_summed = ns.fallback || !(q_predicted >= 0.05);
                    sh.ctl_sum_q = q_summed ? 1 : 0;
                }
                sh.ctl_a = ns.af;
                sh.ctl_b = ns.bf;
            }
        } else if (tid == 64 && j > 0) {
            const int c = j - 1;
            const ChildTest t = node_test_child(sh.before[c & 1], sh.child_lt[c], sh.child_ld[c],
                                                !p.with_replacement && sh.child_dup[c] != 0, V);
            sh.w_rec[c][0] = t.lhs_w; sh.w_rec[c][1] = t.lhs_q;
            sh.w_rec[c][2] = t.rhs_r; sh.w_rec[c][3] = t.rhs_m;
            sh.ctl_stop = t.accepts(sh.child_u[c]) ? 1 : 0;
        }
        __syncthreads();
        CHAIN_STAMP(10);
        // (one way out of the loop for both reasons: every exit keeps a copy of the rows alive)
        if (const int stop = __builtin_amdgcn_readfirstlane(sh.ctl_stop) | (TEAM ? __builtin_amdgcn_readfirstlane(sh.team_fail) << 1 : 0)) {
            if (TEAM && (stop & 2)) {   // a member is missing: the team gives up
                failed = true;
            } else {
                // child j-1 was accepted: no rejection followed it, the children after it are never looked at
                if (tid == 0) sh.w_rec[j - 1][4] = 0.f;
                for (int k = j + tid; k < K; k += NT) {
#pragma unroll
                    for (int w = 0; w < kChildRecordWords; ++w) sh.w_rec[k][w] = 0.f;   // 0 < 0: never accepted
                }
                stopped = true;
            }
            break;
        }
        // records wait in shared memory; they leave together once the chain is done
        if (tid == 0 && j > 0) sh.w_rec[j - 1][4] = __uint_as_float(events);
        if (j == K) break;
        const float af = sh.ctl_a, bf = sh.ctl_b;
        // the rejected token leaves both distributions: only the wavefront that holds it looks
        const int zero_local = sh.ctl_zero >= 0 ? sh.ctl_zero - row_base : -1;   // (below 0 or past my part: not mine)
        if (zero_local >= 0 && zero_local < EPT * NT && ((zero_local / kChunk) % NT) / 64 == wave) {
            const int slot = (zero_local / (kChunk * NT)) * kChunk + zero_local % kChunk;
            if ((zero_local / kChunk) % NT == tid) {
#pragma unroll
                for (int e = 0; e < EPT; ++e)
                    if (e == slot) { pr[e] = 0.f; qr[e] = 0.f; }
            }
        }
        float r_loc = 0.f, q_loc = 0.f;
        // (p - A q never exceeds p <= 1, so the maximum with 0 is a clamp to [0, 1], which rides on
        // the multiply-add as an output modifier)
        if (bf == 0.f && !sh.ctl_sum_q) {   // the common pass: two instructions per token
#pragma unroll
            for (int e = 0; e < EPT; ++e) r_loc += __builtin_amdgcn_fmed3f(fmaf(-af, qr[e], pr[e]), 0.f, 1.f);
        } else if (bf == 0.f) {   // B only moves once the draft has run out of mass
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                r_loc += __builtin_amdgcn_fmed3f(fmaf(-af, qr[e], pr[e]), 0.f, 1.f);
                q_loc += qr[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                r_loc += residual_of(pr[e], qr[e], af, bf);
                q_loc += qr[e];
            }
        }
        r_loc = wave_reduce<kOpSum>(r_loc);
        q_loc = wave_reduce<kOpSum>(q_loc);
        if (lane == 0) { sh.part[par][wave][0] = r_loc; sh.part[par][wave][1] = q_loc; }
        par ^= 1;
        __syncthreads();
        CHAIN_STAMP(11);
    }

    // ---- the bonus token this node would emit: x ~ R by inverse CDF with uniforms[0] ----------
    bool writes_node_record = !TEAM || rank == 0;   // a team: the member that holds the bonus token
    if (failed) {
        // nothing to report but the failure
    } else if (stopped) {   // the walk goes on through the accepted child: no token is drawn here
        if (tid == 0) { sh.bonus_token = -1; sh.bonus_info[0] = sh.bonus_info[1] = sh.bonus_info[2] = 0.f; }
        __syncthreads();
    } else {
        const float af = sh.ctl_a, bf = sh.ctl_b;
        const float u0 = p.uniforms[0];
        float mass[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float m = 0.f;
#pragma unroll
            for (int e = 0; e < kChunk; ++e) m += residual_of(pr[c * kChunk + e], qr[c * kChunk + e], af, bf);
            mass[c] = m;
            const float wm = wave_reduce<kOpSum>(m);
            if (lane == 0) sh.block_mass[c * NW + wave] = wm;
        }
        __syncthreads();
        if (TEAM) ++step;
        if (wave == 0) {
            const float sw = lane < CH * NW ? sh.block_mass[lane] : 0.f;
            if constexpr (TEAM) {
                // which member holds the cumulative mass u0 * total, then which of its blocks
                float got_mass, unused1, unused2, unused3;
                const bool ok = team_exchange<1>(slot_buf(step), rank, W, tag + step, p.spin_limit,
                                                 (float)lane_value(wave_scan((double)sw), 63), 0.f, 0.f, 0.f,
                                                 got_mass, unused1, unused2, unused3);
                const BlockPick members = pick_block(u0, lane < W ? got_mass : 0.f, W);
                const double goal = (double)u0 * members.total;
                const bool is_mine = members.owner == rank;
                BlockPick b = pick_block_at(goal - members.before, members.forced != 0, sw, CH * NW);
                b.before += members.before;
                b.total = members.total;
                if (lane == 0) {
                    sh.pick = b; sh.pick_goal = goal; sh.pick_is_mine = is_mine ? 1 : 0; sh.bonus_token = -1;
                    if (!ok) sh.team_fail = 1;
                }
            } else {
                const BlockPick b = pick_block(u0, sw, CH * NW);
                if (lane == 0) { sh.pick = b; sh.pick_goal = (double)u0 * b.total; sh.pick_is_mine = 1; sh.bonus_token = -1; }
            }
        }
        __syncthreads();
        const BlockPick b = sh.pick;
        if (TEAM && __builtin_amdgcn_readfirstlane(sh.team_fail)) failed = true;
        writes_node_record = __builtin_amdgcn_readfirstlane(sh.pick_is_mine) != 0;
        if (!failed && writes_node_record && wave == b.owner % NW) {
            const int cs = b.owner / NW;
            float mine_f = mass[0];
#pragma unroll
            for (int c = 1; c < CH; ++c) mine_f = c == cs ? mass[c] : mine_f;
            const double mine = (double)mine_f;
            const double incl = wave_scan(mine);
            const double goal = sh.pick_goal;
            const int base = row_base + (cs * NT + tid) * kChunk;
            double run = b.before + incl - mine;
            int found = 0x7FFFFFFF, last_pos = -1;
            double lo = 0.0, hi = 0.0;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                if (c != cs) continue;
#pragma unroll
                for (int e = 0; e < kChunk; ++e) {
                    const float r = residual_of(pr[c * kChunk + e], qr[c * kChunk + e], af, bf);
                    const double prev = run;
                    run += (double)r;
                    if (found == 0x7FFFFFFF && !b.forced && run > goal) { found = base + e; lo = prev; hi = run; }
                    if (r > 0.f) last_pos = base + e;
                }
            }
            const int wave_found = wave_min(found), wave_last = wave_max(last_pos);
            if (wave_found != 0x7FFFFFFF) {
                if (found == wave_found) {
                    sh.bonus_token = found;
                    sh.bonus_info[0] = (float)b.total;
                    sh.bonus_info[1] = (float)(lo / b.total);
                    sh.bonus_info[2] = (float)(hi / b.total);
                }
            } else if (lane == 0) {
                sh.bonus_token = wave_last >= 0 ? wave_last : min(V - 1, row_base + (cs * NT + wave * 64) * kChunk);
                sh.bonus_info[0] = (float)b.total;
                sh.bonus_info[1] = 1.f;
                sh.bonus_info[2] = 1.f;
            }
        }
        __syncthreads();
    }
    CHAIN_STAMP(30);
    CHAIN_WG_TIME(2);

    // ---- hand over, and see whether everybody else is done ------------------------------------
    if (!failed && (!TEAM || rank == 0)) {
        for (int k = tid; k < K; k += NT) {
            unsigned long long* rec = child_rec + (size_t)p.child_list[c_begin + k] * kChildRecordWords;
#pragma unroll
            for (int w = 0; w < kChildRecordWords; ++w) put(rec + w, tag, sh.w_rec[k][w]);
        }
    }
    __syncthreads();   // all records are on their way before this workgroup counts as arrived
    if (tid == 0) {
        if (failed) {
            put(team_fail_cell(p.chain_area), tag, 1u);
        } else if (writes_node_record) {
            unsigned long long* rec = node_rec + (size_t)v * kNodeRecordWords;
            put(rec + 0, tag, (uint32_t)sh.bonus_token);
            put(rec + 1, tag, sh.bonus_info[0]);
            put(rec + 2, tag, sh.bonus_info[1]);
            put(rec + 3, tag, sh.bonus_info[2]);
        }
        CHAIN_STAMP(40);
        const uint32_t expected = TEAM ? (uint32_t)(p.n_internal * W) : (uint32_t)p.n;
        const uint32_t arrived = __hip_atomic_fetch_add(p.arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = arrived == expected - 1u;
        if (last) __hip_atomic_store(p.arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
        sh.last = last;
        sh.w_fail = 0;
        if (TEAM && last) {
            const unsigned long long w = __hip_atomic_load(team_fail_cell(p.chain_area), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((uint32_t)(w >> 32) == tag) sh.w_fail = 1;
        }
    }
    __syncthreads();
    CHAIN_STAMP(41);
    CHAIN_WG_TIME(3);
    if (!sh.last) {
        launch_member_done<BATCHED>(p, false);
        return;
    }
    CHAIN_LAST(0);

    // ---- the walk (Sec. 2.2: Algorithm 2 applied recursively from the root) -------------------
    // (after a failure nobody waits for records that will not come)
    const uint32_t patience = sh.w_fail ? 0u : p.spin_limit;
    __syncthreads();   // everybody has read w_fail before anybody raises it
    for (int i = tid; i < p.n; i += NT) {
        sh.w_child_start[i] = p.child_start[i];
        sh.w_uniform[i] = p.uniforms[i];
        if (i < p.n - 1) sh.w_child_list[i] = p.child_list[i];
        bool ok = true;
        if (i > 0) {
            const unsigned long long* rec = child_rec + (size_t)i * kChildRecordWords;
            unsigned long long w[kChildRecordWords];
#pragma unroll
            for (int k = 0; k < kChildRecordWords; ++k)
                w[k] = __hip_atomic_load(rec + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int k = 0; k < kChildRecordWords; ++k) {
                uint32_t payload = (uint32_t)w[k];
                if ((uint32_t)(w[k] >> 32) != tag) ok = ok && get(rec + k, tag, patience, &payload);
                sh.w_rec[i][k] = __uint_as_float(payload);
            }
        }
        // (a team: leaves have no record; what the walk needs of them it works out itself)
        if (!TEAM || p.child_start[i + 1] > p.child_start[i]) {
            const unsigned long long* rec = node_rec + (size_t)i * kNodeRecordWords;
            unsigned long long w[kNodeRecordWords];
#pragma unroll
            for (int k = 0; k < kNodeRecordWords; ++k)
                w[k] = __hip_atomic_load(rec + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int k = 0; k < kNodeRecordWords; ++k) {
                uint32_t payload = (uint32_t)w[k];
                if ((uint32_t)(w[k] >> 32) != tag) ok = ok && get(rec + k, tag, patience, &payload);
                sh.w_node[i][k] = payload;
            }
        }
        if (!ok) sh.w_fail = 1;
    }
    if (tid == 0) sh.w_child_start[p.n] = p.child_start[p.n];
    __syncthreads();
    CHAIN_STAMP(42);
    CHAIN_LAST(1);
    // every accept test of the tree at once; the walk itself only follows pointers
    for (int c = 1 + tid; c < p.n; c += NT) {
        ChildTest t;
        t.lhs_w = sh.w_rec[c][0]; t.lhs_q = sh.w_rec[c][1]; t.rhs_r = sh.w_rec[c][2]; t.rhs_m = sh.w_rec[c][3];
        sh.w_accept[c] = t.accepts(sh.w_uniform[c]) ? 1 : 0;
        sh.w_ratio[c] = t.ratio();
    }
    __syncthreads();
    if (wave == 0) {
        // one node per step: a lane per child (64 at a time), the first accepted one is followed
        int cur = 0, path_len = 0, n_dec = 0, fallbacks = 0, degenerate = 0;
        for (;;) {
            const int c_lo = sh.w_child_start[cur], c_hi = sh.w_child_start[cur + 1];
            int next = -1;
            for (int b = c_lo; b < c_hi && next < 0; b += 64) {
                const bool have = b + lane < c_hi;
                const int c = have ? sh.w_child_list[b + lane] : 0;
                const bool acc = have && sh.w_accept[c] != 0;
                const uint32_t events = have ? __float_as_uint(sh.w_rec[c][4]) : 0u;
                const unsigned long long acc_mask = __ballot(acc);
                const int first = acc_mask ? __ffsll((long long)acc_mask) - 1 : 64;
                const int tested = acc_mask ? first + 1 : min(64, c_hi - b);
                const unsigned long long rejected = first >= 64 ? ~0ull : (1ull << first) - 1ull;
                if (lane < tested) sh.w_tested[n_dec + lane] = c;
                fallbacks += __popcll(__ballot((events & 1u) != 0u) & rejected);
                degenerate += __popcll(__ballot((events & 2u) != 0u) & rejected);
                n_dec += tested;
                if (acc_mask) next = __builtin_amdgcn_readlane(c, __builtin_amdgcn_readfirstlane(first));
            }
            if (next < 0) break;
            if (lane == 0) sh.w_path[path_len] = next;
            ++path_len;
            cur = next;
        }
        if (lane == 0) {
            const bool at_leaf = sh.w_child_start[cur + 1] == sh.w_child_start[cur];
            if (TEAM && at_leaf) {
                sh.w_leaf = cur;   // the bonus token is still to be drawn, from the leaf's own row
            } else {
                const uint32_t* nr = sh.w_node[cur];
                sh.w_leaf = -1;
                sh.bonus_token = (int32_t)nr[0];
                sh.bonus_info[0] = __uint_as_float(nr[1]);
                sh.bonus_info[1] = __uint_as_float(nr[2]);
                sh.bonus_info[2] = __uint_as_float(nr[3]);
            }
            p.trace[0] = n_dec;
            p.trace[2] = cur;
            p.trace[3] = fallbacks;
            p.trace[4] = degenerate;
            p.trace[5] = p.trace[6] = p.trace[7] = 0;
            sh.w_path_len = path_len;
            sh.w_n_dec = n_dec;
        }
    }
    __syncthreads();
    for (int i = tid; i < p.n; i += NT) p.path[i] = i < sh.w_path_len ? sh.w_path[i] : -1;
    for (int k = tid; k < sh.w_n_dec; k += NT) {
        const int c = sh.w_tested[k];
        int32_t* out = p.trace + SEQ_TRACE_HEADER_INTS + k * SEQ_TRACE_RECORD_WORDS;
        out[0] = c;
        out[1] = sh.w_accept[c];
        out[2] = __float_as_int(sh.w_ratio[c]);
        out[3] = __float_as_int(sh.w_uniform[c]);
    }
    CHAIN_LAST(2);
    if constexpr (TEAM) {
        // (the per-block numbers of the draw go where the records were: the walk has read them)
        const int leaf = sh.w_leaf;
        if (leaf >= 0 && !sh.w_fail)
            leaf_draw<LT, NT>(static_cast<const LT*>(p.target) + (size_t)leaf * V, V, slope, sh.w_uniform[0], vec_ok, sh);
    }
    if (tid == 0) {
        const bool ok = sh.w_fail == 0;
        p.bonus[0] = ok ? sh.bonus_token : -1;
        float* binfo = reinterpret_cast<float*>(p.trace + SEQ_TRACE_HEADER_INTS +
                                                SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS);
        binfo[0] = sh.w_uniform[0];
        binfo[1] = sh.bonus_info[0];
        binfo[2] = sh.bonus_info[1];
        binfo[3] = sh.bonus_info[2];
        p.trace[1] = ok ? 0 : 1;
        CHAIN_STAMP(43);
        CHAIN_LAST(3);
    }
    launch_member_done<BATCHED>(p, true);
}

}  // namespace

#ifdef SEQTREE_STAMPS
extern "C" void seqtree_internal_read_chain_wg_times(long long* out, int count) {
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_chain_wg_times), sizeof(long long) * 8 * count);
}
extern "C" void seqtree_internal_read_chain_last(long long* out) {
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_chain_last), sizeof(long long) * 8);
}
extern "C" int seqtree_internal_read_chain_stamps(long long* out) {
    int count = 0;
    (void)hipMemcpyFromSymbol(&count, HIP_SYMBOL(g_chain_stamp_count), sizeof(int));
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_chain_stamps), sizeof(long long) * 64);
    return count;
}
#endif

void launch_verify_chains(const VerifyParams& p, int dtype, hipStream_t stream, int batch) {
    const dim3 grid((unsigned)p.n, (unsigned)batch), block(kThreads);
    const int chunks = (p.V + kThreads * kChunk - 1) / (kThreads * kChunk);
#define SEQ_CHAINS_CH(LT, CH)                                                                                      \
    do {                                                                                                           \
        if (batch > 1) hipLaunchKernelGGL((verify_chains_kernel<LT, CH, true, 0>), grid, block, 0, stream, p); \
        else hipLaunchKernelGGL((verify_chains_kernel<LT, CH, false, 0>), grid, block, 0, stream, p);          \
    } while (0)
#define SEQ_CHAINS(LT)                                  \
    do {                                                \
        if (chunks <= 1) SEQ_CHAINS_CH(LT, 1);          \
        else if (chunks <= 2) SEQ_CHAINS_CH(LT, 2);     \
        else SEQ_CHAINS_CH(LT, 4);                      \
    } while (0)
    if (dtype == SEQ_BF16) SEQ_CHAINS(uint16_t);
    else SEQ_CHAINS(float);
#undef SEQ_CHAINS
#undef SEQ_CHAINS_CH
}

int team_size_for(int vocab) { return (vocab + kTeamTokens - 1) / kTeamTokens; }

// p.W = team_size_for(p.V) members per node of p.internal_nodes (at least one node); with
// p.team_xcd the grid is dealt to the XCDs in whole teams, eight teams at a time.
void launch_verify_chains_team(const VerifyParams& p, int dtype, hipStream_t stream) {
    const int teams = p.team_xcd ? (p.n_internal + 7) / 8 * 8 : p.n_internal;
    const dim3 grid((unsigned)(teams * p.W)), block(kTeamThreads);
    if (dtype == SEQ_BF16) hipLaunchKernelGGL((verify_chains_kernel<uint16_t, kTeamChunks, false, kTeamThreads>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((verify_chains_kernel<float, kTeamChunks, false, kTeamThreads>), grid, block, 0, stream, p);
}
}  // namespace verify
}  // namespace seqtree
