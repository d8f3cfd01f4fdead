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
#include "seq_internal.h"
#include "verify_device.h"

namespace seqtree {
namespace verify {
namespace {

constexpr int kChunk = 8;   // consecutive tokens per thread and chunk: token (c * kThreads + tid) * 8 + e

struct ChainShared {
    float part[2][kWaves][4];          // per-wavefront partials, double-buffered by step parity
    float block_mass[64];              // residual mass of (chunk, wavefront) blocks, in token order
    float ctl_a, ctl_b;                // coefficients of the residual for the next pass
    int ctl_zero;                      // token whose probabilities the next pass clears (-1: none)
    int ctl_sum_q;                     // the next pass also sums the draft mass that is left
    int ctl_stop;                      // the child before was accepted: the walk leaves this node through it, nothing after it is needed
    BlockPick pick;
    int bonus_token;
    float bonus_info[3];               // total mass, CDF just below and just above the bonus token
    int last;
    // this node's rows at its children's tokens: tempered logits, then probabilities
    float child_lt[SEQ_MAX_TREE];
    float child_ld[SEQ_MAX_TREE];
    int child_tok[SEQ_MAX_TREE];
    unsigned char child_dup[SEQ_MAX_TREE];
    float child_u[SEQ_MAX_TREE];       // the children's uniforms
    // the final walk (last workgroup only)
    int w_child_start[SEQ_MAX_TREE + 1];
    int w_child_list[SEQ_MAX_TREE];
    float w_uniform[SEQ_MAX_TREE];
    float w_rec[SEQ_MAX_TREE][kChildRecordWords];
    float w_ratio[SEQ_MAX_TREE];
    uint32_t w_node[SEQ_MAX_TREE][kNodeRecordWords];
    int w_fail;
    int w_path[SEQ_MAX_TREE];
    int w_tested[SEQ_MAX_TREE];
    unsigned char w_accept[SEQ_MAX_TREE];
    int w_path_len, w_n_dec;
};

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
__device__ long long g_chain_wg_times[4 * 1024];   // per workgroup: start, rows in registers, chain done, end
#define CHAIN_STAMP_RESET() do { if (blockIdx.x == 0 && threadIdx.x == 0) g_chain_stamp_count = 0; } while (0)
#define CHAIN_WG_TIME(k) do { if (threadIdx.x == 0 && blockIdx.x < 1024) g_chain_wg_times[4 * blockIdx.x + (k)] = wall_clock64(); } while (0)
#define CHAIN_STAMP(id) do { if (blockIdx.x == 0 && threadIdx.x == 0 && g_chain_stamp_count < 31) { \
    g_chain_stamps[2 * g_chain_stamp_count] = (id); g_chain_stamps[2 * g_chain_stamp_count + 1] = wall_clock64(); ++g_chain_stamp_count; } } while (0)
#else
#define CHAIN_STAMP_RESET() do {} while (0)
#define CHAIN_STAMP(id) do {} while (0)
#define CHAIN_WG_TIME(k) do {} while (0)
#endif

template <typename LT, int CH, bool BATCHED>
__global__ __launch_bounds__(kThreads) void verify_chains_kernel(const VerifyParams p_in) {
    const VerifyParams p = BATCHED ? params_of_sequence(p_in, blockIdx.y, false) : p_in;
    __shared__ ChainShared sh;
    constexpr int EPT = CH * kChunk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int v = blockIdx.x;
    const int V = p.V;
    const LT* trow = static_cast<const LT*>(p.target) + (size_t)v * V;
    const LT* drow = static_cast<const LT*>(p.draft) + (size_t)v * V;
    const int c_begin = p.child_start[v], c_end = p.child_start[v + 1];
    const int K = c_end - c_begin;
    unsigned long long* const child_rec = p.records;                                    // [n][kChildRecordWords]
    unsigned long long* const node_rec = p.records + (size_t)p.n * kChildRecordWords;   // [n][kNodeRecordWords]
    // Tag of this launch: every workgroup reads the workspace's epoch on entry, and the last one to
    // arrive moves it on -- after all have read it.
    uint32_t* const epoch = chain_epoch_cell(p.records);
    const uint32_t tag = __hip_atomic_load(epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
    CHAIN_STAMP_RESET();
    CHAIN_STAMP(0);
    CHAIN_WG_TIME(0);

    const bool vec_ok = (V % (16 / (int)sizeof(LT)) == 0) &&
                        ((reinterpret_cast<uintptr_t>(p.target) | reinterpret_cast<uintptr_t>(p.draft)) & 15) == 0;
    float pr[EPT], qr[EPT];
#pragma unroll
    for (int c = 0; c < CH; ++c)
        load_row_slice<LT, kChunk>(trow, (c * kThreads + tid) * kChunk, V, 1.0f, vec_ok, pr + c * kChunk);
    if (K > 0) {
#pragma unroll
        for (int c = 0; c < CH; ++c)
            load_row_slice<LT, kChunk>(drow, (c * kThreads + tid) * kChunk, V, 1.0f, vec_ok, qr + c * kChunk);
    } else {
#pragma unroll
        for (int e = 0; e < EPT; ++e) qr[e] = -INFINITY;   // a leaf has no draft row to read
    }
    // both rows at the children's tokens, in flight together with the rows themselves
    for (int k = tid; k < K; k += kThreads) {
        const int s = min(max(p.tokens[p.child_list[c_begin + k]], 0), V - 1);  // stay inside the row
        sh.child_tok[k] = s;
        sh.child_u[k] = p.uniforms[p.child_list[c_begin + k]];
        sh.child_lt[k] = load_logit<LT>(trow, s);   // raw: the temperature is in the exponent's slope
        sh.child_ld[k] = load_logit<LT>(drow, s);
        bool dup = false;
        for (int j = 0; j < k; ++j) dup |= min(max(p.tokens[p.child_list[c_begin + j]], 0), V - 1) == s;
        sh.child_dup[k] = dup ? 1 : 0;
    }

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
    auto offset_of = [&](float raw_max) __attribute__((always_inline)) {
        return raw_max == -INFINITY ? INFINITY : __builtin_rintf(-raw_max * slope * 256.0f) * (1.0f / 256.0f);
    };
    float mt_wave = -INFINITY, md_wave = -INFINITY;
#pragma unroll
    for (int e = 0; e < EPT; ++e) { mt_wave = fmaxf(mt_wave, pr[e]); md_wave = fmaxf(md_wave, qr[e]); }
    const float bt_wave = offset_of(wave_reduce<kOpMax>(mt_wave));   // +inf: nothing but -inf in my part of the row
    const float bd_wave = offset_of(wave_reduce<kOpMax>(md_wave));
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
    float bt_row, bd_row, inv_zt, inv_zd;   // offsets of the rows (those of the wavefronts with the largest maxima)
    {
        // every wavefront folds the same 16 partials in the same order: identical results
        const int w = lane & 15;
        const float bt_w = sh.part[0][w][0], zt_w = sh.part[0][w][1];
        const float bd_w = sh.part[0][w][2], zd_w = sh.part[0][w][3];
        bt_row = -lane_value(row_reduce<kOpMax>(-bt_w), 0);
        bd_row = -lane_value(row_reduce<kOpMax>(-bd_w), 0);
        // (bt_row - bt_w is an exact multiple of 1/256, at most 0: the hardware exponential of it
        // is the same number wherever it is taken)
        const float zt = lane_value(row_reduce<kOpSum>(bt_w != INFINITY ? zt_w * __builtin_amdgcn_exp2f(bt_row - bt_w) : 0.f), 0);
        const float zd = lane_value(row_reduce<kOpSum>(bd_w != INFINITY ? zd_w * __builtin_amdgcn_exp2f(bd_row - bd_w) : 0.f), 0);
        inv_zt = 1.0f / zt;
        inv_zd = 1.0f / zd;
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
    // Thread 0 owns the scalar state.  Iteration j: it applies the pass that followed child j-1,
    // writes that child's record, tests child j and publishes the coefficients of the next pass;
    // iteration K only closes child K-1 and publishes the coefficients of the bonus draw.
    //
    // The draft mass left after a rejection is the mass before it minus the rejected token's: as
    // long as a twentieth of the mass is left, thread 0 takes that difference (in fp64; its error
    // is that of the initial normalisation, 1e-7 absolute) and the pass skips the sum over q.  Once
    // less is left the pass sums q again, which is also what finds the mass exactly zero.
    NodeState ns, before;
    bool accepted = false, stopped = false;   // (accepted: thread 0 only)
    uint32_t events = 0;
    double q_predicted = 1.0;
    bool q_summed = true;
    if (tid == 0) { node_begin(ns); ns.fallbacks = 0; ns.degenerate = 0; }
    int par = 1;
    for (int j = 0; j <= K; ++j) {
        if (wave == 0) {
            // lanes 0..15 read the 16 per-wavefront partials (the other rows repeat them)
            const float w_new = lane_value(row_reduce<kOpSum>(sh.part[par ^ 1][lane & 15][0]), 0);
            const float q_new = lane_value(row_reduce<kOpSum>(sh.part[par ^ 1][lane & 15][1]), 0);
            if (tid == 0) {
                // Everybody waits for the coefficients of the next pass, so they go out first; the
                // test of child j, which needs the state before its rejection, is worked out from
                // a copy after the barrier, while the pass runs.  The uniforms are inputs: if that
                // test accepts, the walk will leave this node through child j and never look at
                // the later children or at this node's bonus token, so the chain ends at the next
                // step (the pass under way is the price of not waiting for the test here).
                sh.ctl_stop = accepted ? 1 : 0;
                if (accepted) {
                    sh.w_rec[j - 1][4] = 0.f;   // no rejection followed child j - 1
                } else if (j > 0) {
                    const int fb = ns.fallbacks, dg = ns.degenerate;
                    node_apply_pass(ns, (double)w_new, q_summed ? (double)q_new : q_predicted);
                    events = (uint32_t)(ns.fallbacks - fb) | ((uint32_t)(ns.degenerate - dg) << 1);
                }
                if (j < K && !accepted) {
                    before = ns;
                    // (SpecInfer: the draft distribution stays what it was -- nothing is struck out)
                    const bool in_s = !p.with_replacement && sh.child_dup[j] != 0;
                    const bool strike = !in_s && !p.with_replacement;
                    node_reject_child(ns, in_s, V, p.with_replacement != 0);
                    sh.ctl_zero = strike ? sh.child_tok[j] : -1;
                    q_predicted = ns.massQ - (strike ? (double)sh.child_ld[j] : 0.0);
                    q_summed = ns.fallback || !(q_predicted >= 0.05);
                    sh.ctl_sum_q = q_summed ? 1 : 0;
                }
                sh.ctl_a = ns.af;
                sh.ctl_b = ns.bf;
            }
        }
        __syncthreads();
        CHAIN_STAMP(10);
        if (sh.ctl_stop) {
            for (int k = j + tid; k < K; k += kThreads) {
#pragma unroll
                for (int w = 0; w < kChildRecordWords; ++w) sh.w_rec[k][w] = 0.f;   // 0 < 0: never accepted
            }
            stopped = true;
            break;
        }
        if (tid == 0) {
            // records wait in shared memory; they leave together once the chain is done
            if (j > 0) sh.w_rec[j - 1][4] = __uint_as_float(events);
            if (j < K) {
                const ChildTest t = node_test_child(before, sh.child_lt[j], sh.child_ld[j],
                                                    !p.with_replacement && sh.child_dup[j] != 0, V);
                sh.w_rec[j][0] = t.lhs_w; sh.w_rec[j][1] = t.lhs_q;
                sh.w_rec[j][2] = t.rhs_r; sh.w_rec[j][3] = t.rhs_m;
                accepted = t.accepts(sh.child_u[j]);
            }
        }
        if (j == K) break;
        const float af = sh.ctl_a, bf = sh.ctl_b;
        const int zero_token = sh.ctl_zero;
        // the rejected token leaves both distributions: only the wavefront that holds it looks
        if (zero_token >= 0 && ((zero_token / kChunk) % kThreads) / 64 == wave) {
            const int slot = (zero_token / (kChunk * kThreads)) * kChunk + zero_token % kChunk;
            if ((zero_token / kChunk) % kThreads == tid) {
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
    if (stopped) {   // the walk goes on through the accepted child: no token is drawn here
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
            if (lane == 0) sh.block_mass[c * kWaves + wave] = wm;
        }
        __syncthreads();
        if (wave == 0) {
            const BlockPick b = pick_block(u0, lane < CH * kWaves ? sh.block_mass[lane] : 0.f, CH * kWaves);
            if (lane == 0) { sh.pick = b; sh.bonus_token = -1; }
        }
        __syncthreads();
        const BlockPick b = sh.pick;
        if (wave == b.owner % kWaves) {
            const int cs = b.owner / kWaves;
            float mine_f = mass[0];
#pragma unroll
            for (int c = 1; c < CH; ++c) mine_f = c == cs ? mass[c] : mine_f;
            const double mine = (double)mine_f;
            const double incl = wave_scan(mine);
            const double goal = (double)u0 * b.total;
            const int base = (cs * kThreads + tid) * kChunk;
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
                sh.bonus_token = wave_last >= 0 ? wave_last : min(V - 1, (cs * kThreads + wave * 64) * kChunk);
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
    for (int k = tid; k < K; k += kThreads) {
        unsigned long long* rec = child_rec + (size_t)p.child_list[c_begin + k] * kChildRecordWords;
#pragma unroll
        for (int w = 0; w < kChildRecordWords; ++w) put(rec + w, tag, sh.w_rec[k][w]);
    }
    __syncthreads();   // all records are on their way before this workgroup counts as arrived
    if (tid == 0) {
        unsigned long long* rec = node_rec + (size_t)v * kNodeRecordWords;
        put(rec + 0, tag, (uint32_t)sh.bonus_token);
        put(rec + 1, tag, sh.bonus_info[0]);
        put(rec + 2, tag, sh.bonus_info[1]);
        put(rec + 3, tag, sh.bonus_info[2]);
        CHAIN_STAMP(40);
        const uint32_t arrived = __hip_atomic_fetch_add(p.arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = arrived == (uint32_t)(p.n - 1);
        if (last) __hip_atomic_store(p.arrivals, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
        sh.last = last;
        sh.w_fail = 0;
    }
    __syncthreads();
    CHAIN_STAMP(41);
    CHAIN_WG_TIME(3);
    if (!sh.last) return;

    // ---- the walk (Sec. 2.2: Algorithm 2 applied recursively from the root) -------------------
    for (int i = tid; i < p.n; i += kThreads) {
        sh.w_child_start[i] = p.child_start[i];
        sh.w_uniform[i] = p.uniforms[i];
        if (i < p.n - 1) sh.w_child_list[i] = p.child_list[i];
        if (i > 0) {
            const unsigned long long* rec = child_rec + (size_t)i * kChildRecordWords;
            unsigned long long w[kChildRecordWords];
#pragma unroll
            for (int k = 0; k < kChildRecordWords; ++k)
                w[k] = __hip_atomic_load(rec + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < kChildRecordWords; ++k) {
                uint32_t payload = (uint32_t)w[k];
                if ((uint32_t)(w[k] >> 32) != tag) ok &= get(rec + k, tag, p.spin_limit, &payload);
                sh.w_rec[i][k] = __uint_as_float(payload);
            }
            if (!ok) sh.w_fail = 1;
        }
        {
            const unsigned long long* rec = node_rec + (size_t)i * kNodeRecordWords;
            unsigned long long w[kNodeRecordWords];
#pragma unroll
            for (int k = 0; k < kNodeRecordWords; ++k)
                w[k] = __hip_atomic_load(rec + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < kNodeRecordWords; ++k) {
                uint32_t payload = (uint32_t)w[k];
                if ((uint32_t)(w[k] >> 32) != tag) ok &= get(rec + k, tag, p.spin_limit, &payload);
                sh.w_node[i][k] = payload;
            }
            if (!ok) sh.w_fail = 1;
        }
    }
    if (tid == 0) sh.w_child_start[p.n] = p.child_start[p.n];
    __syncthreads();
    CHAIN_STAMP(42);
    // every accept test of the tree at once; the walk itself only follows pointers
    for (int c = 1 + tid; c < p.n; c += kThreads) {
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
        const uint32_t* nr = sh.w_node[cur];
        const bool ok = sh.w_fail == 0;
        p.bonus[0] = ok ? (int32_t)nr[0] : -1;
        float* binfo = reinterpret_cast<float*>(p.trace + SEQ_TRACE_HEADER_INTS +
                                                SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS);
        binfo[0] = sh.w_uniform[0];
        binfo[1] = __uint_as_float(nr[1]);
        binfo[2] = __uint_as_float(nr[2]);
        binfo[3] = __uint_as_float(nr[3]);
        p.trace[0] = n_dec;
        p.trace[1] = ok ? 0 : 1;
        p.trace[2] = cur;
        p.trace[3] = fallbacks;
        p.trace[4] = degenerate;
        p.trace[5] = p.trace[6] = p.trace[7] = 0;
        sh.w_path_len = path_len;
        sh.w_n_dec = n_dec;
        __hip_atomic_fetch_add(epoch, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        CHAIN_STAMP(43);
      }
    }
    __syncthreads();
    for (int i = tid; i < p.n; i += kThreads) p.path[i] = i < sh.w_path_len ? sh.w_path[i] : -1;
    for (int k = tid; k < sh.w_n_dec; k += kThreads) {
        const int c = sh.w_tested[k];
        int32_t* out = p.trace + SEQ_TRACE_HEADER_INTS + k * SEQ_TRACE_RECORD_WORDS;
        out[0] = c;
        out[1] = sh.w_accept[c];
        out[2] = __float_as_int(sh.w_ratio[c]);
        out[3] = __float_as_int(sh.w_uniform[c]);
    }
}

}  // namespace

#ifdef SEQTREE_STAMPS
extern "C" void seqtree_internal_read_chain_wg_times(long long* out, int count) {
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_chain_wg_times), sizeof(long long) * 4 * count);
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
#define SEQ_CHAINS_CH(LT, CH)                                                                                   \
    do {                                                                                                        \
        if (batch > 1) hipLaunchKernelGGL((verify_chains_kernel<LT, CH, true>), grid, block, 0, stream, p);     \
        else hipLaunchKernelGGL((verify_chains_kernel<LT, CH, false>), grid, block, 0, stream, p);              \
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
}  // namespace verify
}  // namespace seqtree
