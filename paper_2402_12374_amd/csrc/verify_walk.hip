// seq_verify: the Sequoia verification walk (Algorithm 2, Sec. 3.2.1, applied recursively from
// the root, Sec. 2.2) as ONE kernel launch.
//
// Only the rows of nodes the walk actually visits are read (the accepted path plus the node
// where it stops), so the logit traffic is (len(path)+1) * 2 * vocab elements instead of the
// whole [n_tree, vocab] matrices.
//
// A small team of workgroups (at most 64) shares the vocabulary: each thread keeps a few
// consecutive tokens of the current node's target and draft rows in registers, first as tempered
// logits, then as probabilities p[x], q[x].  Every step of the algorithm that needs a
// vocabulary-wide number (softmax max/normaliser, the mass of the new residual, the mass of
// the remaining draft) is one reduction per workgroup followed by one all-to-all exchange of the
// per-workgroup partials through tagged 64-bit slots in global memory; the first wavefront of
// every workgroup then combines the same partials in the same order and its first lane takes
// the next step of the algorithm, so all workgroups reach identical decisions without a leader
// workgroup.  A step costs two workgroup barriers and one exchange.  Waiting is bounded: a
// workgroup that does not see its peers within `spin_limit` polls records status 1 in the trace
// and leaves.
#include <cmath>

#include "seq_internal.h"
#include "verify_device.h"

namespace seqtree {
using namespace verify;



namespace {


__device__ __forceinline__ int wg_rank() { return (int)blockIdx.x; }

// Phase timestamps of workgroup 0 (100 MHz wall clock), compiled in with -DSEQTREE_STAMPS only.
#ifdef SEQTREE_STAMPS
__device__ long long g_stamps[64];
__device__ int g_stamp_count;
#define SEQ_STAMP_RESET() do { if (blockIdx.x == 0 && threadIdx.x == 0) g_stamp_count = 0; } while (0)
#define SEQ_STAMP(id) do { if (blockIdx.x == 0 && threadIdx.x == 0 && g_stamp_count < 31) { \
    g_stamps[2 * g_stamp_count] = (id); g_stamps[2 * g_stamp_count + 1] = wall_clock64(); ++g_stamp_count; } } while (0)
#else
#define SEQ_STAMP_RESET() do {} while (0)
#define SEQ_STAMP(id) do {} while (0)
#endif

constexpr int kActPass = 0, kActAccepted = 1, kActExhausted = 2;

struct Shared {
    float part[2][kWaves][4];           // per-wavefront partials, double-buffered by step parity
    float stat[4];                      // max and 1/normaliser of the target and draft rows
    double bonus_d[2];                  // total residual mass, mass before the owning workgroup
    int bonus_i[2];                     // owning workgroup, 1 if rounding left no owner
    double scan[kWaves];
    float red_f[kWaves];
    int red_i[kWaves];
    int fail;
    int cand_min;
    int cand_max;
    // the tree and the per-node draws, staged once so the walk never chases them through memory
    int child_start[SEQ_MAX_TREE + 1];
    int child_list[SEQ_MAX_TREE];
    int token[SEQ_MAX_TREE];
    float uniform[SEQ_MAX_TREE];
    // the current node's rows at its children's tokens: tempered logits, then probabilities
    float child_lt[SEQ_MAX_TREE];
    float child_ld[SEQ_MAX_TREE];
    unsigned char child_dup[SEQ_MAX_TREE];  // child's token already carried by an earlier sibling
    // What the first wavefront, which keeps the state of Algorithm 2 at the current node in its
    // registers, tells the others after every step (written by its lane 0, read after a barrier).
    // The four words everybody needs after every step come first and are read with one 16-byte
    // load, together with `fail`: read one after the other, behind the branches that use them,
    // they were three trips to shared memory on the path of every rejection.
    struct __attribute__((aligned(16))) {
        float af, bf;               // coefficients of the residual for the next pass
        int action, zero_token;
        int next, n_dec, sums_valid, fallbacks, degenerate;
    } st;
};

// What a thread takes from the first wavefront's message after a step's barrier.
struct StepWord {
    float af, bf;
    int action, zero_token, fail;
};
__device__ __forceinline__ StepWord read_step(const Shared& sh) {
    const uint4 w = *reinterpret_cast<const uint4*>(&sh.st);
    const int fail = sh.fail;
    StepWord s;
    s.af = __uint_as_float(w.x); s.bf = __uint_as_float(w.y);
    s.action = (int)w.z; s.zero_token = (int)w.w; s.fail = fail;
    return s;
}

// All-to-all of K floats per workgroup, run by the first wavefront only.  mine[k] is this
// workgroup's value; afterwards lane w of the wavefront holds workgroup w's values in got[]
// (lanes >= W keep `fill`).  Two slot buffers alternate by step parity: a workgroup can be at
// most one step ahead of the slowest one, because it cannot finish a step without that
// workgroup's contribution.
template <int K>
__device__ __forceinline__ bool exchange(const VerifyParams& p, uint32_t tag_base, uint32_t step,
                                         const float (&mine)[K], float fill, float (&got)[K]) {
    // (inside, plain floats and no arrays: an array that the compiler cannot dissolve into
    // registers goes to a per-thread slice of shared memory, whose address needs the workgroup's
    // size, which the kernel would have to fetch from the dispatch packet -- a trip to host memory)
    static_assert(K >= 1 && K <= kVerifySlotWords, "slot words per step");
    const int lane = threadIdx.x;  // first wavefront: 0..63
    const float mine0 = mine[0], mine1 = mine[K > 1 ? 1 : 0], mine2 = mine[K > 2 ? 2 : 0], mine3 = mine[K > 3 ? 3 : 0];
    float got0 = fill, got1 = fill, got2 = fill, got3 = fill;
    auto hand_back = [&]() __attribute__((always_inline)) {
        got[0] = got0;
        if constexpr (K > 1) got[1] = got1;
        if constexpr (K > 2) got[2] = got2;
        if constexpr (K > 3) got[3] = got3;
    };
    if (p.W == 1) {   // nobody to talk to
        if (lane == 0) { got0 = mine0; got1 = mine1; got2 = mine2; got3 = mine3; }
        hand_back();
        return true;
    }
    const uint32_t tag = tag_base + step;
    unsigned long long* buf = p.slots + (size_t)(step & 1u) * kVerifyMaxGroups * kVerifySlotWords;
    if (lane < K) {
        const float v = lane == 0 ? mine0 : lane == 1 ? mine1 : lane == 2 ? mine2 : mine3;
        const unsigned long long word = ((unsigned long long)tag << 32) | __float_as_uint(v);
        __hip_atomic_store(&buf[lane * kVerifyMaxGroups + wg_rank()], word, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    bool done = lane >= p.W;
    uint32_t spins = 0;
    auto look = [&](int k, float& value) __attribute__((always_inline)) {
        const unsigned long long word = __hip_atomic_load(&buf[k * kVerifyMaxGroups + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(word >> 32) != tag) return false;
        value = __uint_as_float((uint32_t)word);
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
        if (__all(done)) { hand_back(); return true; }
        if (++spins > p.spin_limit) { hand_back(); return false; }   // bounded wait: every wave leaves this loop
        __builtin_amdgcn_s_sleep(1);
    }
}

// Tags must differ from launch to launch (also when a captured graph replays the same kernel
// arguments) and agree between the workgroups of one launch.  epoch[0] is the tag base: every
// workgroup reads it on entry and workgroup 0 moves it on when it leaves -- which it cannot do
// before every workgroup has published, hence read the epoch, at least once.  That argument
// fails only after a timed-out wait, so a timeout also sets the poison flag, and every later launch
// refuses to run (status 1) until seq_shutdown() has discarded the area.  (A batched launch has
// an epoch, a flag and a set of slots per sequence: its teams share nothing.)
__device__ __forceinline__ uint32_t launch_tag_base(const VerifyParams& p, bool* poisoned) {
    *poisoned = __hip_atomic_load(p.poison, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
    return __hip_atomic_load(p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void stage_tree(const VerifyParams& p, Shared& sh) {
    for (int i = threadIdx.x; i < p.n; i += kThreads) {
        sh.child_start[i] = p.child_start[i];
        sh.token[i] = min(max(p.tokens[i], 0), p.V - 1);  // stay inside the row whatever was sent
        sh.uniform[i] = p.uniforms[i];
        if (i < p.n - 1) sh.child_list[i] = p.child_list[i];
    }
    if (threadIdx.x == 0) sh.child_start[p.n] = p.child_start[p.n];
}

// The status word of the trace is cleared by workgroup 0 on entry and only ever raised after
// that, by whichever workgroup gives up waiting: it may be the one that owns the bonus token,
// and workgroup 0 may have left with a clean status by then.
__device__ __forceinline__ void begin_trace(const VerifyParams& p) {
    if (wg_rank() == 0 && threadIdx.x == 0)
        __hip_atomic_store(&p.trace[1], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void finish(const VerifyParams& p, int path_len, int n_dec, int status,
                                       int stop_node, int fallbacks, int degenerate) {
    if (status != 0 && threadIdx.x == 0) {
        __hip_atomic_store(p.poison, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_max(&p.trace[1], status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        p.bonus[0] = -1;
    }
    if (wg_rank() != 0) return;
    for (int i = path_len + (int)threadIdx.x; i < p.n; i += kThreads) p.path[i] = -1;
    if (threadIdx.x == 0) {
        p.trace[0] = n_dec;
        p.trace[2] = stop_node;
        p.trace[3] = fallbacks;
        p.trace[4] = degenerate;
        p.trace[5] = p.trace[6] = p.trace[7] = 0;
        atomicAdd(p.epoch, (uint32_t)kVerifyTagsPerCall);
    }
}

__device__ __forceinline__ void record(const VerifyParams& p, int n_dec, int node, bool accepted,
                                       float ratio, float u) {
    if (wg_rank() == 0 && threadIdx.x == 0) {
        int32_t* rec = p.trace + SEQ_TRACE_HEADER_INTS + n_dec * SEQ_TRACE_RECORD_WORDS;
        rec[0] = node;
        rec[1] = accepted ? 1 : 0;
        rec[2] = __float_as_int(ratio);
        rec[3] = __float_as_int(u);
    }
}

// The scalar side of Algorithm 2 at the current node, kept by the first wavefront in registers
// (every lane holds the same values; nothing of it waits for shared memory on the path from a
// vocabulary sum to the next pass's coefficients), and what it knows of the child that will be
// tested next, fetched ahead -- while the others' partials are still on their way.
struct NextChild {
    int node, token;
    float u, ps, qs;     // the child's uniform, and both rows' probabilities at its token
    int dup;             // its token was already carried by an earlier sibling
};
struct Leader {
    NodeState ns;
    int ci, n_dec;
    NextChild nx;
};
__device__ __forceinline__ void fetch_child(const Shared& sh, Leader& ld, int c_begin, int c_end) {
    if (ld.ci >= c_end) return;
    const int k = ld.ci - c_begin;
    const int c = sh.child_list[ld.ci];
    ld.nx.node = c;
    ld.nx.token = sh.token[c];
    ld.nx.u = sh.uniform[c];
    ld.nx.ps = sh.child_lt[k];   // probabilities by now
    ld.nx.qs = sh.child_ld[k];
    ld.nx.dup = sh.child_dup[k];
}
// One step: applies the result of the previous vocabulary pass if there was one, then tests the
// next child: accepted, or rejected (a pass over the vocabulary is needed before the next
// test), or none is left.  Publishes the outcome (lane 0) for the other wavefronts.
__device__ __forceinline__ void leader_step(const VerifyParams& p, Shared& sh, Leader& ld, int c_end, int V,
                                            bool have_pass, double w_new, double q_new) {
    if (have_pass) node_apply_pass(ld.ns, w_new, q_new);
    int action, next = -1, zero_token = -1;
    if (ld.ci == c_end) {
        action = kActExhausted;
    } else {
        // SpecInfer keeps the draft distribution as it is: no token is ever struck out
        const bool in_s = !p.with_replacement && ld.nx.dup != 0;
        const ChildTest t = node_test_child(ld.ns, ld.nx.ps, ld.nx.qs, in_s, V);
        const bool accept = t.accepts(ld.nx.u);
        record(p, ld.n_dec, ld.nx.node, accept, t.ratio(), ld.nx.u);
        ++ld.n_dec;
        if (accept) {
            action = kActAccepted;
            next = ld.nx.node;
        } else {
            node_reject_child(ld.ns, in_s, V, p.with_replacement != 0);
            zero_token = (in_s || p.with_replacement) ? -1 : ld.nx.token;
            ++ld.ci;
            action = kActPass;
        }
    }
    if (threadIdx.x == 0) {
        sh.st.af = ld.ns.af; sh.st.bf = ld.ns.bf;
        sh.st.action = action; sh.st.next = next; sh.st.zero_token = zero_token;
        sh.st.n_dec = ld.n_dec; sh.st.sums_valid = ld.ns.sums_valid;
        sh.st.fallbacks = ld.ns.fallbacks; sh.st.degenerate = ld.ns.degenerate;
    }
}

// First wavefront: which workgroup holds the token at cumulative residual mass u * total?
// `sw_f` is the mass of workgroup `lane`.
__device__ __forceinline__ void find_bonus_owner(const VerifyParams& p, float u0, float sw_f, Shared& sh) {
    const BlockPick b = pick_block(u0, sw_f, p.W);
    if (threadIdx.x == 0) { sh.bonus_d[0] = b.total; sh.bonus_d[1] = b.before; sh.bonus_i[0] = b.owner; sh.bonus_i[1] = b.forced; }
}

// Per-wavefront partials -> this workgroup's values, inside the first wavefront (lane w < kWaves
// reads wavefront w's partial; kWaves <= 16, so one 16-lane row holds them all).
template <int OP>
__device__ __forceinline__ float fold_waves(const Shared& sh, int par, int k, float identity) {
    const int lane = threadIdx.x;
    const float v = lane < kWaves ? sh.part[par][lane][k] : identity;
    return lane_value(row_reduce<OP>(v), 0);
}

template <typename LT, int EPT, bool BATCHED>
__global__ __launch_bounds__(kThreads) void verify_walk_kernel(const VerifyParams p_in) {
    const VerifyParams p = BATCHED ? params_of_sequence(p_in, blockIdx.y, true) : p_in;
    __shared__ Shared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int base = (wg_rank() * kThreads + tid) * EPT;  // my EPT consecutive tokens
    const LT* target = static_cast<const LT*>(p.target);
    const LT* draft = static_cast<const LT*>(p.draft);
    const int V = p.V;

    SEQ_STAMP_RESET();
    SEQ_STAMP(0);
    const bool vec_ok = (V % (16 / (int)sizeof(LT)) == 0) &&
                        ((reinterpret_cast<uintptr_t>(p.target) | reinterpret_cast<uintptr_t>(p.draft)) & 15) == 0;
    float pr[EPT], qr[EPT];
    // the root's rows are needed whatever happens: ask for them before anything else
    load_row_slices<LT, EPT, 1, true>(target, draft, base, 0, V, p.inv_T, vec_ok, pr, qr);
    bool poisoned;
    const uint32_t tag_base = launch_tag_base(p, &poisoned);
    begin_trace(p);
    if (poisoned) { finish(p, 0, 0, 1, 0, 0, 0); return; }
    stage_tree(p, sh);
    uint32_t step = 0;
    int par = 0, v = 0, path_len = 0;
    Leader ld;   // (first wavefront)
    ld.n_dec = 0; ld.ns.fallbacks = 0; ld.ns.degenerate = 0;
    if (tid == 0) { sh.st.n_dec = 0; sh.st.fallbacks = 0; sh.st.degenerate = 0; }
    __syncthreads();

    for (;;) {
        const LT* trow = target + (size_t)v * V;
        const LT* drow = draft + (size_t)v * V;
        const int c_begin = sh.child_start[v], c_end = sh.child_start[v + 1];
        // both rows at the children's tokens (needed for the accept tests), in flight together
        // with the row slices themselves
        const int K = c_end - c_begin;
        if (K > 64) {
            for (int k = tid; k < K; k += kThreads) {
                const int s = sh.token[sh.child_list[c_begin + k]];
                sh.child_lt[k] = load_logit<LT>(trow, s) * p.inv_T;
                sh.child_ld[k] = load_logit<LT>(drow, s) * p.inv_T;
                bool dup = false;
                for (int j = 0; j < k; ++j) dup |= sh.token[sh.child_list[c_begin + j]] == s;
                sh.child_dup[k] = dup ? 1 : 0;
            }
        } else if (tid < 64 && K > 0) {
            // a lane per child: "an earlier sibling has the same token" is a walk over lanes
            const int k = tid;
            const int s = sh.token[sh.child_list[c_begin + min(k, K - 1)]];
            const float lt = load_logit<LT>(trow, s) * p.inv_T, ld_ = load_logit<LT>(drow, s) * p.inv_T;
            bool dup = false;
            for (int j = 0; j < K - 1; ++j) dup |= j < k && __builtin_amdgcn_readlane(s, j) == s;
            if (k < K) {
                sh.child_lt[k] = lt;
                sh.child_ld[k] = ld_;
                sh.child_dup[k] = dup ? 1 : 0;
            }
        }
        if (v != 0) {
            load_row_slices<LT, EPT, 1, true>(trow, drow, base, 0, V, p.inv_T, vec_ok, pr, qr);
        }
        SEQ_STAMP(1);
        // softmax statistics: per wavefront first (no barrier), then folded by the first wavefront.
        // pr/qr become e^(x - wave max); one more factor per wavefront turns them into
        // probabilities once the vocabulary-wide max and normaliser are known.
        float mt_wave = -INFINITY, md_wave = -INFINITY;
        {
#pragma unroll
            for (int e = 0; e < EPT; ++e) { mt_wave = fmaxf(mt_wave, pr[e]); md_wave = fmaxf(md_wave, qr[e]); }
            mt_wave = wave_reduce<kOpMax>(mt_wave);
            md_wave = wave_reduce<kOpMax>(md_wave);
            float zt = 0.f, zd = 0.f;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                pr[e] = prob_of(pr[e], mt_wave, 1.0f);
                qr[e] = prob_of(qr[e], md_wave, 1.0f);
                zt += pr[e];
                zd += qr[e];
            }
            zt = wave_reduce<kOpSum>(zt);
            zd = wave_reduce<kOpSum>(zd);
            if (lane == 0) { sh.part[par][wave][0] = mt_wave; sh.part[par][wave][1] = zt; sh.part[par][wave][2] = md_wave; sh.part[par][wave][3] = zd; }
        }
        __syncthreads();
        SEQ_STAMP(2);
        if (wave == 0) {
            float mine[4], got[4];
            {
                const bool have = lane < kWaves;
                const float mt_w = have ? sh.part[par][lane][0] : -INFINITY, zt_w = have ? sh.part[par][lane][1] : 0.f;
                const float md_w = have ? sh.part[par][lane][2] : -INFINITY, zd_w = have ? sh.part[par][lane][3] : 0.f;
                mine[0] = lane_value(row_reduce<kOpMax>(mt_w), 0);
                mine[2] = lane_value(row_reduce<kOpMax>(md_w), 0);
                mine[1] = lane_value(row_reduce<kOpSum>(zt_w > 0.f ? zt_w * exp_fast(mt_w - mine[0]) : 0.f), 0);
                mine[3] = lane_value(row_reduce<kOpSum>(zd_w > 0.f ? zd_w * exp_fast(md_w - mine[2]) : 0.f), 0);
            }
            const bool ok = exchange<4>(p, tag_base, ++step, mine, 0.f, got);
            SEQ_STAMP(3);
            const bool have = lane < p.W;
            const float mt = wave_reduce<kOpMax>(have && got[1] > 0.f ? got[0] : -INFINITY);
            const float md = wave_reduce<kOpMax>(have && got[3] > 0.f ? got[2] : -INFINITY);
            const float zt = wave_reduce<kOpSum>(have && got[1] > 0.f ? got[1] * exp_fast(got[0] - mt) : 0.f);
            const float zd = wave_reduce<kOpSum>(have && got[3] > 0.f ? got[3] * exp_fast(got[2] - md) : 0.f);
            // the children's logits become probabilities, a lane per child
            for (int k = lane; k < c_end - c_begin; k += 64) {
                sh.child_lt[k] = prob_of(sh.child_lt[k], mt, 1.0f / zt);
                sh.child_ld[k] = prob_of(sh.child_ld[k], md, 1.0f / zd);
            }
            if (lane == 0) {
                sh.fail = ok ? 0 : 1;
                sh.stat[0] = mt; sh.stat[1] = md; sh.stat[2] = 1.0f / zt; sh.stat[3] = 1.0f / zd;
            }
            node_begin(ld.ns);
            ld.ci = c_begin;
            fetch_child(sh, ld, c_begin, c_end);   // (the probabilities above were written by this wavefront)
            leader_step(p, sh, ld, c_end, V, false, 0.0, 0.0);
            fetch_child(sh, ld, c_begin, c_end);   // the one after, while everybody turns logits into probabilities
        } else {
            ++step;
        }
        par ^= 1;
        __syncthreads();
        SEQ_STAMP(4);
        StepWord sw = read_step(sh);
        if (sw.fail) { finish(p, path_len, sh.st.n_dec, 1, v, sh.st.fallbacks, sh.st.degenerate); return; }
        {
            const float ft = mt_wave == -INFINITY ? 0.f : exp_fast(mt_wave - sh.stat[0]) * sh.stat[2];
            const float fd = md_wave == -INFINITY ? 0.f : exp_fast(md_wave - sh.stat[1]) * sh.stat[3];
#pragma unroll
            for (int e = 0; e < EPT; ++e) { pr[e] *= ft; qr[e] *= fd; }
        }

        // Algorithm 2 at node v: one vocabulary pass + exchange per rejection
        while (sw.action == kActPass) {
            const int zero_token = sw.zero_token;
            const float af = sw.af, bf = sw.bf;
            float r_loc = 0.f, q_loc = 0.f;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                if (base + e == zero_token) { pr[e] = 0.f; qr[e] = 0.f; }
                r_loc += residual_of(pr[e], qr[e], af, bf);
                q_loc += qr[e];
            }
            r_loc = wave_reduce<kOpSum>(r_loc);
            q_loc = wave_reduce<kOpSum>(q_loc);
            if (lane == 0) { sh.part[par][wave][0] = r_loc; sh.part[par][wave][1] = q_loc; }
            __syncthreads();
            SEQ_STAMP(10);
            if (wave == 0) {
                float mine[2], got[2];
                mine[0] = fold_waves<kOpSum>(sh, par, 0, 0.f);
                mine[1] = fold_waves<kOpSum>(sh, par, 1, 0.f);
                const bool ok = exchange<2>(p, tag_base, ++step, mine, 0.f, got);
                SEQ_STAMP(11);
                const float w_new = wave_reduce<kOpSum>(got[0]);
                const float q_new = wave_reduce<kOpSum>(got[1]);
                if (lane == 0) sh.fail = ok ? 0 : 1;
                const bool exhausted = ld.ci == c_end;
                leader_step(p, sh, ld, c_end, V, true, (double)w_new, (double)q_new);
                if (ok && exhausted && ld.ns.sums_valid) find_bonus_owner(p, sh.uniform[0], got[0], sh);
                fetch_child(sh, ld, c_begin, c_end);   // for the step after the pass that starts now
            } else {
                ++step;
            }
            par ^= 1;
            __syncthreads();
            SEQ_STAMP(12);
            sw = read_step(sh);
            if (sw.fail) { finish(p, path_len, sh.st.n_dec, 1, v, sh.st.fallbacks, sh.st.degenerate); return; }
        }
        if (sw.action == kActAccepted) {
            const int next = sh.st.next;
            if (wg_rank() == 0 && tid == 0) p.path[path_len] = next;
            ++path_len;
            v = next;
            __syncthreads();  // everyone has read the state before the next node rewrites it
            continue;
        }

        // no child accepted: bonus token ~ R by inverse CDF with uniforms[0]
        const float af = sw.af, bf = sw.bf;
        const float u0 = sh.uniform[0];
        if (!sh.st.sums_valid) {   // no pass has left the workgroups' residual masses yet
            float r_loc = 0.f;
#pragma unroll
            for (int e = 0; e < EPT; ++e) r_loc += residual_of(pr[e], qr[e], af, bf);
            r_loc = wave_reduce<kOpSum>(r_loc);
            if (lane == 0) sh.part[par][wave][0] = r_loc;
            __syncthreads();
            if (wave == 0) {
                float mine[1], got[1];
                mine[0] = fold_waves<kOpSum>(sh, par, 0, 0.f);
                const bool ok = exchange<1>(p, tag_base, ++step, mine, 0.f, got);
                if (lane == 0) sh.fail = ok ? 0 : 1;
                if (ok) find_bonus_owner(p, u0, got[0], sh);
            }
            __syncthreads();
            if (sh.fail) { finish(p, path_len, sh.st.n_dec, 1, v, sh.st.fallbacks, sh.st.degenerate); return; }
        }
        const double total = sh.bonus_d[0], before = sh.bonus_d[1];
        const double goal = (double)u0 * total;
        const int owner = sh.bonus_i[0];
        const bool pick_last = sh.bonus_i[1] != 0;
        if (wg_rank() == owner) {
            if (tid == 0) { sh.cand_min = 0x7FFFFFFF; sh.cand_max = -1; }
            float r[EPT];
            double mine = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) { r[e] = residual_of(pr[e], qr[e], af, bf); mine += (double)r[e]; }
            // exclusive prefix of the per-thread masses over the block
            const double incl = wave_scan(mine);
            if (lane == 63) sh.scan[wave] = incl;
            __syncthreads();
            double run = before + incl - mine;
            for (int w = 0; w < wave; ++w) run += sh.scan[w];
            int found = 0x7FFFFFFF, last_pos = -1;
            double lo = 0.0, hi = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const double prev = run;
                run += (double)r[e];
                if (found == 0x7FFFFFFF && !pick_last && run > goal) { found = base + e; lo = prev; hi = run; }
                if (r[e] > 0.f) last_pos = base + e;
            }
            // one shared-memory atomic per wavefront, not per element
            const int wave_found = wave_min(found), wave_last = wave_max(last_pos);
            if (lane == 0) {
                if (wave_found != 0x7FFFFFFF) atomicMin(&sh.cand_min, wave_found);
                if (wave_last >= 0) atomicMax(&sh.cand_max, wave_last);
            }
            __syncthreads();
            int pick = sh.cand_min;
            if (pick == 0x7FFFFFFF) pick = sh.cand_max >= 0 ? sh.cand_max : min(V - 1, base);
            float* binfo = reinterpret_cast<float*>(p.trace + SEQ_TRACE_HEADER_INTS +
                                                    SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS);
            if (found == pick) {
                binfo[0] = u0; binfo[1] = (float)total;
                binfo[2] = (float)(lo / total); binfo[3] = (float)(hi / total);
            } else if (sh.cand_min == 0x7FFFFFFF && tid == 0) {
                binfo[0] = u0; binfo[1] = (float)total; binfo[2] = 1.f; binfo[3] = 1.f;
            }
            if (tid == 0) p.bonus[0] = pick;
        }
        SEQ_STAMP(20);
        finish(p, path_len, sh.st.n_dec, 0, v, sh.st.fallbacks, sh.st.degenerate);
        return;
    }
}

// Greedy decoding (T = 0): P and Q are one-hot, and Algorithm 2 as written then accepts a child
// exactly when its token is the arg-max of the target row (lowest index on ties) -- a token
// with D[s] = 0 is accepted iff R[s] > 0, the residual stays one-hot through every rejection,
// and the draft falls back to uniform once its single token has been rejected.  The bonus token
// is the arg-max at the node where the walk stops.  Only the target rows are read.
template <typename LT, int EPT, bool BATCHED>
__global__ __launch_bounds__(kThreads) void verify_greedy_kernel(const VerifyParams p_in) {
    const VerifyParams p = BATCHED ? params_of_sequence(p_in, blockIdx.y, true) : p_in;
    __shared__ Shared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int base = (wg_rank() * kThreads + tid) * EPT;
    const LT* target = static_cast<const LT*>(p.target);
    const int V = p.V;
    constexpr int kNone = 0x7FFFFFFF;
    bool poisoned;
    const uint32_t tag_base = launch_tag_base(p, &poisoned);
    begin_trace(p);
    if (poisoned) { finish(p, 0, 0, 1, 0, 0, 0); return; }
    stage_tree(p, sh);
    __syncthreads();
    uint32_t step = 0;
    int v = 0, path_len = 0, n_dec = 0;
    auto better = [](float ov, int ox, float bv, int bx) {   // larger value, lower index on ties
        return ox != kNone && (bx == kNone || ov > bv || (ov == bv && ox < bx));
    };
    for (;;) {
        const LT* trow = target + (size_t)v * V;
        float best = -INFINITY;
        int best_x = kNone;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int x = base + e;
            if (x < V) {
                const float val = load_logit<LT>(trow, x);
                if (better(val, x, best, best_x)) { best = val; best_x = x; }
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(best, off);
            const int ox = __shfl_xor(best_x, off);
            if (better(ov, ox, best, best_x)) { best = ov; best_x = ox; }
        }
        if (lane == 0) { sh.red_f[wave] = best; sh.red_i[wave] = best_x; }
        __syncthreads();
        if (wave == 0) {
            best = sh.red_f[0]; best_x = sh.red_i[0];
            for (int w = 1; w < kWaves; ++w)
                if (better(sh.red_f[w], sh.red_i[w], best, best_x)) { best = sh.red_f[w]; best_x = sh.red_i[w]; }
            float mine[2] = {best, __int_as_float(best_x)}, got[2];
            const bool ok = exchange<2>(p, tag_base, ++step, mine, __int_as_float(kNone), got);
            float top = lane < p.W ? got[0] : -INFINITY;
            int top_x = lane < p.W ? __float_as_int(got[1]) : kNone;
            for (int off = 32; off > 0; off >>= 1) {
                const float ov = __shfl_xor(top, off);
                const int ox = __shfl_xor(top_x, off);
                if (better(ov, ox, top, top_x)) { top = ov; top_x = ox; }
            }
            if (lane == 0) { sh.fail = ok ? 0 : 1; sh.cand_min = top_x; }
        } else {
            ++step;
        }
        __syncthreads();
        if (sh.fail) { finish(p, path_len, n_dec, 1, v, 0, 0); return; }
        const int top_x = sh.cand_min;
        int next = -1;
        const int c_begin = sh.child_start[v], c_end = sh.child_start[v + 1];
        for (int ci = c_begin; ci < c_end; ++ci) {
            const int c = sh.child_list[ci];
            const bool accept = sh.token[c] == top_x;
            record(p, n_dec, c, accept, accept ? 1.f : 0.f, sh.uniform[c]);
            ++n_dec;
            if (accept) { next = c; break; }
        }
        if (next >= 0) {
            if (wg_rank() == 0 && tid == 0) p.path[path_len] = next;
            ++path_len;
            v = next;
            __syncthreads();  // sh.cand_min and the wave partials are rewritten at the next node
            continue;
        }
        if (wg_rank() == 0 && tid == 0) p.bonus[0] = top_x;
        finish(p, path_len, n_dec, 0, v, 0, 0);
        return;
    }
}

uint32_t g_spin_limit = 1u << 22;

// One team of p.W workgroups per sequence; `batch` > 1 puts the teams of that many sequences
// side by side in one launch (grid.y).  The caller keeps p.W * batch within what the chip holds
// at once: a team waits for its own members only, but they must all be running.
template <typename LT>
void launch_verify(const VerifyParams& p, bool greedy, hipStream_t stream, int batch) {
    const dim3 grid((unsigned)p.W, (unsigned)batch), block(kThreads);
    if (batch > 1) {
        if (greedy) hipLaunchKernelGGL((verify_greedy_kernel<LT, 8, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((verify_walk_kernel<LT, 8, true>), grid, block, 0, stream, p);
    } else {
        if (greedy) hipLaunchKernelGGL((verify_greedy_kernel<LT, 8, false>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((verify_walk_kernel<LT, 8, false>), grid, block, 0, stream, p);
    }
}

}  // namespace
}  // namespace seqtree

using namespace seqtree;

// Test hook (not part of the public header): bound of the inter-workgroup wait, in polls.
#ifdef SEQTREE_STAMPS
extern "C" int seqtree_internal_read_stamps(long long* out) {
    int count = 0;
    (void)hipMemcpyFromSymbol(&count, HIP_SYMBOL(g_stamp_count), sizeof(int));
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_stamps), sizeof(long long) * 64);
    return count;
}
#endif
extern "C" void seqtree_internal_set_spin_limit(uint32_t polls) { g_spin_limit = polls; }
// Test hook: 0 = choose by vocabulary size, 1 = always the lazy walk, 2 = the per-node kernel
// wherever the vocabulary allows it.
static int g_verify_mode = 0;
extern "C" void seqtree_internal_set_verify_mode(int mode) { g_verify_mode = mode; }
// Test hook for SEQ_VERIFY_TOPK: 0 = the library chooses, 1 = every node draws at once, 2 = one
// workgroup draws where the walk goes.
extern "C" void seqtree_internal_set_topk_mode(int mode) { set_topk_mode(mode); }

extern "C" size_t seq_verify_workspace(int32_t n_tree, int32_t vocab, int32_t dtype) {
    (void)n_tree; (void)vocab; (void)dtype;
    return kVerifyWorkspaceBytes;
}

extern "C" int seq_verify(const void* target_logits, const void* draft_logits,
                          const int32_t* tree_tokens, const int32_t* parent, float temperature,
                          const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
                          int32_t n_tree, int32_t vocab, int32_t dtype, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    return seq_verify_with(SEQ_VERIFY_SEQUOIA, target_logits, draft_logits, tree_tokens, parent, temperature,
                           uniforms, accepted_path, bonus_token, n_tree, vocab, dtype, workspace,
                           workspace_bytes, hip_stream);
}

extern "C" int seq_verify_with(int32_t algorithm, const void* target_logits, const void* draft_logits,
                               const int32_t* tree_tokens, const int32_t* parent, float temperature,
                               const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
                               int32_t n_tree, int32_t vocab, int32_t dtype, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
    return seq_verify_batched(algorithm, 1, target_logits, draft_logits, tree_tokens, parent, temperature, uniforms,
                              accepted_path, bonus_token, n_tree, vocab, dtype, workspace, workspace_bytes, hip_stream);
}

extern "C" int seq_verify_batched(int32_t algorithm, int32_t batch, const void* target_logits, const void* draft_logits,
                                  const int32_t* tree_tokens, const int32_t* parent, float temperature,
                                  const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
                                  int32_t n_tree, int32_t vocab, int32_t dtype, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
    if (algorithm != SEQ_VERIFY_SEQUOIA && algorithm != SEQ_VERIFY_SPECINFER && algorithm != SEQ_VERIFY_TOPK)
        return SEQ_ERR_ALGORITHM;
    if (!target_logits || (!draft_logits && algorithm != SEQ_VERIFY_TOPK) || !tree_tokens || !parent ||
        !uniforms || !accepted_path || !bonus_token)
        return SEQ_ERR_NULL;
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE || vocab < 2 || vocab > SEQ_MAX_VOCAB || batch < 1 || batch > kVerifyMaxBatch)
        return SEQ_ERR_SHAPE;
    if (!(temperature >= 0.0f) || std::isinf(temperature)) return SEQ_ERR_TEMPERATURE;
    int rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    const size_t per_sequence = seq_verify_workspace(n_tree, vocab, dtype);
    if (!workspace || workspace_bytes < per_sequence * (size_t)batch ||
        (reinterpret_cast<uintptr_t>(workspace) & 15) != 0)
        return SEQ_ERR_WORKSPACE;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    TreePlan plan;
    rc = get_tree_plan(parent, n_tree, stream, &plan);
    if (rc != SEQ_OK) return rc;
    SyncArea* sync = nullptr;
    rc = get_sync_area(stream, &sync);
    if (rc != SEQ_OK) return rc;

    constexpr int ept = 8;  // kVerifyMaxGroups * kThreads * 8 = SEQ_MAX_VOCAB
    static_assert((long long)kVerifyMaxGroups * kThreads * 8 >= SEQ_MAX_VOCAB, "vocabulary limit");
    VerifyParams p;
    p.target = target_logits;
    p.draft = draft_logits;
    p.tokens = tree_tokens;
    p.uniforms = uniforms;
    p.child_start = plan.child_start;
    p.child_list = plan.child_list;
    p.path = accepted_path;
    p.bonus = bonus_token;
    p.trace = static_cast<int32_t*>(workspace);
    p.records = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + kTraceBytesPadded);
    p.arrivals = sync->verify_arrivals;
    p.slots = sync->verify_slots;
    p.epoch = sync->verify_epoch;
    p.poison = sync->verify_epoch + 1;
    p.spin_limit = g_spin_limit;
    p.n = n_tree;
    p.V = vocab;
    p.W = (vocab + kThreads * ept - 1) / (kThreads * ept);
    const bool greedy = temperature == 0.0f;
    p.inv_T = greedy ? 1.0f : 1.0f / temperature;
    p.with_replacement = algorithm == SEQ_VERIFY_SPECINFER;
    const size_t elt = dtype == SEQ_BF16 ? 2 : 4;
    p.batch_logit_bytes = (size_t)n_tree * vocab * elt;
    p.batch_workspace_bytes = per_sequence;
    p.batch_ctl = sync->verify_batch_ctl;
    p.batch_slots = sync->verify_batch_slots;
    p.chain_area = sync->chain_area;
    p.chain_records = chain_records_of(sync->chain_area);
    p.team_slots = team_slots_of(sync->chain_area);
    p.internal_nodes = plan.internal_nodes;
    p.n_internal = plan.n_internal;
    p.team_xcd = sync->round_robin_xcds ? 1 : 0;
    // Sampling with a vocabulary one workgroup can hold, and a tree whose nodes all find a CU at
    // once: all nodes at once -- of as many sequences of the batch as still fit.  Otherwise (and
    // for greedy decoding, which needs one arg-max per visited node) the lazy walk.
    // (T = 0: all three algorithms accept a child exactly when its token is the target's arg-max
    // and emit that arg-max, so the greedy kernel serves them all.)
    // (one workgroup of 1024 threads fits a compute unit at a time: the device's count of them is
    // how many workgroups run at once)
    const int at_once = sync->compute_units;
    bool per_node_kernel = !greedy && algorithm != SEQ_VERIFY_TOPK && vocab <= kChainsMaxVocab &&
                           g_verify_mode != 1 && (n_tree <= at_once || g_verify_mode == 2);
    // Larger vocabularies, one sequence: a team of workgroups per node that has children.  Worth
    // it while every member finds a compute unit of its own (64 nodes over 128256 tokens, 32 teams
    // of 8: 25.5 us against 27.5 us for the lazy walk where the walk is short, 31 against 41 us
    // where it runs to a leaf); with two members to a unit the lazy walk is faster again (128
    // nodes: 32.2 against 29.9 us), and beyond that by far (768 nodes: 104 against 39 us).
    const int team_w = team_size_for(vocab);
    const bool per_node_teams = !greedy && algorithm != SEQ_VERIFY_TOPK && vocab > kChainsMaxVocab && batch == 1 &&
                                plan.n_internal > 0 && g_verify_mode != 1 &&
                                (plan.n_internal * team_w <= at_once || g_verify_mode == 2);
    if (per_node_teams) {
        VerifyParams q = p;
        q.W = team_w;
        launch_verify_chains_team(q, dtype, stream);
        return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
    }
    const bool topk_draws = algorithm == SEQ_VERIFY_TOPK && !greedy;
    // sequences per launch: as many as find a CU for every workgroup they need -- a workgroup per
    // node in the per-node kernel, a team of W in the lazy walk (whose members wait for each
    // other, so all of them must be running); the top-k draws, which wait for nobody, all of them
    // (their records share the area's SEQ_MAX_TREE node records)
    const int per_launch_nodes = std::max(1, std::min(at_once, SEQ_MAX_TREE) / n_tree);
    const int per_launch_teams = std::min(kWalkMaxBatch, std::max(1, at_once / p.W));
    // A batch that the per-node kernel needs more launches for than the teams do goes to the
    // teams: a launch of either costs about the same whatever it holds (64 nodes, 32000 tokens:
    // 4 sequences per per-node launch of 22 us; 16 sequences as teams 42 us, 64 sequences 55 us).
    if (per_node_kernel && g_verify_mode != 2 &&
        (batch + per_launch_nodes - 1) / per_launch_nodes > (batch + per_launch_teams - 1) / per_launch_teams)
        per_node_kernel = false;
    const int group = topk_draws ? batch : per_node_kernel ? per_launch_nodes : per_launch_teams;
    for (int b = 0; b < batch; b += group) {      // one group of sequences after the other on the stream
        const int count = std::min(group, batch - b);
        VerifyParams q = p;
        q.target = static_cast<const char*>(target_logits) + (size_t)b * p.batch_logit_bytes;
        q.draft = draft_logits ? static_cast<const char*>(draft_logits) + (size_t)b * p.batch_logit_bytes : nullptr;
        q.tokens = tree_tokens + (size_t)b * n_tree;
        q.uniforms = uniforms + (size_t)b * n_tree;
        q.path = accepted_path + (size_t)b * n_tree;
        q.bonus = bonus_token + b;
        q.trace = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + (size_t)b * per_sequence);
        q.records = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + (size_t)b * per_sequence + kTraceBytesPadded);
        if (topk_draws) launch_verify_topk(q, dtype, stream, count);
        else if (per_node_kernel) launch_verify_chains(q, dtype, stream, count);
        else if (dtype == SEQ_BF16) launch_verify<uint16_t>(q, greedy, stream, count);
        else launch_verify<float>(q, greedy, stream, count);
    }
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
