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
// the remaining draft) is one block reduction per workgroup followed by one all-to-all exchange
// of the per-workgroup partials through tagged 64-bit slots in global memory; every workgroup
// then combines the same partials in the same order, so all of them take identical decisions
// without a leader.  Waiting is bounded: a workgroup that does not see its peers within
// `spin_limit` polls records status 1 in the trace and leaves.
//
// Residual and draft are never rewritten.  After j rejections at a node, with S the rejected
// tokens (whose p and q registers are set to zero when they are rejected):
//     D_j[x] = q[x] / massQ,   massQ = sum_x q[x]                       (or 1/(V-|S|) off S once
//                                                                        massQ has reached 0)
//     R_j[x] = max(p[x] - A q[x] - B, 0) / W
// where A (resp. B) accumulates W / massQ (resp. W / (V-|S|)) at every rejection and W is the
// vocabulary sum of the numerator.  This is the update R <- norm(max(R - D, 0)) unrolled: the
// nested max(., 0) collapse because the subtracted amounts never decrease.  A rejection thus
// costs one read-only pass over registers and one exchange.
#include <cmath>

#include "seq_internal.h"

namespace seqtree {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

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
    unsigned long long* slots;
    uint32_t* epoch;
    uint32_t spin_limit;
    int n, V, W;
    float inv_T;
};

template <typename LT> __device__ __forceinline__ float load_logit(const LT* row, int x);
template <> __device__ __forceinline__ float load_logit<float>(const float* row, int x) { return row[x]; }
template <> __device__ __forceinline__ float load_logit<uint16_t>(const uint16_t* row, int x) {
    return __uint_as_float((uint32_t)row[x] << 16);
}

struct Shared {
    float gath[kVerifyMaxGroups][kVerifySlotWords];
    double red_d[kWavesPerBlock];
    float red_f[kWavesPerBlock];
    int red_i[kWavesPerBlock];
    double res_d[4];
    float res_f[2];
    int res_i[2];
    int fail;
    int cand_min;
    int cand_max;
    int rejected[SEQ_MAX_TREE];
};

__device__ __forceinline__ float block_max(float v, Shared& sh) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.red_f[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sh.red_f[0];
    for (int w = 1; w < kWavesPerBlock; ++w) r = fmaxf(r, sh.red_f[w]);
    return r;
}

__device__ __forceinline__ double block_sum(double v, Shared& sh) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.red_d[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = sh.red_d[0];
    for (int w = 1; w < kWavesPerBlock; ++w) r += sh.red_d[w];
    return r;
}

// All-to-all of K floats per workgroup.  Afterwards sh.gath[w][k] holds workgroup w's k-th
// value in every workgroup.  Two slot buffers alternate by round parity: a workgroup can be at
// most one round ahead of the slowest one, because it cannot finish a round without that
// workgroup's contribution.
template <int K>
__device__ __forceinline__ bool exchange(const VerifyParams& p, uint32_t tag_base, uint32_t round,
                                         float v0, float v1, float v2, float v3, Shared& sh) {
    const uint32_t tag = tag_base + round;
    unsigned long long* buf = p.slots + (size_t)(round & 1u) * kVerifyMaxGroups * kVerifySlotWords;
    const int tid = threadIdx.x;
    __syncthreads();  // everyone is done reading sh.gath of the previous exchange
    if (tid < K) {
        const float mine = tid == 0 ? v0 : (tid == 1 ? v1 : (tid == 2 ? v2 : v3));
        const unsigned long long word = ((unsigned long long)tag << 32) | __float_as_uint(mine);
        __hip_atomic_store(&buf[blockIdx.x * kVerifySlotWords + tid], word, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < 64) {
        bool done = tid >= p.W;
        float got[K];
#pragma unroll
        for (int k = 0; k < K; ++k) got[k] = 0.f;
        uint32_t spins = 0;
        for (;;) {
            if (!done) {
                bool all = true;
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    const unsigned long long word = __hip_atomic_load(
                        &buf[tid * kVerifySlotWords + k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((uint32_t)(word >> 32) == tag) got[k] = __uint_as_float((uint32_t)word);
                    else all = false;
                }
                done = all;
            }
            if (__all(done)) break;
            if (++spins > p.spin_limit) break;   // bounded wait: every wave leaves this loop
            __builtin_amdgcn_s_sleep(2);
        }
        const bool ok = __all(done);
        if (tid < p.W) {
#pragma unroll
            for (int k = 0; k < K; ++k) sh.gath[tid][k] = got[k];
        }
        if (tid == 0) sh.fail = ok ? 0 : 1;
    }
    __syncthreads();
    return sh.fail == 0;
}


// Tags must differ from launch to launch (also when a captured graph replays the same kernel
// arguments) and agree between the workgroups of one launch.  Every launch has exactly
// kVerifyMaxGroups workgroups and each takes one ticket from a device counter, so
// ticket / kVerifyMaxGroups numbers the launch whatever happened to earlier ones.
__device__ __forceinline__ uint32_t launch_tag_base(const VerifyParams& p, Shared& sh) {
    if (threadIdx.x == 0) sh.res_i[0] = (int)atomicAdd(p.epoch, 1u);
    __syncthreads();
    const uint32_t ticket = (uint32_t)sh.res_i[0];
    __syncthreads();
    return (ticket / (uint32_t)kVerifyMaxGroups) * (uint32_t)kVerifyTagsPerCall;
}

__device__ __forceinline__ double wave_sum(double v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// The per-workgroup partials sit in sh.gath; the first wavefront folds them (lane w takes
// workgroup w, butterfly order, identical in every workgroup) and leaves the results in shared
// memory for the whole block.
__device__ __forceinline__ void fold_softmax_stats(const VerifyParams& p, Shared& sh) {
    const int tid = threadIdx.x;
    if (tid < 64) {
        const bool have = tid < p.W;
        const float m_t = have ? sh.gath[tid][0] : -INFINITY, z_t = have ? sh.gath[tid][1] : 0.f;
        const float m_d = have ? sh.gath[tid][2] : -INFINITY, z_d = have ? sh.gath[tid][3] : 0.f;
        float mt = m_t, md = m_d;
        for (int off = 32; off > 0; off >>= 1) {
            mt = fmaxf(mt, __shfl_xor(mt, off));
            md = fmaxf(md, __shfl_xor(md, off));
        }
        const double zt = wave_sum(z_t > 0.f ? (double)z_t * (double)expf(m_t - mt) : 0.0);
        const double zd = wave_sum(z_d > 0.f ? (double)z_d * (double)expf(m_d - md) : 0.0);
        if (tid == 0) { sh.res_f[0] = mt; sh.res_f[1] = md; sh.res_d[0] = zt; sh.res_d[1] = zd; }
    }
    __syncthreads();
}

__device__ __forceinline__ void fold_sums(const VerifyParams& p, Shared& sh) {
    const int tid = threadIdx.x;
    if (tid < 64) {
        const bool have = tid < p.W;
        const double a = wave_sum(have ? (double)sh.gath[tid][0] : 0.0);
        const double b = wave_sum(have ? (double)sh.gath[tid][1] : 0.0);
        if (tid == 0) { sh.res_d[0] = a; sh.res_d[1] = b; }
    }
    __syncthreads();
}

// Which workgroup holds the token at cumulative mass u * total?  res_d[0] = total,
// res_d[1] = mass before the owner, res_i[0] = owner, res_i[1] = 1 if rounding left no owner
// and the last workgroup with mass was taken instead.
__device__ __forceinline__ void fold_bonus_owner(const VerifyParams& p, float u0, Shared& sh) {
    const int tid = threadIdx.x;
    if (tid < 64) {
        const double sw = tid < p.W ? (double)sh.gath[tid][0] : 0.0;
        double incl = sw;
        for (int off = 1; off < 64; off <<= 1) {
            const double t = __shfl_up(incl, off);
            if (tid >= off) incl += t;
        }
        const double total = __shfl(incl, 63);
        const double goal = (double)u0 * total;
        const unsigned long long hit = __ballot(sw > 0.0 && incl > goal);
        const unsigned long long pos = __ballot(sw > 0.0);
        int owner, forced = 0;
        if (hit) owner = __ffsll((long long)hit) - 1;
        else { forced = 1; owner = pos ? 63 - __clzll((long long)pos) : p.W - 1; }
        const double before = __shfl(incl - sw, owner);
        if (tid == 0) { sh.res_d[0] = total; sh.res_d[1] = before; sh.res_i[0] = owner; sh.res_i[1] = forced; }
    }
    __syncthreads();
}

__device__ __forceinline__ float prob_of(float scaled_logit, float m, float inv_z) {
    return scaled_logit == -INFINITY ? 0.f : expf(scaled_logit - m) * inv_z;
}

__device__ __forceinline__ float residual_of(float p, float q, float a, float b) {
    return fmaxf(fmaf(-a, q, p) - b, 0.f);
}

__device__ __forceinline__ void finish(const VerifyParams& p, int path_len, int n_dec, int status,
                                       int stop_node, int fallbacks, int degenerate) {
    if (blockIdx.x != 0) return;
    for (int i = path_len + (int)threadIdx.x; i < p.n; i += kThreads) p.path[i] = -1;
    if (threadIdx.x == 0) {
        p.trace[0] = n_dec;
        p.trace[1] = status;
        p.trace[2] = stop_node;
        p.trace[3] = fallbacks;
        p.trace[4] = degenerate;
        p.trace[5] = p.trace[6] = p.trace[7] = 0;
        if (status != 0) p.bonus[0] = -1;
    }
}

__device__ __forceinline__ void record(const VerifyParams& p, int n_dec, int node, bool accepted,
                                       float ratio, float u) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        int32_t* rec = p.trace + SEQ_TRACE_HEADER_INTS + n_dec * SEQ_TRACE_RECORD_WORDS;
        rec[0] = node;
        rec[1] = accepted ? 1 : 0;
        rec[2] = __float_as_int(ratio);
        rec[3] = __float_as_int(u);
    }
}

template <typename LT, int EPT>
__global__ __launch_bounds__(kThreads) void verify_walk_kernel(const VerifyParams p) {
    __shared__ Shared sh;
    const int tid = threadIdx.x;
    const int base = ((int)blockIdx.x * kThreads + tid) * EPT;  // my EPT consecutive tokens
    const LT* target = static_cast<const LT*>(p.target);
    const LT* draft = static_cast<const LT*>(p.draft);
    const int V = p.V;

    const uint32_t tag_base = launch_tag_base(p, sh);
    if ((int)blockIdx.x >= p.W) return;
    float pr[EPT], qr[EPT];
    uint32_t round = 0;
    int v = 0, path_len = 0, n_dec = 0, fallbacks = 0, degenerate = 0;

    for (;;) {
        const LT* trow = target + (size_t)v * V;
        const LT* drow = draft + (size_t)v * V;
        // tempered logits of my tokens, then the two softmax statistics
        float mt_loc = -INFINITY, md_loc = -INFINITY;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int x = base + e;
            pr[e] = x < V ? load_logit<LT>(trow, x) * p.inv_T : -INFINITY;
            qr[e] = x < V ? load_logit<LT>(drow, x) * p.inv_T : -INFINITY;
            mt_loc = fmaxf(mt_loc, pr[e]);
            md_loc = fmaxf(md_loc, qr[e]);
        }
        const float mt_blk = block_max(mt_loc, sh);
        const float md_blk = block_max(md_loc, sh);
        double zt_loc = 0.0, zd_loc = 0.0;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            zt_loc += (double)prob_of(pr[e], mt_blk, 1.0f);
            zd_loc += (double)prob_of(qr[e], md_blk, 1.0f);
        }
        const float zt_blk = (float)block_sum(zt_loc, sh);
        const float zd_blk = (float)block_sum(zd_loc, sh);
        if (!exchange<4>(p, tag_base, ++round, mt_blk, zt_blk, md_blk, zd_blk, sh)) {
            finish(p, path_len, n_dec, 1, v, fallbacks, degenerate);
            return;
        }
        fold_softmax_stats(p, sh);
        const float mt = sh.res_f[0], md = sh.res_f[1];
        const double zt = sh.res_d[0], zd = sh.res_d[1];
        const float inv_zt = (float)(1.0 / zt), inv_zd = (float)(1.0 / zd);
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            pr[e] = prob_of(pr[e], mt, inv_zt);
            qr[e] = prob_of(qr[e], md, inv_zd);
        }

        // Algorithm 2 at node v
        double A = 0.0, B = 0.0, Wn = 1.0, massQ = 1.0;
        bool fallback = false, sums_valid = false;
        int n_rej = 0, next = -1;
        const int c_begin = p.child_start[v], c_end = p.child_start[v + 1];
        for (int ci = c_begin; ci < c_end; ++ci) {
            const int c = p.child_list[ci];
            const int s = min(max(p.tokens[c], 0), V - 1);  // stay inside the row whatever the caller sent
            const float u = p.uniforms[c];
            const float ps = prob_of(load_logit<LT>(trow, s) * p.inv_T, mt, inv_zt);
            const float qs = prob_of(load_logit<LT>(drow, s) * p.inv_T, md, inv_zd);
            bool in_s = false;
            for (int k = 0; k < n_rej; ++k) in_s |= (sh.rejected[k] == s);
            const int left = V - n_rej;  // tokens not yet rejected
            const double rs = in_s ? 0.0 : (double)residual_of(ps, qs, (float)A, (float)B) / Wn;
            const double ds = in_s ? 0.0
                                   : (fallback ? (left > 0 ? 1.0 / (double)left : 0.0) : (double)qs / massQ);
            const double ratio = ds > 0.0 ? rs / ds : (rs > 0.0 ? (double)INFINITY : 0.0);
            const bool accept = (double)u < ratio;
            record(p, n_dec, c, accept, (float)ratio, u);
            ++n_dec;
            if (accept) { next = c; break; }

            // rejected: R <- norm(max(R - D, 0)), then D[s] <- 0 (and the uniform fallback)
            double dA = 0.0, dB = 0.0;
            if (fallback) { if (left > 0) dB = Wn / (double)left; }
            else dA = Wn / massQ;
            A += dA;
            B += dB;
            if (!in_s) {
#pragma unroll
                for (int e = 0; e < EPT; ++e)
                    if (base + e == s) { pr[e] = 0.f; qr[e] = 0.f; }
                if (tid == 0) sh.rejected[n_rej] = s;
                ++n_rej;
            }
            const float af = (float)A, bf = (float)B;
            double r_loc = 0.0, q_loc = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                r_loc += (double)residual_of(pr[e], qr[e], af, bf);
                q_loc += (double)qr[e];
            }
            const float r_blk = (float)block_sum(r_loc, sh);
            const float q_blk = (float)block_sum(q_loc, sh);
            if (!exchange<2>(p, tag_base, ++round, r_blk, q_blk, 0.f, 0.f, sh)) {
                finish(p, path_len, n_dec, 1, v, fallbacks, degenerate);
                return;
            }
            fold_sums(p, sh);
            const double w_new = sh.res_d[0], q_new = sh.res_d[1];
            if (w_new > 0.0) { Wn = w_new; sums_valid = true; }
            else { A -= dA; B -= dB; ++degenerate; sums_valid = false; }  // R stays as it was
            massQ = q_new;
            if (!fallback && !(massQ > 0.0)) { fallback = true; ++fallbacks; }
        }
        if (next >= 0) {
            if (blockIdx.x == 0 && tid == 0) p.path[path_len] = next;
            ++path_len;
            v = next;
            continue;
        }

        // no child accepted: bonus token ~ R by inverse CDF with uniforms[0]
        const float af = (float)A, bf = (float)B;
        if (!sums_valid) {
            double r_loc = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) r_loc += (double)residual_of(pr[e], qr[e], af, bf);
            const float r_blk = (float)block_sum(r_loc, sh);
            if (!exchange<1>(p, tag_base, ++round, r_blk, 0.f, 0.f, 0.f, sh)) {
                finish(p, path_len, n_dec, 1, v, fallbacks, degenerate);
                return;
            }
        }
        const float u0 = p.uniforms[0];
        fold_bonus_owner(p, u0, sh);
        const double total = sh.res_d[0], before = sh.res_d[1];
        const double goal = (double)u0 * total;
        const int owner = sh.res_i[0];
        const bool pick_last = sh.res_i[1] != 0;
        if ((int)blockIdx.x == owner) {
            if (tid == 0) { sh.cand_min = 0x7FFFFFFF; sh.cand_max = -1; }
            float r[EPT];
            double mine = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) { r[e] = residual_of(pr[e], qr[e], af, bf); mine += (double)r[e]; }
            // exclusive prefix of the per-thread masses over the block
            double incl = mine;
            for (int off = 1; off < 64; off <<= 1) {
                const double t = __shfl_up(incl, off);
                if ((tid & 63) >= off) incl += t;
            }
            __syncthreads();
            if ((tid & 63) == 63) sh.red_d[tid >> 6] = incl;
            __syncthreads();
            double run = before + incl - mine;
            for (int w = 0; w < (tid >> 6); ++w) run += sh.red_d[w];
            int found = -1;
            double lo = 0.0, hi = 0.0;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const double prev = run;
                run += (double)r[e];
                if (found < 0 && !pick_last && run > goal) { found = base + e; lo = prev; hi = run; }
                if (r[e] > 0.f) atomicMax(&sh.cand_max, base + e);
            }
            if (found >= 0) atomicMin(&sh.cand_min, found);
            __syncthreads();
            int pick = sh.cand_min;
            if (pick == 0x7FFFFFFF) pick = sh.cand_max >= 0 ? sh.cand_max : min(V - 1, base);
            float* binfo = reinterpret_cast<float*>(p.trace + SEQ_TRACE_HEADER_INTS +
                                                    SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS);
            if (found >= 0 && found == pick) {
                binfo[0] = u0; binfo[1] = (float)total;
                binfo[2] = (float)(lo / total); binfo[3] = (float)(hi / total);
            } else if (sh.cand_min == 0x7FFFFFFF && tid == 0) {
                binfo[0] = u0; binfo[1] = (float)total; binfo[2] = 1.f; binfo[3] = 1.f;
            }
            if (tid == 0) p.bonus[0] = pick;
        }
        finish(p, path_len, n_dec, 0, v, fallbacks, degenerate);
        return;
    }
}

// Greedy decoding (T = 0): P and Q are one-hot, and Algorithm 2 as written then accepts a child
// exactly when its token is the arg-max of the target row (lowest index on ties) -- a token
// with D[s] = 0 is accepted iff R[s] > 0, the residual stays one-hot through every rejection,
// and the draft falls back to uniform once its single token has been rejected.  The bonus token
// is the arg-max at the node where the walk stops.  Only the target rows are read.
template <typename LT, int EPT>
__global__ __launch_bounds__(kThreads) void verify_greedy_kernel(const VerifyParams p) {
    __shared__ Shared sh;
    const int tid = threadIdx.x;
    const int base = ((int)blockIdx.x * kThreads + tid) * EPT;
    const LT* target = static_cast<const LT*>(p.target);
    const int V = p.V;
    const uint32_t tag_base = launch_tag_base(p, sh);
    if ((int)blockIdx.x >= p.W) return;
    uint32_t round = 0;
    int v = 0, path_len = 0, n_dec = 0;
    for (;;) {
        const LT* trow = target + (size_t)v * V;
        float best = -INFINITY;
        int best_x = 0x7FFFFFFF;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int x = base + e;
            if (x < V) {
                const float val = load_logit<LT>(trow, x);
                if (val > best || best_x == 0x7FFFFFFF) { best = val; best_x = x; }
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(best, off);
            const int ox = __shfl_xor(best_x, off);
            if (ov > best || (ov == best && ox < best_x)) { best = ov; best_x = ox; }
        }
        __syncthreads();
        if ((tid & 63) == 0) { sh.red_f[tid >> 6] = best; sh.red_i[tid >> 6] = best_x; }
        __syncthreads();
        best = sh.red_f[0]; best_x = sh.red_i[0];
        for (int w = 1; w < kWavesPerBlock; ++w)
            if (sh.red_f[w] > best || (sh.red_f[w] == best && sh.red_i[w] < best_x)) {
                best = sh.red_f[w]; best_x = sh.red_i[w];
            }
        if (!exchange<2>(p, tag_base, ++round, best, __int_as_float(best_x), 0.f, 0.f, sh)) {
            finish(p, path_len, n_dec, 1, v, 0, 0);
            return;
        }
        float top = -INFINITY;
        int top_x = 0x7FFFFFFF;
        for (int w = 0; w < p.W; ++w) {
            const float ov = sh.gath[w][0];
            const int ox = __float_as_int(sh.gath[w][1]);
            if (ox == 0x7FFFFFFF) continue;  // workgroup owns no token
            if (top_x == 0x7FFFFFFF || ov > top || (ov == top && ox < top_x)) { top = ov; top_x = ox; }
        }
        int next = -1;
        const int c_begin = p.child_start[v], c_end = p.child_start[v + 1];
        for (int ci = c_begin; ci < c_end; ++ci) {
            const int c = p.child_list[ci];
            const bool accept = p.tokens[c] == top_x;
            record(p, n_dec, c, accept, accept ? 1.f : 0.f, p.uniforms[c]);
            ++n_dec;
            if (accept) { next = c; break; }
        }
        if (next >= 0) {
            if (blockIdx.x == 0 && tid == 0) p.path[path_len] = next;
            ++path_len;
            v = next;
            continue;
        }
        if (blockIdx.x == 0 && tid == 0) p.bonus[0] = top_x;
        finish(p, path_len, n_dec, 0, v, 0, 0);
        return;
    }
}

uint32_t g_spin_limit = 1u << 22;

template <typename LT>
void launch_verify(const VerifyParams& p, bool greedy, int ept, hipStream_t stream) {
    const dim3 grid((unsigned)kVerifyMaxGroups), block(kThreads);  // workgroups >= W only take a ticket
#define SEQ_LAUNCH(E)                                                                          \
    do {                                                                                       \
        if (greedy) hipLaunchKernelGGL((verify_greedy_kernel<LT, E>), grid, block, 0, stream, p); \
        else hipLaunchKernelGGL((verify_walk_kernel<LT, E>), grid, block, 0, stream, p);       \
    } while (0)
    if (ept == 8) SEQ_LAUNCH(8);
    else if (ept == 16) SEQ_LAUNCH(16);
    else SEQ_LAUNCH(32);
#undef SEQ_LAUNCH
}

constexpr size_t kTraceBytes =
    sizeof(int32_t) * (SEQ_TRACE_HEADER_INTS + (size_t)SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS + 4);

}  // namespace
}  // namespace seqtree

using namespace seqtree;

// Test hook (not part of the public header): bound of the inter-workgroup wait, in polls.
extern "C" void seqtree_internal_set_spin_limit(uint32_t polls) { g_spin_limit = polls; }

extern "C" size_t seq_verify_workspace(int32_t n_tree, int32_t vocab, int32_t dtype) {
    (void)n_tree; (void)vocab; (void)dtype;
    return (kTraceBytes + 255) / 256 * 256;
}

extern "C" int seq_verify(const void* target_logits, const void* draft_logits,
                          const int32_t* tree_tokens, const int32_t* parent, float temperature,
                          const float* uniforms, int32_t* accepted_path, int32_t* bonus_token,
                          int32_t n_tree, int32_t vocab, int32_t dtype, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    if (!target_logits || !draft_logits || !tree_tokens || !parent || !uniforms || !accepted_path ||
        !bonus_token)
        return SEQ_ERR_NULL;
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_tree < 1 || n_tree > SEQ_MAX_TREE || vocab < 2 || vocab > SEQ_MAX_VOCAB) return SEQ_ERR_SHAPE;
    if (!(temperature >= 0.0f) || std::isinf(temperature)) return SEQ_ERR_TEMPERATURE;
    int rc = validate_parent(parent, n_tree);
    if (rc != SEQ_OK) return rc;
    if (!workspace || workspace_bytes < seq_verify_workspace(n_tree, vocab, dtype)) return SEQ_ERR_WORKSPACE;

    TreePlan plan;
    rc = get_tree_plan(parent, n_tree, &plan);
    if (rc != SEQ_OK) return rc;
    SyncArea* sync = nullptr;
    rc = get_sync_area(&sync);
    if (rc != SEQ_OK) return rc;

    int ept = 8;
    while ((long long)kVerifyMaxGroups * kThreads * ept < vocab) ept *= 2;  // <= 32 by SEQ_MAX_VOCAB
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
    p.slots = sync->verify_slots;
    p.epoch = sync->verify_epoch;
    p.spin_limit = g_spin_limit;
    p.n = n_tree;
    p.V = vocab;
    p.W = (vocab + kThreads * ept - 1) / (kThreads * ept);
    const bool greedy = temperature == 0.0f;
    p.inv_T = greedy ? 1.0f : 1.0f / temperature;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dtype == SEQ_BF16) launch_verify<uint16_t>(p, greedy, ept, stream);
    else launch_verify<float>(p, greedy, ept, stream);
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
