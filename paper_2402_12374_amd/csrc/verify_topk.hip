// Naive / top-k sampling verification (Sec. 2.2), the second baseline the paper holds Sequoia's
// algorithm against: at the node v the walk stands on, a token x is drawn from the TARGET
// distribution softmax(target_logits[v] / T); if x is the token of one of v's children the walk
// continues at that child, otherwise x is what the step emits.
//
// A node's draw depends on nothing but its own row and its own uniform, so every node draws at
// once -- one workgroup per node, three sweeps over its row: the maximum, the total mass, then
// the inverse CDF in ascending token id, with fp64 running sums like the bonus draw of the other
// kernels.  A single wavefront then follows the draws down the tree.  The later sweeps find the
// row in L2.  This reads all n rows where the
// walk visits only a few; it is a baseline for comparisons, latency-optimal rather than frugal.
#include "verify_device.h"

namespace seqtree {
namespace verify {
namespace {

constexpr int kEpt = 8;
constexpr int kStep = kThreads * kEpt;

struct Draw { int32_t token; float u, total, lo, hi; int32_t pad[3]; };   // 32 bytes per node

struct DrawShared {
    float part[kWaves];
    double scan[kWaves];
    int found_at, last_with_mass;
    double found_lo, found_hi;
    Draw result;
};

// The draw of node v by the whole workgroup; the result is left in sh.result (valid after the
// barrier this ends with).
template <typename LT>
__device__ __forceinline__ void draw_node(const VerifyParams& p, int v, DrawShared& sh) {
    float (&part)[kWaves] = sh.part;
    double (&scan)[kWaves] = sh.scan;
    int& found_at = sh.found_at;
    int& last_with_mass = sh.last_with_mass;
    double& found_lo = sh.found_lo;
    double& found_hi = sh.found_hi;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = p.V;
    const LT* row = static_cast<const LT*>(p.target) + (size_t)v * V;
    const bool vec_ok = (V % (16 / (int)sizeof(LT)) == 0) && (reinterpret_cast<uintptr_t>(p.target) & 15) == 0;
    const float u = p.uniforms[v];

    // sweep 1: the row's maximum
    float m = -INFINITY;
    for (int base = tid * kEpt; base < V; base += kStep) {
        float x[kEpt];
        load_row_slice<LT, kEpt>(row, base, V, p.inv_T, vec_ok, x);
#pragma unroll
        for (int e = 0; e < kEpt; ++e) m = fmaxf(m, x[e]);
    }
    m = wave_reduce<kOpMax>(m);
    if (lane == 0) part[wave] = m;
    if (tid == 0) { found_at = 0x7FFFFFFF; last_with_mass = -1; }
    __syncthreads();
    float m_all = -INFINITY;
    for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, part[w]);

    // sweep 2: the total mass, in fp64, of the very fp32 terms sweep 3 adds up
    double total = 0.0;
    {
        double mine = 0.0;
        for (int base = tid * kEpt; base < V; base += kStep) {
            float x[kEpt];
            load_row_slice<LT, kEpt>(row, base, V, p.inv_T, vec_ok, x);
#pragma unroll
            for (int e = 0; e < kEpt; ++e) mine += (double)prob_of(x[e], m_all, 1.0f);
        }
        const double incl = wave_scan(mine);
        if (lane == 63) scan[wave] = incl;
        __syncthreads();
        for (int w = 0; w < kWaves; ++w) total += scan[w];
        __syncthreads();
    }
    // sweep 3: the first token whose inclusive cumulative mass exceeds u * total (if rounding
    // leaves none: the last token with mass)
    const double goal = (double)u * total;
    double before_step = 0.0;
    for (int step_base = 0; step_base < V; step_base += kStep) {
        const int base = step_base + tid * kEpt;
        float x[kEpt], r[kEpt];
        load_row_slice<LT, kEpt>(row, base, V, p.inv_T, vec_ok, x);
        double mine = 0.0;
#pragma unroll
        for (int e = 0; e < kEpt; ++e) { r[e] = prob_of(x[e], m_all, 1.0f); mine += (double)r[e]; }
        const double incl = wave_scan(mine);
        if (lane == 63) scan[wave] = incl;
        __syncthreads();
        double run = before_step + incl - mine, step_total = 0.0;
        for (int w = 0; w < kWaves; ++w) { if (w < wave) run += scan[w]; step_total += scan[w]; }
        int found = 0x7FFFFFFF, last_pos = -1;
        double lo = 0.0, hi = 0.0;
#pragma unroll
        for (int e = 0; e < kEpt; ++e) {
            const double prev = run;
            run += (double)r[e];
            if (found == 0x7FFFFFFF && run > goal && base + e < V) { found = base + e; lo = prev; hi = run; }
            if (r[e] > 0.f && base + e < V) last_pos = base + e;
        }
        const int wave_found = wave_min(found), wave_last = wave_max(last_pos);
        if (lane == 0) {
            if (wave_found != 0x7FFFFFFF) atomicMin(&found_at, wave_found);
            if (wave_last >= 0) atomicMax(&last_with_mass, wave_last);
        }
        __syncthreads();
        if (found != 0x7FFFFFFF && found == found_at) { found_lo = lo; found_hi = hi; }
        before_step += step_total;
        __syncthreads();
        if (found_at != 0x7FFFFFFF) break;
    }
    if (tid == 0) {
        Draw d;
        d.u = u;
        d.total = (float)total;
        if (found_at != 0x7FFFFFFF) {
            d.token = found_at;
            d.lo = (float)(found_lo / total);
            d.hi = (float)(found_hi / total);
        } else {
            d.token = last_with_mass >= 0 ? last_with_mass : V - 1;
            d.lo = d.hi = 1.f;
        }
        d.pad[0] = d.pad[1] = d.pad[2] = 0;
        sh.result = d;
    }
    __syncthreads();
}

// The draws of a sequence live where the per-node kernel keeps its records: after the trace.
__device__ __forceinline__ Draw* draws_of(const VerifyParams& p) { return reinterpret_cast<Draw*>(p.records); }

// grid.x = node, grid.y = sequence of the batch (nothing is shared between sequences but the tree)
template <typename LT>
__global__ void __launch_bounds__(kThreads) topk_draw_kernel(const VerifyParams p_in) {
    const VerifyParams p = params_of_sequence(p_in, blockIdx.y, false);
    __shared__ DrawShared sh;
    draw_node<LT>(p, blockIdx.x, sh);
    if (threadIdx.x == 0) draws_of(p)[blockIdx.x] = sh.result;
}

// Follows the draws from the root: a lane per child looks for the drawn token.  With draws made
// beforehand one wavefront reads them; without, one workgroup makes each draw when the walk gets
// there (a big tree over a big vocabulary: the walk visits a handful of the nodes).  grid.y =
// sequence of the batch.
template <typename LT>
__global__ void __launch_bounds__(kThreads) topk_walk_kernel(const VerifyParams p_in, int have_draws) {
    const VerifyParams p = params_of_sequence(p_in, blockIdx.y, false);
    const Draw* draws = have_draws ? draws_of(p) : nullptr;
    __shared__ DrawShared sh;
    const int lane = threadIdx.x & 63;
    int v = 0, path_len = 0, n_rec = 0;
    Draw d;
    for (;;) {
        if (draws) d = draws[v];
        else { draw_node<LT>(p, v, sh); d = sh.result; __syncthreads(); }
        const int c_begin = p.child_start[v], c_end = p.child_start[v + 1];
        int next = -1;
        for (int k0 = c_begin; k0 < c_end && next < 0; k0 += 64) {
            const int k = k0 + lane;
            const int c = k < c_end ? p.child_list[k] : -1;
            const bool match = c >= 0 && p.tokens[c] == d.token;
            const unsigned long long hits = __ballot(match);
            if (hits) next = __builtin_amdgcn_readlane(c, __builtin_ctzll(hits));   // the first such child
        }
        if (threadIdx.x == 0) {
            int32_t* rec = p.trace + SEQ_TRACE_HEADER_INTS + n_rec * SEQ_TRACE_RECORD_WORDS;
            rec[0] = v; rec[1] = next; rec[2] = d.token; rec[3] = __float_as_int(d.u);
        }
        ++n_rec;
        if (next < 0) break;
        if (threadIdx.x == 0) p.path[path_len] = next;
        ++path_len;
        v = next;
    }
    for (int i = path_len + (int)threadIdx.x; i < p.n; i += (int)blockDim.x) p.path[i] = -1;
    if (threadIdx.x == 0) {
        p.bonus[0] = d.token;
        p.trace[0] = n_rec; p.trace[1] = 0; p.trace[2] = v;
        p.trace[3] = p.trace[4] = p.trace[5] = p.trace[6] = p.trace[7] = 0;
        float* binfo = reinterpret_cast<float*>(p.trace + SEQ_TRACE_HEADER_INTS + SEQ_MAX_TREE * SEQ_TRACE_RECORD_WORDS);
        binfo[0] = d.u; binfo[1] = d.total; binfo[2] = d.lo; binfo[3] = d.hi;
    }
}

int g_topk_mode = 0;   // test hook: 1 = always all draws at once, 2 = always where the walk goes

}  // namespace

void set_topk_mode(int mode) { g_topk_mode = mode; }

void launch_verify_topk(const VerifyParams& p, int dtype, hipStream_t stream, int batch) {
    static_assert(sizeof(Draw) * SEQ_MAX_TREE <=
                  sizeof(unsigned long long) * (size_t)SEQ_MAX_TREE * (kChildRecordWords + kNodeRecordWords), "workspace");
    // all draws at once while that is cheap (three sweeps over every row); beyond 2^24 logits one
    // workgroup draws only where the walk goes (measured at 768 x 128256: 73 us against 205 us)
    const bool lazy = (long long)p.n * p.V > (1ll << 24) || g_topk_mode == 2;
    const dim3 per_sequence(1, (unsigned)batch);
    if (lazy && g_topk_mode != 1) {
        if (dtype == SEQ_BF16) topk_walk_kernel<uint16_t><<<per_sequence, kThreads, 0, stream>>>(p, 0);
        else topk_walk_kernel<float><<<per_sequence, kThreads, 0, stream>>>(p, 0);
        return;
    }
    const dim3 per_node((unsigned)p.n, (unsigned)batch);
    if (dtype == SEQ_BF16) topk_draw_kernel<uint16_t><<<per_node, kThreads, 0, stream>>>(p);
    else topk_draw_kernel<float><<<per_node, kThreads, 0, stream>>>(p);
    topk_walk_kernel<uint16_t><<<per_sequence, 64, 0, stream>>>(p, 1);
}

}  // namespace verify
}  // namespace seqtree
