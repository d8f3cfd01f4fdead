// seq_top_p_filter: nucleus (top-p) filtering of logit rows, the sampling hyper-parameter of the
// paper's robustness table (appendix "Robustness additional results").  Of softmax(logits / T)
// the most probable tokens are kept, as few as reach a total probability of top_p; every other
// logit becomes -inf, which the verification walk and the drafter's draw read as probability
// zero.  Equal probabilities at the cut: lower token id first.
//
// No sort.  The cut is the largest threshold t such that the tokens with e >= t (e = the
// unnormalised probability exp((x - max) / T), an fp32 number in (0, 1]) still hold top_p of the
// mass; positive floats order like their bit patterns, so t is found by bisection over 30 bits,
// one masked sum over the row per bisection step (fp32 within a thread, fp64 across).  Tokens above
// the cut are kept, tokens exactly at it in ascending id as far as needed (one prefix count).
// One workgroup per row.  Rows of up to 32768 tokens stay in registers (32 values per lane);
// longer rows are re-read and re-exponentiated at every step (they sit in L2) -- slow, correct.
#include <type_traits>

#include "verify_device.h"

namespace seqtree {
namespace verify {
namespace {

constexpr int kEpt = 8;
constexpr int kStep = kThreads * kEpt;       // 8192 tokens per sweep step
constexpr int kRegSteps = 4;                 // rows up to 4 steps are held in registers

struct TopPParams {
    const void* logits;
    void* filtered;
    int32_t* kept;
    float top_p, inv_T;
    int rows, V, greedy;
};

struct Shared {
    double sum[kWaves];
    float fmax_[kWaves];
    unsigned long long cnt[kWaves];
    int best[kWaves];
};

// 8 consecutive tempered logits; NaN reads as -inf (probability zero), like everywhere else
template <typename LT>
__device__ __forceinline__ void load_clean(const LT* row, int base, int V, float inv_T, bool vec_ok, float* x) {
    load_row_slice<LT, kEpt>(row, base, V, inv_T, vec_ok, x);
#pragma unroll
    for (int i = 0; i < kEpt; ++i) x[i] = x[i] == x[i] ? x[i] : -INFINITY;
}

// sum over the workgroup of a per-thread double; every thread gets the result
__device__ __forceinline__ double block_sum(double v, Shared& sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double incl = wave_scan(v);
    __syncthreads();
    if (lane == 63) sh.sum[wave] = incl;
    __syncthreads();
    double total = 0.0;
    for (int w = 0; w < kWaves; ++w) total += sh.sum[w];
    return total;
}

template <typename LT, bool REG>
__global__ void __launch_bounds__(kThreads) top_p_kernel(const TopPParams p) {
    __shared__ Shared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = p.V, row_id = blockIdx.x;
    const LT* row = static_cast<const LT*>(p.logits) + (size_t)row_id * V;
    LT* out = static_cast<LT*>(p.filtered) + (size_t)row_id * V;
    const bool vec_ok = (V % (16 / (int)sizeof(LT)) == 0) && (reinterpret_cast<uintptr_t>(p.logits) & 15) == 0;
    const int steps = (V + kStep - 1) / kStep;
    // the row's maximum (T = 0: and where it is, lowest id)
    float e[REG ? kRegSteps * kEpt : 1];
    float m = -INFINITY;
    int where = 0x7FFFFFFF;
    auto take_step = [&](int s, auto reg_slot) {
        float x[kEpt];
        const int base = s * kStep + tid * kEpt;
        load_clean<LT>(row, base, V, p.inv_T, vec_ok, x);
#pragma unroll
        for (int i = 0; i < kEpt; ++i) {
            if (x[i] > m) { m = x[i]; where = base + i; }
            if constexpr (REG) e[decltype(reg_slot)::value * kEpt + i] = x[i];
        }
    };
    if constexpr (REG) {
        // compile-time slots: the values stay in registers (tokens past the row read as -inf)
        take_step(0, std::integral_constant<int, 0>{});
        take_step(1, std::integral_constant<int, 1>{});
        take_step(2, std::integral_constant<int, 2>{});
        take_step(3, std::integral_constant<int, 3>{});
        static_assert(kRegSteps == 4, "one call per register step");
    } else {
        for (int s = 0; s < steps; ++s) take_step(s, std::integral_constant<int, 0>{});
    }
    const float m_wave = wave_reduce<kOpMax>(m);
    const int where_wave = wave_min(m == m_wave && m > -INFINITY ? where : 0x7FFFFFFF);
    if (lane == 0) { sh.fmax_[wave] = m_wave; sh.best[wave] = where_wave; }
    __syncthreads();
    float m_all = -INFINITY;
    for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, sh.fmax_[w]);
    int arg = 0x7FFFFFFF;
    for (int w = 0; w < kWaves; ++w) if (sh.fmax_[w] == m_all) arg = min(arg, sh.best[w]);

    // e = exp((x - max) / T); visit(f) calls f(value, token id) for every token of this thread
    if constexpr (REG) {
#pragma unroll
        for (int i = 0; i < kRegSteps * kEpt; ++i) e[i] = prob_of(e[i], m_all, 1.0f);
    }
    auto visit = [&](auto&& f) {
        if constexpr (REG) {
#pragma unroll
            for (int s = 0; s < kRegSteps; ++s)
#pragma unroll
                for (int i = 0; i < kEpt; ++i) f(e[s * kEpt + i], s * kStep + tid * kEpt + i);
        } else {
            for (int s = 0; s < steps; ++s) {
                float x[kEpt];
                const int base = s * kStep + tid * kEpt;
                load_clean<LT>(row, base, V, p.inv_T, vec_ok, x);
#pragma unroll
                for (int i = 0; i < kEpt; ++i) f(prob_of(x[i], m_all, 1.0f), base + i);
            }
        }
    };

    uint32_t cut = 0;          // bit pattern of the cut value
    int need = 0;              // how many of the tokens exactly at the cut are kept
    if (p.greedy || !(m_all > -INFINITY)) {
        cut = 0xFFFFFFFFu;     // nothing is "above"; the arg-max alone is kept below
    } else {
        float z_f = 0.f;
        visit([&](float v, int) { z_f += v; });
        const double goal = (double)p.top_p * block_sum((double)z_f, sh);
        uint32_t lo = 1, hi = 0x3F800001u;     // sum(e >= lo) >= goal > sum(e >= hi) = 0
        while (hi - lo > 1) {
            const uint32_t mid = lo + (hi - lo) / 2;
            float s_f = 0.f;
            visit([&](float v, int) { s_f += __float_as_uint(v) >= mid ? v : 0.f; });
            if (block_sum((double)s_f, sh) >= goal) lo = mid; else hi = mid;
        }
        cut = lo;
        float above_f = 0.f;
        int equal = 0;
        visit([&](float v, int) { const uint32_t b = __float_as_uint(v); above_f += b > cut ? v : 0.f; equal += b == cut; });
        const double above = block_sum((double)above_f, sh);
        const double cut_value = (double)__uint_as_float(cut);
        const double count = ceil((goal - above) / cut_value);
        const double equal_all = block_sum((double)equal, sh);
        need = (int)fmin(fmax(count, 1.0), equal_all);
    }

    // rank, in ascending id, of this thread's tokens among those exactly at the cut: ids ascend
    // with (step, thread, element), so a prefix count per step over the threads does it
    unsigned long long mine = 0;   // tokens exactly at the cut in the steps before this one
    int kept_here = 0;
    for (int s = 0; s < steps; ++s) {
        float x[kEpt];
        const int base = s * kStep + tid * kEpt;
        load_clean<LT>(row, base, V, p.inv_T, vec_ok, x);
        int eq = 0;
        uint32_t bits[kEpt];
#pragma unroll
        for (int i = 0; i < kEpt; ++i) {
            bits[i] = __float_as_uint(prob_of(x[i], m_all, 1.0f));
            eq += (base + i < V && bits[i] == cut);
        }
        // exclusive prefix of eq over the workgroup, in thread order
        int incl = eq;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int o = __shfl_up(incl, d); if (lane >= d) incl += o; }
        __syncthreads();
        if (lane == 63) sh.cnt[wave] = (unsigned long long)incl;
        __syncthreads();
        int before = incl - eq, step_total = 0;
        for (int w = 0; w < kWaves; ++w) { if (w < wave) before += (int)sh.cnt[w]; step_total += (int)sh.cnt[w]; }
        int rank = (int)mine + before;
        mine += (unsigned long long)step_total;     // tokens at the cut in the steps so far
        // write the step: kept logits as they were, the rest -inf
#pragma unroll
        for (int i = 0; i < kEpt; ++i) {
            const int t = base + i;
            if (t >= V) continue;
            bool keep;
            if (p.greedy || !(m_all > -INFINITY)) keep = t == arg || (!(m_all > -INFINITY) && !p.greedy);
            else if (bits[i] > cut) keep = true;
            else if (bits[i] == cut) { keep = rank < need; ++rank; }
            else keep = false;
            kept_here += keep;
            if constexpr (sizeof(LT) == 2) out[t] = keep ? row[t] : (LT)0xFF80u;
            else out[t] = keep ? row[t] : (LT)(-INFINITY);
        }
    }
    const double kept_all = block_sum((double)kept_here, sh);
    if (tid == 0 && p.kept) p.kept[row_id] = (int)kept_all;
}

}  // namespace
}  // namespace verify
}  // namespace seqtree

using namespace seqtree;
using namespace seqtree::verify;

extern "C" int seq_top_p_filter(const void* logits, void* filtered, float top_p, float temperature,
                                int32_t n_rows, int32_t vocab, int32_t dtype, int32_t* kept, void* hip_stream) {
    if (!logits || !filtered) return SEQ_ERR_NULL;
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_rows < 1 || n_rows > SEQ_MAX_TREE || vocab < 2 || vocab > SEQ_MAX_VOCAB || !(top_p > 0.0f) || !(top_p <= 1.0f))
        return SEQ_ERR_SHAPE;
    if (!(temperature >= 0.0f) || std::isinf(temperature)) return SEQ_ERR_TEMPERATURE;
    TopPParams p;
    p.logits = logits;
    p.filtered = filtered;
    p.kept = kept;
    p.top_p = top_p;
    p.greedy = temperature == 0.0f;
    p.inv_T = p.greedy ? 1.0f : 1.0f / temperature;
    p.rows = n_rows;
    p.V = vocab;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool reg = vocab <= kRegSteps * kStep;
    if (dtype == SEQ_BF16) {
        if (reg) top_p_kernel<uint16_t, true><<<n_rows, kThreads, 0, stream>>>(p);
        else top_p_kernel<uint16_t, false><<<n_rows, kThreads, 0, stream>>>(p);
    } else {
        if (reg) top_p_kernel<float, true><<<n_rows, kThreads, 0, stream>>>(p);
        else top_p_kernel<float, false><<<n_rows, kThreads, 0, stream>>>(p);
    }
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
