// seq_top_p_filter: nucleus (top-p) filtering of logit rows, the sampling hyper-parameter of the
// paper's robustness table (appendix "Robustness additional results").  Of softmax(logits / T)
// the most probable tokens are kept, as few as reach a total probability of top_p; every other
// logit becomes -inf, which the verification walk and the drafter's draw read as probability
// zero.  Equal probabilities at the cut: lower token id first.
//
// No sort.  The cut is the largest threshold t such that the tokens with e >= t (e = the
// unnormalised probability exp((x - max) / T), an fp32 number in (0, 1]) still hold top_p of the
// mass; positive floats order like their bit patterns, so t is found by bisection over 30 bits,
// one masked sum over the row per bisection step (fp32 within a thread, fp64 across).  As soon as
// at most 256 values are left between the bounds (about 10 steps in) they are put in order and
// added up directly.  If the bisection runs to its end instead (many equal values at the cut),
// tokens above the cut are kept and tokens exactly at it in ascending id as far as needed (one
// prefix count).
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

constexpr int kFewCandidates = 256;      // four per lane of one wavefront

struct Shared {
    unsigned long long cand[kFewCandidates], sorted[kFewCandidates], cut_word;
    int n_cand;
    double sum[kWaves], sum2[kWaves];
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

// the same for two values at once (one pair of barriers)
__device__ __forceinline__ void block_sum2(double a, double b, Shared& sh, double* ta, double* tb) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double ia = wave_scan(a), ib = wave_scan(b);
    __syncthreads();
    if (lane == 63) { sh.sum[wave] = ia; sh.sum2[wave] = ib; }
    __syncthreads();
    double x = 0.0, y = 0.0;
    for (int w = 0; w < kWaves; ++w) { x += sh.sum[w]; y += sh.sum2[w]; }
    *ta = x; *tb = y;
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
    bool by_word = false;      // the cut is one token: (probability, id) packed in cut_word
    unsigned long long cut_word = 0;
    if (p.greedy || !(m_all > -INFINITY)) {
        cut = 0xFFFFFFFFu;     // nothing is "above"; the arg-max alone is kept below
    } else if (p.top_p >= 1.0f) {
        cut = 0;               // everything of non-zero probability stays: no search, no rounding
    } else {
        float z_f = 0.f;
        visit([&](float v, int) { z_f += v; });
        const double goal = (double)p.top_p * block_sum((double)z_f, sh);
        uint32_t lo = 1, hi = 0x3F800001u;     // sum(e >= lo) >= goal > sum(e >= hi) = 0
        double above_hi = 0.0;                 // sum(e >= hi)
        double count_lo = (double)V, count_hi = 0.0;   // how many values are >= lo (an upper bound at first), >= hi
        while (hi - lo > 1 && count_lo - count_hi > (double)kFewCandidates) {
            const uint32_t mid = lo + (hi - lo) / 2;
            float s_f = 0.f;
            int c = 0;
            visit([&](float v, int) { const bool in = __float_as_uint(v) >= mid; s_f += in ? v : 0.f; c += in; });
            double s_mid, c_mid;
            block_sum2((double)s_f, (double)c, sh, &s_mid, &c_mid);
            if (s_mid >= goal) { lo = mid; count_lo = c_mid; }
            else { hi = mid; above_hi = s_mid; count_hi = c_mid; }
        }
        if (hi - lo > 1) {
            // Few values are left between the bounds: put them in order (probability descending,
            // id ascending -- one 64-bit word each, as the drafter's draw does) and add them up.
            if (tid == 0) sh.n_cand = 0;
            __syncthreads();
            visit([&](float v, int t) {
                const uint32_t b = __float_as_uint(v);
                if (b >= lo && b < hi && t < V) {
                    const int at = atomicAdd(&sh.n_cand, 1);
                    if (at < kFewCandidates) sh.cand[at] = ((unsigned long long)b << 32) | (0xFFFFFFFFu - (uint32_t)t);
                }
            });
            __syncthreads();
            const int n_cand = min(sh.n_cand, kFewCandidates);
            if (tid < n_cand) {
                const unsigned long long mine_word = sh.cand[tid];
                int place = 0;
                for (int j = 0; j < n_cand; ++j) place += sh.cand[j] > mine_word;
                sh.sorted[place] = mine_word;
            }
            __syncthreads();
            if (wave == 0) {
                // running sums of the ordered candidates, four per lane: where is top_p reached?
                double v[4], local = 0.0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = lane * 4 + q;
                    v[q] = j < n_cand ? (double)__uint_as_float((uint32_t)(sh.sorted[j] >> 32)) : 0.0;
                    local += v[q];
                }
                double run = above_hi + wave_scan(local) - local;
                int first = 0x7FFFFFFF;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    run += v[q];
                    if (first == 0x7FFFFFFF && lane * 4 + q < n_cand && run >= goal) first = lane * 4 + q;
                }
                const int take_at = wave_min(first);
                if (lane == 0) sh.cut_word = sh.sorted[take_at == 0x7FFFFFFF ? n_cand - 1 : take_at];
            }
            __syncthreads();
            cut_word = sh.cut_word;
            by_word = true;
        } else {
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
    }

    // Write pass.  In the tie case a token exactly at the cut needs its rank, in ascending id,
    // among its equals: ids ascend with (step, thread, element), so a prefix count per step over
    // the threads does it.
    unsigned long long mine = 0;   // tokens exactly at the cut in the steps before this one
    int kept_here = 0;
    const bool all_or_one = p.greedy || !(m_all > -INFINITY);
    auto write_step = [&](int s, const uint32_t (&bits)[kEpt]) {
        const int base = s * kStep + tid * kEpt;
        int rank = 0;
        if (!by_word && !all_or_one) {        // uniform over the workgroup
            int eq = 0;
#pragma unroll
            for (int i = 0; i < kEpt; ++i) eq += (base + i < V && bits[i] == cut);
            int incl = eq;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) { const int o = __shfl_up(incl, d); if (lane >= d) incl += o; }
            __syncthreads();
            if (lane == 63) sh.cnt[wave] = (unsigned long long)incl;
            __syncthreads();
            int before = incl - eq, step_total = 0;
            for (int w = 0; w < kWaves; ++w) { if (w < wave) before += (int)sh.cnt[w]; step_total += (int)sh.cnt[w]; }
            rank = (int)mine + before;
            mine += (unsigned long long)step_total;
        }
        bool keep[kEpt];
#pragma unroll
        for (int i = 0; i < kEpt; ++i) {
            const int t = base + i;
            if (all_or_one) keep[i] = t == arg || !p.greedy;
            else if (by_word) keep[i] = (((unsigned long long)bits[i] << 32) | (0xFFFFFFFFu - (uint32_t)t)) >= cut_word;
            else if (bits[i] > cut) keep[i] = true;
            else if (bits[i] == cut) { keep[i] = rank < need; ++rank; }
            else keep[i] = false;
            keep[i] = keep[i] && t < V;
            kept_here += keep[i];
        }
        // kept logits as they were, the rest -inf; 16 bytes at a time where the row allows it
        if (vec_ok && base + kEpt <= V) {
            constexpr int kVecs = (int)sizeof(LT) * kEpt / 16;
#pragma unroll
            for (int q = 0; q < kVecs; ++q) {
                uint4 raw = *reinterpret_cast<const uint4*>(row + base + q * (kEpt / kVecs));
                uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
                if constexpr (sizeof(LT) == 2) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t lo16 = keep[2 * k] ? (w[k] & 0xFFFFu) : 0xFF80u;
                        const uint32_t hi16 = keep[2 * k + 1] ? (w[k] & 0xFFFF0000u) : 0xFF800000u;
                        w[k] = lo16 | hi16;
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) w[k] = keep[q * 4 + k] ? w[k] : 0xFF800000u;
                }
                *reinterpret_cast<uint4*>(out + base + q * (kEpt / kVecs)) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kEpt; ++i) {
                const int t = base + i;
                if (t >= V) continue;
                if constexpr (sizeof(LT) == 2) out[t] = keep[i] ? row[t] : (LT)0xFF80u;
                else out[t] = keep[i] ? row[t] : (LT)(-INFINITY);
            }
        }
    };
    if constexpr (REG) {
#pragma unroll 1
        for (int s = 0; s < steps; ++s) {      // one copy of the step's code; the values come out of their registers by a switch
            uint32_t bits[kEpt];
#pragma unroll
            for (int i = 0; i < kEpt; ++i) {
                const float v = s == 0 ? e[i] : (s == 1 ? e[kEpt + i] : (s == 2 ? e[2 * kEpt + i] : e[3 * kEpt + i]));
                bits[i] = __float_as_uint(v);
            }
            write_step(s, bits);
        }
    } else {
        for (int s = 0; s < steps; ++s) {
            float x[kEpt];
            uint32_t bits[kEpt];
            load_clean<LT>(row, s * kStep + tid * kEpt, V, p.inv_T, vec_ok, x);
#pragma unroll
            for (int i = 0; i < kEpt; ++i) bits[i] = __float_as_uint(prob_of(x[i], m_all, 1.0f));
            write_step(s, bits);
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
