// seq_draft_sample: the drafter's ordered draw of child tokens, without replacement.
//
// Algorithm 2 (Sec. 3.2.1) verifies children that were drawn one after the other without
// replacement from softmax(draft_logits / T); the implementation details (Sec. 4.1) name the
// exponential-sort method for that draw.  Every token x gets an independent Exp(1) variate
// E[x]; the tokens ordered by Q[x] / E[x], largest first, are such a draw.  In logarithms
//
//     key[x] = logits[x] / T + g[x],    g = -ln E = -ln(-ln w),   w uniform in (0,1)
//
// and a row's children are the n_children[row] largest keys in descending order.
//
// One pass over the logits.  A workgroup of four wavefronts takes a run of tokens of one row,
// 8 consecutive tokens per lane and step (two Philox4x32-10 blocks, one 16-byte load of bf16).
// A key and its token id are packed in one 64-bit word that orders like (key descending, id
// ascending), so every comparison below is one unsigned compare.  Each wavefront keeps its 64
// best words sorted across its lanes (lane j holds the j-th best): the first step seeds the
// list with a bitonic sort of the lanes' own best words; after that a word enters only if it
// beats the k-th best, which the wavefront tests with one compare and a ballot per token -- in
// a long row that happens about k ln(N / 64) times in all.  The four lists are merged through
// LDS by rank (an entry's rank is its own index plus, by binary search, the number of better
// entries in the other lists).  A row split over several workgroups leaves its partial lists
// in the workspace and a second, small kernel merges them the same way.
//
// Arithmetic per token: Philox (~14 vector instructions per word), two hardware logarithms,
// three multiply-adds, one 64-bit compare.  At T > 0 that, not the 2 or 4 bytes of the logit,
// is what bounds the kernel; at T = 0 (keys = logits, no random numbers) it streams.
#include <cmath>

#include "seq_internal.h"

namespace seqtree {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kPerLane = 8;                     // tokens per lane and step
constexpr int kStepTokens = kThreads * kPerLane;  // 2048
constexpr int kMaxChunks = 16;                  // workgroups that share one row, at most
constexpr int kTargetGroups = 1024;             // aim for this many workgroups per launch

typedef unsigned long long u64;

struct DraftParams {
    const void* logits;
    const int32_t* n_children;
    const uint64_t* rng;        // seed, step
    int32_t* tokens;            // [rows][k_max]
    u64* partial;               // [rows][chunks][k_max]
    int32_t rows, V, k_max, chunks, chunk_tokens;
    float inv_T;
};

// ---------------------------------------------------------------------------------------
// random numbers: Philox4x32-10 (Salmon et al., SC'11), key = seed, counter = (x / 4, row, step)
// ---------------------------------------------------------------------------------------
struct Words4 { uint32_t w[4]; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const u64 a = (u64)0xD2511F53u * c0;
        const u64 b = (u64)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)b;
        c3 = (uint32_t)a;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words4{{c0, c1, c2, c3}};
}

// Standard Gumbel variate of a 32-bit word.  w = ((word >> 9) + 1/2) 2^-23 is exact in fp32;
// g = -ln(-ln w) = -ln 2 * log2(-log2 w) - ln(ln 2).
__device__ __forceinline__ float gumbel_of(uint32_t word) {
    const float w = fmaf((float)(word >> 9), 0x1p-23f, 0x1p-24f);
    const float l2 = __builtin_amdgcn_logf(w);
    return fmaf(-0.69314718056f, __builtin_amdgcn_logf(-l2), 0.36651292058f);
}

// (key, token) as one word: larger word = earlier in the order.  Floats map to unsigned
// integers of the same order; the id is complemented so that the lower id wins among equal keys.
__device__ __forceinline__ u64 pack(float key, uint32_t token) {
    const uint32_t b = __float_as_uint(key + 0.0f);   // -0 and +0 are one key
    const uint32_t ordered = b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
    return ((u64)ordered << 32) | (0xFFFFFFFFu - token);
}
__device__ __forceinline__ int32_t token_of(u64 word) { return (int32_t)(0xFFFFFFFFu - (uint32_t)word); }

// Tokens of zero probability (logit -inf or NaN, or a tempered logit below -2^103) come after
// all others, ordered by their Gumbel variate alone -- a uniformly random order, the uniform
// continuation Algorithm 2 prescribes once the support is used up.  (32 - g) 2^100 > 15 * 2^100
// keeps them below every other key and keeps their order exact.
__device__ __forceinline__ float sampling_key(float logit, float inv_T, float g) {
    const float key = fmaf(logit, inv_T, g);
    const float last = fmaf(g, 0x1p100f, -0x1p105f);
    return key > -0x1p103f ? key : last;
}
// T = 0: the limit of the above, the logits themselves.
__device__ __forceinline__ float greedy_key(float logit) { return logit > -INFINITY ? logit : -INFINITY; }

// ---------------------------------------------------------------------------------------
// a wavefront's sorted list
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ u64 read_lane(u64 v, int lane) {
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 sort_descending(u64 v, int lane) {
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            const u64 other = __shfl_xor(v, j);
            const bool keep_larger = ((lane & k) == 0) == ((lane & j) == 0);
            const u64 hi = v > other ? v : other, lo = v > other ? other : v;
            v = keep_larger ? hi : lo;
        }
    }
    return v;
}

__device__ __forceinline__ void insert(u64& list, u64 cand, int lane) {
    const int pos = __popcll(__ballot(list > cand));   // the list is sorted: the better ones are a prefix
    const u64 up = __shfl_up(list, 1);
    list = lane < pos ? list : (lane == pos ? cand : up);
}

// Number of entries of a descending list that are larger than v.
__device__ __forceinline__ int count_larger(const u64* list, int k, u64 v) {
    int lo = 0, hi = k;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (list[mid] > v) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------------------
// loads: 8 consecutive logits of a row
// ---------------------------------------------------------------------------------------
template <typename E> __device__ __forceinline__ float to_float(E v);
template <> __device__ __forceinline__ float to_float<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_float<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <typename E, bool VEC>
__device__ __forceinline__ void load8(const E* row, int t0, int end, float (&x)[kPerLane]) {
    if constexpr (VEC) {
        // the row length is a multiple of 8 and the base is 16-byte aligned: all 8 or none
        if (t0 < end) {
            if constexpr (sizeof(E) == 2) {
                const uint4 v = *reinterpret_cast<const uint4*>(row + t0);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[2 * i] = __uint_as_float(w[i] << 16);
                    x[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
                }
            } else {
                const float4 a = *reinterpret_cast<const float4*>(row + t0);
                const float4 b = *reinterpret_cast<const float4*>(row + t0 + 4);
                x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
                x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) x[i] = 0.f;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) x[i] = t0 + i < end ? to_float<E>(row[t0 + i]) : 0.f;
    }
}

// ---------------------------------------------------------------------------------------
// kernel 1: the best k words of a run of tokens
// ---------------------------------------------------------------------------------------
template <typename E, bool VEC, bool GREEDY>
__global__ void __launch_bounds__(kThreads) draft_sample_kernel(const DraftParams p) {
    __shared__ u64 lists[kWaves][64];
    const int row = blockIdx.y, chunk = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int k = p.n_children[row];
    k = k < 0 ? 0 : (k > p.k_max ? p.k_max : k);
    k = __builtin_amdgcn_readfirstlane(k);
    int32_t* out_tokens = p.tokens + (size_t)row * p.k_max;
    u64* out_partial = p.partial + ((size_t)row * p.chunks + chunk) * p.k_max;
    if (p.chunks == 1) {
        if (tid >= k && tid < p.k_max) out_tokens[tid] = -1;
    } else if (tid < k) {
        out_partial[tid] = 0;      // a run shorter than k leaves empty entries
    }
    if (k == 0) return;

    const int begin = chunk * p.chunk_tokens;
    const int end = min(p.V, begin + p.chunk_tokens);
    const E* logits = static_cast<const E*>(p.logits) + (size_t)row * p.V;
    uint32_t seed_lo = 0, seed_hi = 0, step_lo = 0, step_hi = 0;
    if constexpr (!GREEDY) {
        const uint64_t seed = p.rng[0], step = p.rng[1];
        seed_lo = (uint32_t)seed; seed_hi = (uint32_t)(seed >> 32);
        step_lo = (uint32_t)step; step_hi = (uint32_t)(step >> 32);
    }

    u64 list = 0;       // lane j: the j-th best word this wavefront has seen
    u64 bar = 0;        // the k-th best: what a word has to beat
    for (int base = begin; base < end; base += kStepTokens) {
        const int t0 = base + tid * kPerLane;
        float x[kPerLane];
        load8<E, VEC>(logits, t0, end, x);
        u64 word[kPerLane];
        if constexpr (GREEDY) {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) word[i] = pack(greedy_key(x[i]), (uint32_t)(t0 + i));
        } else {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const Words4 r = philox4x32_10((uint32_t)t0 / 4u + h, (uint32_t)row, step_lo, step_hi, seed_lo, seed_hi);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    word[4 * h + i] = pack(sampling_key(x[4 * h + i], p.inv_T, gumbel_of(r.w[i])), (uint32_t)(t0 + 4 * h + i));
            }
        }
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) word[i] = t0 + i < end ? word[i] : 0;

        u64 seeded = 0;   // the word this lane has already put into the list
        if (base == begin) {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) seeded = word[i] > seeded ? word[i] : seeded;
            list = sort_descending(seeded, lane);
            bar = read_lane(list, k - 1);
        }
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            u64 pending = __ballot(word[i] > bar && word[i] != seeded);
            while (pending) {
                const int src = __builtin_amdgcn_readfirstlane(__builtin_ctzll(pending));
                pending &= pending - 1;
                const u64 cand = read_lane(word[i], src);
                if (cand > bar) {            // the bar may have risen since the ballot
                    insert(list, cand, lane);
                    bar = read_lane(list, k - 1);
                }
            }
        }
    }

    // the four lists -> the run's best k, by rank
    lists[wave][lane] = list;
    __syncthreads();
    if (lane < k && list != 0) {
        int rank = lane;
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
            if (w != wave) rank += count_larger(lists[w], k, list);
        if (rank < k) {
            if (p.chunks == 1) out_tokens[rank] = token_of(list);
            else out_partial[rank] = list;
        }
    }
}

// ---------------------------------------------------------------------------------------
// kernel 2: the lists of a row's runs -> the row's tokens
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) draft_merge_kernel(const DraftParams p) {
    __shared__ u64 lists[kMaxChunks * SEQ_MAX_CHILDREN];
    const int row = blockIdx.x, tid = threadIdx.x;
    int k = p.n_children[row];
    k = k < 0 ? 0 : (k > p.k_max ? p.k_max : k);
    int32_t* out_tokens = p.tokens + (size_t)row * p.k_max;
    if (tid >= k && tid < p.k_max) out_tokens[tid] = -1;
    if (k == 0) return;
    const u64* partial = p.partial + (size_t)row * p.chunks * p.k_max;
    const int total = p.chunks * k;
    for (int idx = tid; idx < total; idx += kThreads) {
        const int c = idx / k, j = idx - c * k;
        lists[c * k + j] = partial[(size_t)c * p.k_max + j];
    }
    __syncthreads();
    for (int idx = tid; idx < total; idx += kThreads) {
        const int c = idx / k, j = idx - c * k;
        const u64 v = lists[idx];
        if (v == 0) continue;
        int rank = j;
        for (int other = 0; other < p.chunks && rank < k; ++other)
            if (other != c) rank += count_larger(lists + other * k, k, v);
        if (rank < k) out_tokens[rank] = token_of(v);
    }
}

int g_forced_chunks = 0;

void plan_chunks(int rows, int V, int* chunks, int* chunk_tokens) {
    const int steps = (V + kStepTokens - 1) / kStepTokens;
    int want = g_forced_chunks > 0 ? g_forced_chunks : (kTargetGroups + rows - 1) / rows;
    want = std::max(1, std::min(want, std::min(kMaxChunks, steps)));
    const int steps_per_chunk = (steps + want - 1) / want;
    *chunks = (steps + steps_per_chunk - 1) / steps_per_chunk;
    *chunk_tokens = steps_per_chunk * kStepTokens;
}

template <typename E, bool VEC>
void launch(const DraftParams& p, bool greedy, hipStream_t stream) {
    const dim3 grid(p.chunks, p.rows);
    if (greedy) draft_sample_kernel<E, VEC, true><<<grid, kThreads, 0, stream>>>(p);
    else draft_sample_kernel<E, VEC, false><<<grid, kThreads, 0, stream>>>(p);
    if (p.chunks > 1) draft_merge_kernel<<<p.rows, kThreads, 0, stream>>>(p);
}

}  // namespace
}  // namespace seqtree

using namespace seqtree;

// Test hook: force the number of workgroups that share a row (0 = let the library choose).
extern "C" void seqtree_internal_set_draft_chunks(int chunks) { g_forced_chunks = chunks; }

extern "C" size_t seq_draft_sample_workspace(int32_t n_rows, int32_t vocab, int32_t k_max, int32_t dtype) {
    (void)vocab; (void)dtype;
    const size_t rows = n_rows < 1 ? 1 : (size_t)n_rows, k = k_max < 1 ? 1 : (size_t)k_max;
    return std::max<size_t>(256, rows * kMaxChunks * k * sizeof(u64));
}

extern "C" int seq_draft_sample(const void* draft_logits, const int32_t* n_children, float temperature,
                                const uint64_t* rng, int32_t* tokens, int32_t n_rows, int32_t vocab,
                                int32_t k_max, int32_t dtype, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
    if (!draft_logits || !n_children || !rng || !tokens) return SEQ_ERR_NULL;
    if (dtype != SEQ_BF16 && dtype != SEQ_F32) return SEQ_ERR_DTYPE;
    if (n_rows < 1 || n_rows > SEQ_MAX_TREE || vocab < 2 || vocab > SEQ_MAX_VOCAB || k_max < 1 ||
        k_max > SEQ_MAX_CHILDREN || k_max > vocab)
        return SEQ_ERR_SHAPE;
    if (!(temperature >= 0.0f) || std::isinf(temperature)) return SEQ_ERR_TEMPERATURE;
    if (!workspace || workspace_bytes < seq_draft_sample_workspace(n_rows, vocab, k_max, dtype) ||
        (reinterpret_cast<uintptr_t>(workspace) & 15) != 0)
        return SEQ_ERR_WORKSPACE;

    DraftParams p;
    p.logits = draft_logits;
    p.n_children = n_children;
    p.rng = rng;
    p.tokens = tokens;
    p.partial = static_cast<u64*>(workspace);
    p.rows = n_rows;
    p.V = vocab;
    p.k_max = k_max;
    plan_chunks(n_rows, vocab, &p.chunks, &p.chunk_tokens);
    const bool greedy = temperature == 0.0f;
    p.inv_T = greedy ? 1.0f : 1.0f / temperature;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool vec = vocab % 8 == 0 && (reinterpret_cast<uintptr_t>(draft_logits) & 15) == 0;
    if (dtype == SEQ_BF16) {
        if (vec) launch<uint16_t, true>(p, greedy, stream); else launch<uint16_t, false>(p, greedy, stream);
    } else {
        if (vec) launch<float, true>(p, greedy, stream); else launch<float, false>(p, greedy, stream);
    }
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
