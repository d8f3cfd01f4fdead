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
// list with the lanes' own best words; after that a word enters only if it beats the k-th best,
// which the wavefront tests with one compare and a ballot per token -- in a long row that
// happens about k ln(N / 64) times in all (one at a time if few lanes have such a word,
// otherwise by sorting the 64 candidates and merging the two sorted lists).
// Sorting and merging go by rank through LDS: a word's place is the number of words larger
// than it -- counted over a wavefront's row by broadcast reads, or in sorted lists by binary
// searches that advance in step over all lists, so that the chain of dependent reads is log2 k
// long however many lists there are.  That is how the four lists of a workgroup become one,
// and how a row split over several workgroups is finished by whichever of them arrives last
// (one counter per row): the others leave their lists in a per-device exchange area as 64-bit
// words written and read with device-scope atomics; a word is never zero, the reader waits
// (bounded) for a slot to become non-zero and zeroes it again, so no fence, no second kernel
// and no clearing between calls is needed.
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
constexpr int kTargetGroups = 4096;             // aim for this many workgroups per launch (16 per CU)

typedef unsigned long long u64;

#ifdef SEQTREE_STAMPS
// per workgroup: start, first keys, loop done, lists merged, counted, others' lists read, end (100 MHz clock)
__device__ long long g_draft_wg_times[8 * 4096];
#define DRAFT_WG_TIME(slot) do { if (threadIdx.x == 0 && item < 4096) g_draft_wg_times[8 * item + (slot)] = wall_clock64(); } while (0)
#else
#define DRAFT_WG_TIME(slot) do {} while (0)
#endif

struct DraftParams {
    const void* logits;
    const int32_t* n_children;
    const uint64_t* rng;        // seed, step
    int32_t* tokens;            // [rows][k_max]
    u64* exchange;              // [rows][chunks][64], all zero between calls
    uint32_t* arrivals;         // [rows], all zero between calls
    int32_t rows, V, k_max, chunks, chunk_tokens;
    float inv_T;
    uint32_t spin_limit;
};

// ---------------------------------------------------------------------------------------
// random numbers: Philox4x32-10 (Salmon et al., SC'11), key = seed, counter = (x / 4, row, step)
// ---------------------------------------------------------------------------------------
// Two consecutive counter blocks at once (8 words = the 8 tokens of a lane).  The ten rounds are
// a rolled loop: the instruction cache is cold at every launch, and for a small call fetching
// unrolled rounds would take longer than running them.
struct Words8 { uint32_t w[8]; };

__device__ __forceinline__ void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
    const u64 a = (u64)0xD2511F53u * c[0];
    const u64 b = (u64)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(b >> 32) ^ c[1] ^ k0;
    const uint32_t n2 = (uint32_t)(a >> 32) ^ c[3] ^ k1;
    c[1] = (uint32_t)b;
    c[3] = (uint32_t)a;
    c[0] = n0;
    c[2] = n2;
}

__device__ __forceinline__ Words8 philox4x32_10_pair(uint32_t block, uint32_t c1, uint32_t c2, uint32_t c3,
                                                     uint32_t k0, uint32_t k1) {
    uint32_t a[4] = {block, c1, c2, c3}, b[4] = {block + 1u, c1, c2, c3};
#pragma unroll 1
    for (int round = 0; round < 10; ++round) {
        philox_round(a, k0, k1);
        philox_round(b, k0, k1);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words8{{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]}};
}

// Standard Gumbel variate of a 32-bit word.  w = ((word >> 9) + 1/2) 2^-23 is exact in fp32;
// g = -ln(-ln w) = -ln 2 * log2(-log2 w) - ln(ln 2).
__device__ __forceinline__ float gumbel_of(uint32_t word) {
    // the 23 bits as the fraction of a float in [1,2), minus (1 - 2^-24): the same value, exactly
    const float w = __uint_as_float((word >> 9) | 0x3F800000u) - 0x1.fffffep-1f;
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
// The key a word was made from; -inf for the values that stand for "no token".
__device__ __forceinline__ float key_of(u64 word) {
    const uint32_t ordered = (uint32_t)(word >> 32);
    const uint32_t b = (ordered & 0x80000000u) ? ordered ^ 0x80000000u : ~ordered;
    return ordered == 0 ? -INFINITY : __uint_as_float(b);
}

// Tokens of zero probability (logit -inf or NaN, or a tempered logit below -2^103) come after
// all others, ordered by their Gumbel variate alone -- a uniformly random order, the uniform
// continuation Algorithm 2 prescribes once the support is used up.  (32 - g) 2^100 > 15 * 2^100
// keeps them below every other key and keeps their order exact.
__device__ __forceinline__ float sampling_key(float tempered_plus_g, float g) {
    const float last = fmaf(g, 0x1p100f, -0x1p105f);
    return tempered_plus_g > -0x1p103f ? tempered_plus_g : last;
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

// Every word made from a token is at least this; smaller values stand for "no token".
constexpr u64 kSmallestWord = 1ull << 32;
__device__ __forceinline__ u64 no_token(int lane) { return (u64)lane + 2; }   // distinct, so ranks are too

// Sorts one word per lane, descending, through a row of LDS that belongs to this wavefront:
// a word's place is the number of larger words.  Words must be distinct.
__device__ __forceinline__ u64 sort_descending(u64 v, u64* row, int lane) {
    row[lane] = v;
    int place = 0;
#pragma unroll 8
    for (int l = 0; l < 64; l += 2) {
        const ulonglong2 o = *reinterpret_cast<const ulonglong2*>(row + l);   // same address in every lane
        place += (o.x > v) + (o.y > v);
    }
    row[place] = v;     // LDS serves a wavefront's requests in order: every read above is done
    return row[lane];
}

// The 64 best of two descending lists, descending: the larger of a[j] and b[63 - j] holds them
// as a bitonic sequence, which six compare-exchange stages sort.  (A rolled loop: this is the
// rare path, and the instruction cache is cold at every launch.)
__device__ __forceinline__ u64 merge_descending(u64 a, u64 b, int lane) {
    const u64 rb = __shfl(b, 63 - lane);
    u64 v = a > rb ? a : rb;
#pragma unroll 1
    for (int j = 32; j > 0; j >>= 1) {
        const u64 other = __shfl_xor(v, j);
        const u64 hi = v > other ? v : other, lo = v > other ? other : v;
        v = (lane & j) == 0 ? hi : lo;
    }
    return v;
}

__device__ __forceinline__ void insert(u64& list, u64 cand, int lane) {
    const int pos = __popcll(__ballot(list > cand));   // the list is sorted: the better ones are a prefix
    const u64 up = __shfl_up(list, 1);
    list = lane < pos ? list : (lane == pos ? cand : up);
}

// Takes one word per lane into the list: those that beat the bar, one at a time if they are
// few, else all at once.
constexpr int kOneByOne = 6;
__device__ __forceinline__ void absorb(u64& list, u64& bar, u64 word, bool wanted, int k, u64* row, int lane) {
    u64 pending = __ballot(wanted);
    if (pending == 0) return;
    if (__popcll(pending) > kOneByOne) {
        list = merge_descending(list, sort_descending(wanted ? word : no_token(lane), row, lane), lane);
        bar = read_lane(list, k - 1);
        return;
    }
    while (pending) {
        const int src = __builtin_amdgcn_readfirstlane(__builtin_ctzll(pending));
        pending &= pending - 1;
        const u64 cand = read_lane(word, src);
        if (cand > bar) {            // the bar may have risen since the ballot
            insert(list, cand, lane);
            bar = read_lane(list, k - 1);
        }
    }
}

// idx / d for 0 <= idx < 2^14 and 1 <= d <= 64, through one multiply: (idx + 1/2) / d is at
// least 1/(2d) away from every integer, far more than the rounding of the product.
__device__ __forceinline__ int small_div(int idx, float inv_d) { return (int)(((float)idx + 0.5f) * inv_d); }

// Number of the first k entries of a descending list that are larger than v.
__device__ __forceinline__ int count_larger(const u64* list, int k, u64 v) {
    int pos = 0;
#pragma unroll 1
    for (int step = 1 << (31 - __builtin_clz(k)); step > 0; step >>= 1) {
        const int probe = pos + step;
        if (probe <= k && list[probe - 1] > v) pos = probe;
    }
    return pos;
}

// ---------------------------------------------------------------------------------------
// loads: 8 consecutive logits of a row
// ---------------------------------------------------------------------------------------
// Raw bits of 8 consecutive logits (loaded one step ahead of their use).
template <typename E> struct Raw { uint32_t w[sizeof(E) * 2]; };

template <typename E, bool VEC>
__device__ __forceinline__ Raw<E> load8(const E* row, int t0, int end) {
    Raw<E> r;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(E) * 2); ++i) r.w[i] = 0;
    if constexpr (VEC) {
        // the row length is a multiple of 8 and the base is 16-byte aligned: all 8 or none
        if (t0 < end) {
            const uint4 a = *reinterpret_cast<const uint4*>(row + t0);
            r.w[0] = a.x; r.w[1] = a.y; r.w[2] = a.z; r.w[3] = a.w;
            if constexpr (sizeof(E) == 4) {
                const uint4 b = *reinterpret_cast<const uint4*>(row + t0 + 4);
                r.w[4] = b.x; r.w[5] = b.y; r.w[6] = b.z; r.w[7] = b.w;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            if (t0 + i < end) {
                if constexpr (sizeof(E) == 2) r.w[i / 2] |= (uint32_t)row[t0 + i] << (16 * (i & 1));
                else r.w[i] = __float_as_uint(row[t0 + i]);
            }
        }
    }
    return r;
}

template <typename E>
__device__ __forceinline__ void unpack(const Raw<E>& r, float (&x)[kPerLane]) {
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
        if constexpr (sizeof(E) == 2) x[i] = __uint_as_float((i & 1) ? (r.w[i / 2] & 0xFFFF0000u) : (r.w[i / 2] << 16));
        else x[i] = __uint_as_float(r.w[i]);
    }
}

// ---------------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------------
template <typename E, bool VEC, bool GREEDY>
__global__ void __launch_bounds__(kThreads) draft_sample_kernel(const DraftParams p) {
    __shared__ u64 lists[kMaxChunks][64];      // rows 0..3: one per wavefront until the end
    __shared__ int places[kMaxChunks][64];
    __shared__ int s_last, s_bad;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // A workgroup takes every gridDim.x-th run.  (By default the grid has one workgroup per run:
    // with rows of very different cost -- nodes without children cost nothing -- the hardware's
    // own dispatch balances better than this fixed stride; measured at 768 rows of which 256
    // draw: 66 us against 88 us with 2048 workgroups.)
    const int n_items = p.rows * p.chunks;
#pragma unroll 1
    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    const int row = item / p.chunks, chunk = item - row * p.chunks;
    if (item != (int)blockIdx.x) __syncthreads();      // the previous run is done with LDS
    DRAFT_WG_TIME(0);
    // every load the first step waits for goes out before anything is waited for
    const int begin = chunk * p.chunk_tokens;
    const int end = min(p.V, begin + p.chunk_tokens);
    const E* logits = static_cast<const E*>(p.logits) + (size_t)row * p.V;
    Raw<E> raw = load8<E, VEC>(logits, begin + tid * kPerLane, end);
    uint32_t seed_lo = 0, seed_hi = 0, step_lo = 0, step_hi = 0;
    if constexpr (!GREEDY) {
        const uint64_t seed = p.rng[0], step = p.rng[1];
        seed_lo = (uint32_t)seed; seed_hi = (uint32_t)(seed >> 32);
        step_lo = (uint32_t)step; step_hi = (uint32_t)(step >> 32);
    }
    int k = p.n_children[row];
    k = k < 0 ? 0 : (k > p.k_max ? p.k_max : k);
    k = __builtin_amdgcn_readfirstlane(k);
    int32_t* out_tokens = p.tokens + (size_t)row * p.k_max;
    if (chunk == 0 && tid >= k && tid < p.k_max) out_tokens[tid] = -1;
    if (k == 0) continue;   // all workgroups of the row skip it: nothing is counted or exchanged
    if (tid == 0) s_bad = 0;

    u64 list = no_token(63 - lane);  // lane j: the j-th best word this wavefront has seen
    u64 bar = 0;                     // the k-th best: what a word has to beat
    float pass_key = -INFINITY;         // a token whose key is below this needs no closer look
    Raw<E> ahead = load8<E, VEC>(logits, begin + kStepTokens + tid * kPerLane, end);
    for (int base = begin; base < end; base += kStepTokens) {
        const int t0 = base + tid * kPerLane;
        const Raw<E> further = load8<E, VEC>(logits, t0 + 2 * kStepTokens, end);   // two steps ahead
        float key[kPerLane];     // T > 0: logit / T + g;  T = 0: the logit
        float g[kPerLane];
        unpack<E>(raw, key);
        raw = ahead;
        ahead = further;
        if constexpr (!GREEDY) {
            const Words8 r = philox4x32_10_pair((uint32_t)t0 / 4u, (uint32_t)row, step_lo, step_hi, seed_lo, seed_hi);
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) {
                g[i] = gumbel_of(r.w[i]);
                key[i] = fmaf(key[i], p.inv_T, g[i]);
            }
        }
        // The filter every token passes through: one float compare.  It lets through whatever
        // could beat the bar -- and, harmlessly, equal keys and the padding past the row's end.
        // Zero-probability tokens (NaN or hugely negative here) matter only while the bar itself
        // is one of them or missing; then `pass_key` is -inf and everything passes.
        bool any = false;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) any |= !(key[i] < pass_key);
        if (base == begin) DRAFT_WG_TIME(1);
        if (__ballot(any) == 0) continue;      // the usual case once the bar has settled

        u64 word[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const float exact = GREEDY ? greedy_key(key[i]) : sampling_key(key[i], g[i]);
            word[i] = t0 + i < end ? pack(exact, (uint32_t)(t0 + i)) : 0;
        }
        u64 seeded = 0;   // the word this lane has already put into the list
        if (base == begin) {
#pragma unroll
            for (int i = 0; i < kPerLane; ++i) seeded = word[i] > seeded ? word[i] : seeded;
            seeded = seeded ? seeded : no_token(lane);
            list = sort_descending(seeded, lists[wave], lane);
            bar = read_lane(list, k - 1);
        }
        bool more = false;     // usually the lanes' own best words were all there was to take
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) more |= word[i] > bar && word[i] != seeded;
        if (__ballot(more) != 0) {
#pragma unroll 1
            for (int i = 0; i < kPerLane; ++i) {
                const u64 w = word[0];
#pragma unroll
                for (int j = 0; j + 1 < kPerLane; ++j) word[j] = word[j + 1];
                absorb(list, bar, w, w > bar && w != seeded, k, lists[wave], lane);
            }
        }
        const float bar_key = key_of(bar);
        pass_key = bar_key > -0x1p103f ? bar_key : -INFINITY;
    }

    // Stage 0: the four lists of this workgroup -> the run's best k.  Stage 1 (only in the
    // workgroup that finishes the row): the lists of all runs -> the row's tokens.  Either way
    // every entry's place is the number of larger entries in all lists, found pair by pair
    // (entry, list) over all threads and added up in LDS.
    DRAFT_WG_TIME(2);
    lists[wave][lane] = list;
    places[wave][lane] = 0;
    u64* exchange = p.exchange + (size_t)row * p.chunks * 64;
    const float inv_k = 1.0f / (float)k;
    int n_lists = kWaves;
#pragma unroll 1
    for (int stage = 0;; ++stage) {
        __syncthreads();
        const int entries = n_lists * k;
        const float inv_lists = 1.0f / (float)n_lists;
        for (int idx = tid; idx < entries * n_lists; idx += kThreads) {
            const int e = small_div(idx, inv_lists), c = idx - e * n_lists;
            const int l = small_div(e, inv_k), j = e - l * k;
            const u64 v = lists[l][j];
            if (v >= kSmallestWord) atomicAdd(&places[l][j], c == l ? j : count_larger(lists[c], k, v));
        }
        __syncthreads();
        const bool final_stage = stage == 1 || p.chunks == 1;
        for (int e = tid; e < entries; e += kThreads) {
            const int l = small_div(e, inv_k), j = e - l * k;
            const u64 v = lists[l][j];
            const int place = places[l][j];
            if (v >= kSmallestWord && place < k) {
                if (final_stage) out_tokens[place] = token_of(v);
                else __hip_atomic_store(exchange + chunk * 64 + place, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (final_stage) break;
        // a run shorter than k: 1 = "no token here" (a slot that has been written is never 0)
        if (tid >= end - begin && tid < k)
            __hip_atomic_store(exchange + chunk * 64 + tid, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // whoever arrives last finishes the row
        __syncthreads();
        DRAFT_WG_TIME(3);
        if (tid == 0) {
            const uint32_t arrived = __hip_atomic_fetch_add(p.arrivals + row, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = arrived == (uint32_t)(p.chunks - 1);
            if (s_last) __hip_atomic_store(p.arrivals + row, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        DRAFT_WG_TIME(4);
        if (!s_last) break;
        n_lists = p.chunks;
        for (int e = tid; e < n_lists * k; e += kThreads) {
            const int c = small_div(e, inv_k), j = e - c * k;
            u64* slot = exchange + c * 64 + j;
            // the writer's store may still be on its way: bounded wait, then leave the slot empty again
            u64 v = 0;
            for (uint32_t spin = 0; spin < p.spin_limit; ++spin) {
                v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v != 0) break;
                __builtin_amdgcn_s_sleep(1);
            }
            if (v == 0) s_bad = 1;
            __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            lists[c][j] = v;
            places[c][j] = 0;
        }
        __syncthreads();
        DRAFT_WG_TIME(5);
        // a timed-out wait (never seen; it would take a stalled device) leaves the row without tokens
        if (s_bad) {
            if (tid < k) out_tokens[tid] = -1;
            break;
        }
    }
    DRAFT_WG_TIME(6);
    }
}

int g_forced_chunks = 0;
int g_max_groups = SEQ_MAX_TREE * kMaxChunks;   // workgroups per launch, at most: as many as there can be runs

// Workgroups per row: enough to fill the chip, not more than the row has steps, and few enough
// that the last one's placement of chunks * k entries against chunks lists stays short
// (chunks^2 * k pairs, 256 at a time).  With many rows the per-workgroup fixed work (seeding,
// two placements, the hand-over) is what fills the chip, so the budget of pairs is halved:
// measured at 64 and 128 rows, 8 workgroups per row beat 16 by 4 us; at 1 row 16 beat 8 by 1 us.
void plan_chunks(int rows, int V, int k_max, int* chunks, int* chunk_tokens) {
    const int steps = (V + kStepTokens - 1) / kStepTokens;
    int want = (kTargetGroups + rows - 1) / rows;
    const int pair_budget = rows <= 8 ? 2048 : 1024;
    while (want > 1 && want * want * k_max > pair_budget) --want;
    if (g_forced_chunks > 0) want = g_forced_chunks;
    want = std::max(1, std::min(want, std::min(kMaxChunks, steps)));
    const int steps_per_chunk = (steps + want - 1) / want;
    *chunks = (steps + steps_per_chunk - 1) / steps_per_chunk;
    *chunk_tokens = steps_per_chunk * kStepTokens;
}

template <typename E, bool VEC>
void launch(const DraftParams& p, bool greedy, hipStream_t stream) {
    const dim3 grid(std::min(p.rows * p.chunks, g_max_groups));
    if (greedy) draft_sample_kernel<E, VEC, true><<<grid, kThreads, 0, stream>>>(p);
    else draft_sample_kernel<E, VEC, false><<<grid, kThreads, 0, stream>>>(p);
}

}  // namespace
}  // namespace seqtree

using namespace seqtree;

#ifdef SEQTREE_STAMPS
extern "C" void seqtree_internal_read_draft_wg_times(long long* out, int count) {
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_draft_wg_times), sizeof(long long) * 8 * count);
}
#endif

// Test hook: force the number of workgroups that share a row (0 = let the library choose).
extern "C" void seqtree_internal_set_draft_chunks(int chunks) { g_forced_chunks = chunks; }
// Test hook: the largest grid (0 = the default).  A small value makes every workgroup take many runs.
extern "C" void seqtree_internal_set_draft_max_groups(int groups) { g_max_groups = groups > 0 ? groups : SEQ_MAX_TREE * kMaxChunks; }

extern "C" size_t seq_draft_sample_workspace(int32_t n_rows, int32_t vocab, int32_t k_max, int32_t dtype) {
    (void)n_rows; (void)vocab; (void)k_max; (void)dtype;
    return 256;
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
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    SyncArea* sync = nullptr;
    int rc = get_sync_area(stream, &sync);
    if (rc != SEQ_OK) return rc;

    DraftParams p;
    p.logits = draft_logits;
    p.n_children = n_children;
    p.rng = rng;
    p.tokens = tokens;
    p.exchange = sync->draft_exchange;
    p.arrivals = sync->draft_arrivals;
    p.rows = n_rows;
    p.V = vocab;
    p.k_max = k_max;
    plan_chunks(n_rows, vocab, k_max, &p.chunks, &p.chunk_tokens);
    static_assert(SEQ_MAX_TREE * kMaxChunks <= kDraftMaxGroups, "exchange area");
    const bool greedy = temperature == 0.0f;
    p.inv_T = greedy ? 1.0f : 1.0f / temperature;
    p.spin_limit = 1u << 20;
    const bool vec = vocab % 8 == 0 && (reinterpret_cast<uintptr_t>(draft_logits) & 15) == 0;
    if (dtype == SEQ_BF16) {
        if (vec) launch<uint16_t, true>(p, greedy, stream); else launch<uint16_t, false>(p, greedy, stream);
    } else {
        if (vec) launch<float, true>(p, greedy, stream); else launch<float, false>(p, greedy, stream);
    }
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}
