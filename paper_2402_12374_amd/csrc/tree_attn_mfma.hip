// bf16 tree attention on the gfx950 matrix cores.
//
// Work split.  A "unit" is a block of 32 * WQ query rows of one KV head -- a query row is a
// (tree token i, head hh of the group) pair, numbered rho = i * G + hh -- and one workgroup of
// eight wavefronts owns a unit together with a contiguous range of 32-key tiles of the key axis
// [cache rows 0..P) ++ [tree rows 0..n).  The wavefronts form a WQ x WK grid (WQ * WK = 8):
// wavefront (wq, wk) keeps 32 query rows and takes every WK-th tile of the range.  Few query
// rows per KV head (small trees, no grouped heads): few row blocks, several key groups.
//
// Data path.  K and V tiles go from global memory straight into LDS (global_load_lds_dwordx4,
// 16 bytes per lane, no register staging) into a ring of kStages tile buffers, several tiles
// ahead of the one being consumed, so that the HBM/L2 latency of a tile is covered by the work
// on the tiles before it.  A copy's source is a scalar base (advanced by scalar arithmetic) plus
// a per-lane offset that never changes while the range is inside the prefix; the ring slot of
// every access is a compile-time constant (the tile loop is unrolled over the ring), so LDS
// addresses are one register plus an immediate.  Both tiles are stored row-major; 16-byte chunks are XOR-swizzled
// within their row (the LDS slot is fixed by the lane, so the swizzle is applied to the global
// address each lane fetches) so that the reads below are free of bank conflicts:
//   K is read as the A operand of S^T = K Q^T with ds_read_b128 (a lane = a key, 8 features);
//   V is read as the A operand of O^T += V^T P^T with ds_read_b64_tr_b16, the LDS transpose
//   read of gfx950: within 16 lanes, lanes 4r..4r+3 address 16 consecutive features of key r
//   and lane i receives feature i of the four keys.
// S^T is computed transposed so that a lane owns one query column: running maximum, normaliser
// and output rescaling are per-lane scalars and the only cross-lane step is one exchange with
// lane^32.  The accumulator layout of S^T is, value for value, the B-operand layout of the
// second product, so probabilities go from registers straight back into the matrix unit.
//
// Masking (which keys a tree token may see: cache rows below prefix_len, itself and its
// ancestors) is a bit test on one 32-bit word of the ancestor-or-self bitset per 32 keys; a
// masked score is replaced by -inf, so its weight is exactly zero.  Tile rows past the valid keys
// are filled with a copy of the last valid row (never with memory outside the valid range).
//
// When the key axis is cut into several ranges, every workgroup leaves (max, normaliser,
// normalised output in fp16) in the workspace and the last one to arrive for a unit merges them
// by log-sum-exp; no workgroup ever waits for another.
#include <algorithm>
#include <functional>
#include <mutex>
#include <type_traits>
#include <utility>

#include "seq_internal.h"
#include "tree_attn_kernels.h"
#include "fast_div.h"

namespace seqtree {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int kMaxCells = 8;          // (row block, key group) cells = wavefronts of a workgroup
constexpr int kRing = 8;              // tile buffers in the LDS ring
constexpr int kMaxSplits = 16;

struct MfmaParams {
    const uint16_t* q;
    const uint16_t* k_cache;
    const uint16_t* v_cache;
    const uint16_t* k_tree;
    const uint16_t* v_tree;
    uint16_t* out;
    const uint32_t* anc;
    int words_per_row;
    int P_bound, cap, n, H, Hk, G;   // P_bound: the prefix length, or its upper bound if prefix_lens is given
    int query_blocks;     // units per KV head
    int prefix_tiles_bound;   // ceil(P_bound / 32)
    const int32_t* prefix_lens;   // [sequences] or null: a prefix length per sequence of a batch
    FastDiv by_seq_kv_heads;      // KV heads per sequence (KV head g belongs to sequence g / that)
    int splits;
    int short_ranges, short_weight, long_weight;   // the first short_ranges key ranges of a unit have weight short_weight, the others long_weight
    int long_tiles;       // > 0: every long range has this many tiles, whatever its unit's number of tiles (see range_start)
    int keep_own;         // a long range's workgroup may keep its partial result in registers (see the end of the tile loop)
    float* partials;
    uint32_t* counters;
    float scale_log2;     // log2(e) / sqrt(D)
    int share_l2;         // all workgroups of a unit run on one XCD (checked once per device)
    FastDiv by_units_per_xcd, by_query_blocks, by_G, by_weights;   // the divisions of the prologue (by_weights: by the sum of the ranges' weights)
    FastDiv by_short_ranges;
};

// First tile of key range `range` (of `ranges`) of a unit with `tiles` tiles.  The first
// `short_ranges` ranges have weight `short_weight`, the others `long_weight`; `by_weights` divides
// by the sum of all weights (equal ranges: no short ones, weight 1, the sum is their number).
// tiles x sum < 2^31.
// With `long_tiles` > 0 the long ranges are the same length in every unit instead, counted from
// the end of the unit's tiles, and the short ranges share what is left: the units of a KV head
// differ in their tree tiles (the last row block sees all of them, the first one tile), a long
// range is a workgroup with a compute unit to itself from the start of the launch to its end,
// and the launch ends with the longest of them; the short ranges run several in a row, so their
// differences average out.
__host__ __device__ __forceinline__ int range_start(int tiles, int range, int ranges, int short_ranges, int short_weight,
                                                    int long_weight, int long_tiles, const FastDiv& by_weights,
                                                    const FastDiv& by_short_ranges) {
    if (long_tiles > 0) {
        const int shorts_end = tiles - (ranges - short_ranges) * long_tiles;
        const int short_total = shorts_end > 0 ? shorts_end : 0;
        if (range <= short_ranges) return (int)fast_div((uint32_t)short_total * (uint32_t)range, by_short_ranges);
        const int start = tiles - (ranges - range) * long_tiles;
        return start > short_total ? start : short_total;
    }
    const int before = range <= short_ranges ? range * short_weight
                                             : short_ranges * short_weight + (range - short_ranges) * long_weight;
    return (int)fast_div((uint32_t)tiles * (uint32_t)before, by_weights);
}

// A pointer that is the same in every lane, moved to scalar registers whatever the compiler
// believes about it.
__device__ __forceinline__ const void* scalar_pointer(const void* p) {
    const uint64_t bits = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)bits);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(bits >> 32));
    return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}

// 16 bytes per lane from global memory (uniform base + per-lane byte offset) into LDS at
// lds_base + lane * 16 (lds_base uniform).
__device__ __forceinline__ void async_copy16(uint32_t lane_offset, const void* base, uint32_t lds_base) {
    uint32_t saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %3\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved)
        : "v"(lane_offset), "s"(scalar_pointer(base)), "s"(__builtin_amdgcn_readfirstlane(lds_base))
        : "memory");
}

// 4 bytes per lane into LDS at lds_base + lane * 4.
__device__ __forceinline__ void async_copy4(uint32_t lane_offset, const void* base, uint32_t lds_base) {
    uint32_t saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %3\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dword %1, %2\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved)
        : "v"(lane_offset), "s"(scalar_pointer(base)), "s"(__builtin_amdgcn_readfirstlane(lds_base))
        : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(lds_ptr_t)p;
}

// Swizzles: chunk c (16 bytes) of row r of a tile lives in slot c ^ swz(r) of that row.
template <int D> __device__ __forceinline__ int k_swizzle(int row) { return row & (D / 8 - 1); }
template <int D> __device__ __forceinline__ int v_swizzle(int row) {
    return D == 128 ? (row & 3) << 2 : ((row >> 1) & 1) << 2;
}

// Phase timestamps of one thread of workgroup 0 (100 MHz wall clock), compiled in with
// -DSEQTREE_STAMPS only.  They are kept in LDS while the kernel runs -- a stamp that touched global
// memory would wait for, or add to, the copies in flight that the tile loop counts -- and written
// out where the thread leaves the kernel.
#ifdef SEQTREE_STAMPS
#ifndef SEQTREE_STAMP_THREAD
#define SEQTREE_STAMP_THREAD 0
#endif
#ifndef SEQTREE_STAMP_BLOCK
#define SEQTREE_STAMP_BLOCK 0
#endif
#ifndef SEQTREE_STAMP_WANTED
#define SEQTREE_STAMP_WANTED(id) true   // e.g. ((id) < 10 || (id) >= 20): everything but the tile loop
#endif
__device__ long long g_attn_stamps[128];
__device__ int g_attn_stamp_count;
__device__ long long g_attn_wg_times[2 * 4096];   // start and end of every workgroup
#define ATTN_STAMP_RESET() __shared__ long long s_stamps[128]; int stamp_count = 0; \
    const bool stamp_on = blockIdx.x == SEQTREE_STAMP_BLOCK && threadIdx.x == SEQTREE_STAMP_THREAD; \
    if (threadIdx.x == 0 && blockIdx.x < 4096) { g_attn_wg_times[2 * blockIdx.x] = wall_clock64(); g_attn_wg_times[2 * blockIdx.x + 1] = 0; }
#define ATTN_STAMP(id) do { if (stamp_on && stamp_count < 63 && SEQTREE_STAMP_WANTED(id)) { \
    s_stamps[2 * stamp_count] = (id); s_stamps[2 * stamp_count + 1] = wall_clock64(); ++stamp_count; } } while (0)
#define ATTN_STAMP_FLUSH() do { if (stamp_on) { \
    for (int i = 0; i < 2 * stamp_count; ++i) g_attn_stamps[i] = s_stamps[i]; g_attn_stamp_count = stamp_count; } \
    if (threadIdx.x == 0 && blockIdx.x < 4096) g_attn_wg_times[2 * blockIdx.x + 1] = wall_clock64(); } while (0)
#else
#define ATTN_STAMP_RESET() do {} while (0)
#define ATTN_STAMP(id) do {} while (0)
#define ATTN_STAMP_FLUSH() do {} while (0)
#endif

// LDS: a ring of kRing tile buffers (K and V of 32 keys each), and a ring of visibility words.
// After the last tile the K ring is reused to merge the key groups of the workgroup.
template <int D, int kCells>
struct Rings {
    static constexpr int kTileElems = kKeyTile * D;   // bf16 elements per K (or V) tile
    uint16_t k[kRing][kTileElems];
    uint16_t v[kRing][kTileElems];
    uint32_t mask[kRing][kCells][64];
};

template <int D, int WQ, int kCells>
constexpr size_t epilogue_bytes() {
    // (with a single key group, kCells == WQ, the accumulators never pass through LDS)
    return sizeof(float) * (kCells == WQ ? 64 : (size_t)kCells * (D / 32) * 4 * 256 + kCells * 128);
}

template <int D, int WQ, int kCells>
union Smem {
    Rings<D, kCells> r;
    char epilogue[epilogue_bytes<D, WQ, kCells>()];
};

// ---- pieces of the tile loop shared by its two forms ---------------------------------------

// lane ^ 32 exchange on the gfx950 lane-swap instruction (no LDS round trip): max / sum of a
// value over the two halves of the wavefront, in every lane.
__device__ __forceinline__ float halves_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Replace the scores of invisible keys by -inf.  m: bit x <=> key x of the tile is visible to
// the query of this lane; accumulator element x holds key (x/4)*8 + half*4 + x%4.
__device__ __forceinline__ void mask_scores(f32x16_t& s, uint32_t m, int half) {
    m >>= half * 4;
#pragma unroll
    for (int x = 0; x < 16; ++x) s[x] = ((m >> ((x >> 2) * 8 + (x & 3))) & 1u) ? s[x] : -INFINITY;
}

// One step of the online softmax for one query column per lane: scores of 32 keys in, their
// probabilities out (packed bf16, in the B-operand layout of the second product).
//
// m_run is the reference the exponentials are taken against, not necessarily the running
// maximum: it only moves when a score exceeds it by more than kSlack (in log2 units), so that
// probabilities stay below 2^kSlack and the output accumulated so far has to be rescaled
// rarely -- after the first few tiles, almost never.  Numerator and normaliser share the
// reference, so the quotient is unchanged.
//
// The step comes in two halves of about equal cost, so that a wavefront may take them on either
// side of a workgroup barrier: the first finds the reference and turns keys 0..15 of the tile
// (accumulator elements 0..7) into probabilities, the second does keys 16..31 and closes the
// normaliser.  `alpha` is the factor the output accumulated so far has to be scaled by (1 unless
// `moved`).
constexpr float kSlack = 8.0f;
struct SoftmaxCarry {
    float ref, alpha, psum;
};
__device__ __forceinline__ void softmax_pack8(const f32x16_t& s, int x0, float scale_log2, float ref, uint32_t (&pw)[4], float& psum) {
    const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int x = 0; x < 8; x += 2) {
        f32x2_t e;
        e[0] = __builtin_amdgcn_exp2f(fmaf(s[x0 + x], scale_log2, -ref));
        e[1] = __builtin_amdgcn_exp2f(fmaf(s[x0 + x + 1], scale_log2, -ref));
        const bf16x2_t pk = __builtin_convertvector(e, bf16x2_t);
        pw[x >> 1] = __builtin_bit_cast(uint32_t, pk);
        psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);   // the normaliser sums what the product sees
    }
}
__device__ __forceinline__ SoftmaxCarry softmax_first(const f32x16_t& s, float scale_log2, float& m_run,
                                                      uint32_t (&pw)[2][4], bool& moved) {
    float mx = __builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), s[2]);   // three-operand maxima
#pragma unroll
    for (int x = 3; x < 15; x += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[x]), s[x + 1]);
    mx = fmaxf(mx, s[15]);
    mx = halves_max(mx) * scale_log2;
    moved = mx > m_run + kSlack || (m_run == -INFINITY && mx != -INFINITY);
    const float m_new = moved ? mx : m_run;
    SoftmaxCarry c;
    c.ref = (m_new == -INFINITY) ? 0.f : m_new;
    c.alpha = moved ? __builtin_amdgcn_exp2f(m_run - c.ref) : 1.0f;
    c.psum = 0.f;
    m_run = m_new;
    softmax_pack8(s, 0, scale_log2, c.ref, pw[0], c.psum);
    return c;
}
__device__ __forceinline__ void softmax_second(const f32x16_t& s, float scale_log2, SoftmaxCarry c, float& l_run,
                                               uint32_t (&pw)[2][4]) {
    softmax_pack8(s, 8, scale_log2, c.ref, pw[1], c.psum);
    l_run = l_run * c.alpha + c.psum;
}


// One workgroup = a unit of 32 * WQ query rows x a range of key tiles; wavefront w is cell
// (row block w % WQ, key group w / WQ) of its WQ x WK grid.
//
// What bounds the tile loop at large trees (timing of variants with one part of the work taken
// out, and of single instructions): per tile and wavefront, 16 matrix instructions (512 clocks of
// the SIMD's matrix pipe) stand against about 70 vector instructions.  One wavefront issues a
// vector instruction every 6 clocks at best, every 9 to 11 when it needs the result of the one
// before, so a tile's softmax takes a wavefront 600 to 1000 clocks however idle the SIMD is; the
// vector pipe has room for the second wavefront of the SIMD beside it, the matrix pipe does not.
// A round of the two wavefronts of a SIMD costs about the two products of both (1024 clocks)
// plus one softmax: taking the softmax out of the loop nearly halves the kernel, taking out half
// of the matrix instructions saves a tenth, taking out the exponentials alone 2 %.  Vector work
// that is not softmax arithmetic is kept out of the loop: addresses are scalar or immediate, row
// sums ride on dot2 instructions, the output is rescaled only when a score outgrows the
// reference by 2^8.  Tried and not faster here:
//  - two row blocks per wavefront in four fat wavefronts (halves the LDS traffic, but the
//    accumulators no longer fit the vector registers and travel through AGPR moves); twelve
//    wavefronts; two workgroups of four wavefronts per CU with half the ring each;
//  - raising the priority of a wavefront around its matrix instructions, or around its softmax;
//    fetching the V fragments from LDS before the softmax instead of after it;
//  - scores one tile ahead of the softmax (so that a wavefront has matrix work in flight while
//    it takes exponentials), with the compiler's instruction order or with one matrix
//    instruction pinned after every six vector instructions;
//  - on top of that, the two wavefronts of a SIMD taking turns, one in a matrix phase (scores of
//    tile t + 1, weighted values of tile t) while the other is in its vector phase, a barrier at
//    every change: the matrix work then hides completely, but a lone wavefront's vector phase
//    takes as long as both phases took before; and the same with two tiles per phase (two
//    independent softmax steps fill each other's latencies: the vector phase of a pair of tiles
//    then takes 0.55 us), K copied a pair of tiles further ahead than V, fragments requested
//    from LDS a group ahead of their matrix instructions: now the 32 matrix instructions of a
//    phase take 1.04 us beside the other wavefront's vector phase, twice what they take alone,
//    and the kernel is as fast as before;
//  - the scale folded into Q and minus the reference as the start value of the score product, so
//    that the accumulator comes back as the exponent (one vector instruction per score less, 16
//    registers more: 20 % slower);
//  - splitting a tile's work into a matrix phase and a vector phase for all wavefronts at once,
//    or rotating the loop of wavefronts 4..7 by half a tile;
//  - dealing equal spans of an XCD's (unit, tile) sequence to 256 workgroups instead of equal key
//    ranges: the second prologue, epilogue and merge of a span that crosses into the next unit
//    cost what the even load saves, and wrapping the body in a loop over the pieces of a span
//    makes the compiler's tile loop 10-15 % slower.
template <int D, int WQ, int WK>
__global__ __launch_bounds__(WQ * WK * 64) void tree_attn_mfma_kernel(const MfmaParams p) {
    constexpr int kCells = WQ * WK;
    constexpr int R = 1;   // row blocks per wavefront (the loops below are written for R of them)
    static_assert(kCells == 8 && R == 1, "cell grid");
        constexpr int kW = kCells / R;         // wavefronts
    constexpr int kT = kW * 64;            // threads
    constexpr int WQW = WQ / R;            // wavefronts along the query axis
    constexpr int kKSteps = D / 16;        // contraction steps of Q K^T
    constexpr int kDBlocks = D / 32;       // 32-row blocks of O^T
    constexpr int kChunks = D / 8;         // 16-byte chunks per K/V row
    constexpr int kRowBytes = D * 2;
    constexpr int kRowsPerCopy = 64 / kChunks;               // rows one wave-wide copy covers
    constexpr int kCopiesPerTile = kKeyTile / kRowsPerCopy;  // per K (or V) tile
    constexpr int kCopiesPerRound = 2 * kCopiesPerTile * WK; // K and V of the WK tiles of a round
    constexpr int kCopiesPerWave = kCopiesPerRound / kW;
    constexpr int kLoadsPerRound = kCopiesPerWave + R;       // + my visibility words
    static_assert(kCopiesPerRound % kW == 0, "copies divide evenly among the wavefronts");
    constexpr int kAheadRounds = kRing / WK - 1;             // rounds in flight beyond the one being waited for
    constexpr int kUnitRows = 32 * WQ;
    constexpr uint32_t kTileBytes = kKeyTile * D * 2;
    static_assert(kAheadRounds >= 1, "ring too small");
    static_assert(kAheadRounds * kLoadsPerRound <= 63, "vmcnt is a 6-bit counter");
    using SM = Smem<D, WQ, kCells>;
    __shared__ __attribute__((aligned(1024))) SM sm_union;
    Rings<D, kCells>& sm = sm_union.r;
    __shared__ int s_last;

    ATTN_STAMP_RESET();
    ATTN_STAMP(0);
    // The arguments span four cache lines that nobody has touched yet; left to itself the compiler
    // fetches them in three groups where they are first needed, a trip to memory each.  Asking
    // for one field of every line here puts all of them in flight at once.
    asm volatile("" :: "s"(p.q), "s"(p.words_per_row), "s"(p.scale_log2), "s"(p.by_weights.one));
    const int S = p.splits;
    const int bid = blockIdx.x;
    // Consecutive workgroup ids go to consecutive XCDs, each with its own L2.  Give every XCD a
    // contiguous run of units: all key ranges of a unit, and all units of a KV head, then share
    // one L2, which holds that head's K and V for all of them.
    const int xcd = bid & 7, idx = bid >> 3;
    const int total_units = p.Hk * p.query_blocks;
    const int units_per_xcd = (total_units + 7) >> 3;
    // Range-major within an XCD: the workgroups that run at the same time then mostly work on
    // the same key range of their head and find its tiles in L2.
    // (An integer division is a 25-instruction sequence on the vector unit, fetched cold, and it
    // leaves its result in a vector register even when every lane computes the same thing, so
    // that everything derived from it would be vector arithmetic and every branch on it a
    // divergent one.  All divisors here are fixed per launch: the host supplies multipliers, and
    // a uniform quotient is three scalar instructions.)
    // Dearest first: the last range of a unit holds the tree tiles (masked, so slower per tile),
    // and the last query blocks of a head see the most of them.  When a launch takes several
    // batches of workgroups, what is left for the last batch should be the cheap ones.
    const int turn = (int)fast_div((uint32_t)idx, p.by_units_per_xcd);
    const int local = units_per_xcd - 1 - (idx - turn * units_per_xcd);
    const int unit = xcd * units_per_xcd + local;
    if (turn >= S || unit >= total_units) return;
    const int split = S - 1 - turn;
    const int g = (int)fast_div((uint32_t)unit, p.by_query_blocks);
    const int qb = unit - g * p.query_blocks;
    // The prefix length: one for the whole launch, or -- a batch whose sequences differ in it --
    // that of the sequence this KV head belongs to, read from device memory (so that a captured
    // launch follows the lengths as they change) and held to the bound the host planned with.
    int P = p.P_bound, prefix_tiles = p.prefix_tiles_bound;
    if (p.prefix_lens) {
        const int seq = (int)fast_div((uint32_t)g, p.by_seq_kv_heads);
        P = __builtin_amdgcn_readfirstlane(min(max(p.prefix_lens[seq], 0), p.P_bound));
        prefix_tiles = (P + kKeyTile - 1) / kKeyTile;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform, and the compiler knows it
    __builtin_assume(wave >= 0 && wave < kW);   // (lets the copy plan below fold: most of its items coincide)
    const int wqw = wave % WQW, wk = wave / WQW;   // place of this wavefront in the cell grid
    const int half = lane >> 5, col = lane & 31;
    const int rows = p.G * p.n;
    // my R row blocks: rb = wqw * R + r; cell = wk * WQ + rb
    const bool blk_valid = qb * kUnitRows + wqw * R * 32 < rows;
    bool qvalid[R];
    int qi[R], qh[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int qrow = qb * kUnitRows + (wqw * R + r) * 32 + col;
        qvalid[r] = qrow < rows;
        const int node = (int)fast_div((uint32_t)qrow, p.by_G);
        qi[r] = qvalid[r] ? node : 0;
        qh[r] = qvalid[r] ? g * p.G + (qrow - node * p.G) : 0;
    }

    // key tiles of this workgroup
    const int last_row = min(rows - 1, qb * kUnitRows + kUnitRows - 1);
    const int i_max = (int)fast_div((uint32_t)last_row, p.by_G);   // tree rows beyond i_max are masked for all
    const int tree_tiles = i_max / kKeyTile + 1;
    const int total_tiles = prefix_tiles + tree_tiles;
    // (at most 2^26 tiles times 16 ranges: below 2^31)
    const int t_begin = range_start(total_tiles, split, S, p.short_ranges, p.short_weight, p.long_weight, p.long_tiles, p.by_weights, p.by_short_ranges);
    const int t_end = range_start(total_tiles, split + 1, S, p.short_ranges, p.short_weight, p.long_weight, p.long_tiles, p.by_weights, p.by_short_ranges);
    const int n_rounds = (t_end - t_begin + WK - 1) / WK;

    const uint32_t k_lds = lds_address(&sm.k[0][0]);
    const uint32_t v_lds = lds_address(&sm.v[0][0]);
    const uint32_t m_lds = lds_address(&sm.mask[0][0][0]);

    // One round = the WK tiles t_begin + rho*WK .. +WK-1; tile j of the range lives in ring
    // buffer j % kRing.  Every wavefront issues the same number of copies per round (the waits
    // below count them), so tiles past the end of the range and rows past the valid keys fetch
    // valid memory that is never used: the last valid row of the last tile.
    // What a copy of mine moves is fixed for the whole kernel (which tile of the round, K or V,
    // which 1 KB block of the tile).  A copy's source is a uniform base, advanced by scalar
    // arithmetic, plus a per-lane byte offset that for tiles inside the prefix never changes.
    int cp_row[kCopiesPerWave];
    uint32_t cp_lane_off[kCopiesPerWave];   // (row * D + swizzled chunk) * 2 bytes: prefix layout
    uint32_t cp_chunk_bytes[kCopiesPerWave];
#pragma unroll
    for (int c = 0; c < kCopiesPerWave; ++c) {
        const int item = wave + c * kW;                       // (tile of the round, K|V, copy)
        const int is_v = (item / kCopiesPerTile) & 1, copy = item % kCopiesPerTile;
        cp_row[c] = copy * kRowsPerCopy + lane / kChunks;
        const int swz = is_v ? v_swizzle<D>(cp_row[c]) : k_swizzle<D>(cp_row[c]);
        cp_chunk_bytes[c] = (uint32_t)(((lane % kChunks) ^ swz) * 16);
        cp_lane_off[c] = (uint32_t)cp_row[c] * kRowBytes + cp_chunk_bytes[c];
    }
    uint32_t mask_lane_off[R];   // my query's row of the ancestor bitset
#pragma unroll
    for (int r = 0; r < R; ++r) mask_lane_off[r] = qvalid[r] ? (uint32_t)(qi[r] * p.words_per_row) * 4u : 0u;

    // Issue the copies of round rho into ring slot `slot` = rho % (kRing / WK).  (Every helper
    // below takes the slot as a plain int and is inlined: where the tile loop is unrolled over
    // the ring the slot is a literal and ends up in the instructions' offset fields.)
    auto issue_round = [&](int rho, int slot) __attribute__((always_inline)) {
        const int j0 = rho * WK;
        const bool inside = (t_begin + j0 + WK) * kKeyTile <= P && t_begin + j0 + WK <= t_end;
#pragma unroll
        for (int c = 0; c < kCopiesPerWave; ++c) {
            const int item = wave + c * kW;
            const int is_v = (item / kCopiesPerTile) & 1, copy = item % kCopiesPerTile;
            const int tr = item / (2 * kCopiesPerTile);
            const uint32_t dst = (is_v ? v_lds : k_lds) + (uint32_t)copy * 1024u + (uint32_t)(slot * WK + tr) * kTileBytes;
            const int t = max(min(t_begin + j0 + tr, t_end - 1), 0);
            if (inside) {   // every tile of the round lies wholly inside the prefix
                const uint16_t* base = (is_v ? p.v_cache : p.k_cache) + ((size_t)g * p.cap + (size_t)t * kKeyTile) * D;
                async_copy16(cp_lane_off[c], base, dst);
            } else {
                const bool is_prefix = t < prefix_tiles;
                const int key0 = is_prefix ? t * kKeyTile : (t - prefix_tiles) * kKeyTile;
                const int limit = is_prefix ? P : p.n;
                const uint16_t* base = is_prefix ? (is_v ? p.v_cache : p.k_cache) + (size_t)g * p.cap * D
                                                 : (is_v ? p.v_tree : p.k_tree) + (size_t)g * D;
                const uint32_t row_bytes = is_prefix ? (uint32_t)kRowBytes : (uint32_t)(p.Hk * kRowBytes);
                const int key = min(key0 + cp_row[c], limit - 1);
                async_copy16((uint32_t)key * row_bytes + cp_chunk_bytes[c], base, dst);
            }
        }
        // visibility words of my queries for my tile of this round (used for tree tiles only)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int t = max(min(t_begin + j0 + wk, t_end - 1), 0);
            const int word = min(max(t - prefix_tiles, 0), p.words_per_row - 1);
            const int cell = wk * WQ + wqw * R + r;
            async_copy4(mask_lane_off[r], p.anc + word, m_lds + (uint32_t)(((slot * WK + wk) * kCells + cell) * 256));
        }
    };
    // One turn of the ring: rounds rho0 .. rho0 + kSlots - 1 (rho0 a multiple of kSlots), each
    // through a copy of the body that is given its slot as a literal.
    constexpr int kSlots = kRing / WK;
    auto one_turn = [&](int rho0, int rho_end, auto&& body) __attribute__((always_inline)) {
        [&]<int... Is>(std::integer_sequence<int, Is...>) __attribute__((always_inline)) {
            (void)(((rho0 + Is < rho_end) ? (body(rho0 + Is, Is), true) : false) && ...);
        }(std::make_integer_sequence<int, kSlots>{});
    };

    // Q fragments (B operand): lane holds query `col`, features ks*16 + half*8 .. +7.  Requested
    // first, settled after the tile copies have been issued.
    bf16x8_t qf[R][kKSteps];
    constexpr bool kEagerQ = WK > 1;
    ATTN_STAMP(3);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint16_t* qp = p.q + ((size_t)qi[r] * p.H + qh[r]) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            // Short key ranges: a row past the end reads row 0 and is zeroed below (under a
            // condition the compiler waits for one of these loads on the spot, a trip to memory
            // before the first copy is issued).  Long ranges keep the conditional form: there the
            // trip hides behind the copies, and the registers the other form leaves the fragments
            // in make the unrolled tile loop 1.5 % slower.
            uint4 v = make_uint4(0, 0, 0, 0);
            if (kEagerQ || qvalid[r]) v = *reinterpret_cast<const uint4*>(qp + ks * 16);
            qf[r][ks] = __builtin_bit_cast(bf16x8_t, v);
        }
    }

    // start the tile pipeline (a rolled loop: code that runs once is fetched cold, and slowly)
    ATTN_STAMP(4);
#pragma unroll 1
    for (int a = 0; a < kAheadRounds; ++a) { issue_round(a, a); ATTN_STAMP(5); }
    ATTN_STAMP(1);

    // Make the compiler settle these loads here.  It cannot see the copies issued in assembly,
    // and a wait for the Q fragments placed at their first use inside the tile loop would also
    // wait, on every iteration, for every copy in flight.  (Loading Q in assembly as well, to
    // count its wait exactly, is not an option: the compiler may move or reuse the destination
    // registers of a load it does not know to be in flight.)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            asm volatile("" : "+v"(qf[r][ks]));
            if (kEagerQ) {
                uint4 v = __builtin_bit_cast(uint4, qf[r][ks]);
                const uint32_t keep = qvalid[r] ? ~0u : 0u;
                v.x &= keep; v.y &= keep; v.z &= keep; v.w &= keep;
                qf[r][ks] = __builtin_bit_cast(bf16x8_t, v);
            }
        }
    ATTN_STAMP(2);

    // Per-lane LDS addresses of my fragments in ring buffer `wk` (my key group's tile of slot
    // 0), fixed for the whole kernel; the slot and everything else in an address are
    // compile-time constants that go into the instruction's offset field.
    //   K (ds_read_b128): key row `col`, chunk (2*ks + half) ^ swizzle
    //   V (transpose read): 16-lane group, lanes 4r..4r+3 address 16 features of key row r
    typedef __attribute__((address_space(3))) const char* lds_cptr;
    const int grp = lane >> 4, li = lane & 15;
    lds_cptr kaddr[kKSteps], vaddr[kDBlocks];
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks)
        kaddr[ks] = (lds_cptr)(lds_ptr_t)&sm.k[0][0] + wk * kTileBytes +
                    (uint32_t)(col * kRowBytes + (((ks * 2 + half) ^ k_swizzle<D>(col)) * 16));
#pragma unroll
    for (int b = 0; b < kDBlocks; ++b) {
        const int vrow = half * 4 + (li >> 2);                    // + (2m+a)*8, multiples of 8
        const int feat = b * 32 + (grp & 1) * 16 + (li & 3) * 4;  // 4 features = 8 bytes
        vaddr[b] = (lds_cptr)(lds_ptr_t)&sm.v[0][0] + wk * kTileBytes +
                   (uint32_t)(vrow * kRowBytes + (((feat >> 3) ^ v_swizzle<D>(vrow)) * 16) + (feat & 7) * 2);
    }
    const __attribute__((address_space(3))) uint32_t* maddr[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
        maddr[r] = (const __attribute__((address_space(3))) uint32_t*)(lds_ptr_t)&sm.mask[wk][wk * WQ + wqw * R + r][col];

    f32x16_t oacc[R][kDBlocks];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) oacc[r][b][x] = 0.f;
    float m_run[R], l_run[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { m_run[r] = -INFINITY; l_run[r] = 0.f; }

    // S^T = K Q^T for my row blocks (32 keys x 32 queries each), tile in ring slot `slot`.  All
    // K fragments are requested before the first matrix instruction: one LDS latency per tile.
    auto load_k = [&](int slot, bf16x8_t (&kf)[kKSteps]) __attribute__((always_inline)) {
        const uint32_t kSlotBytes = (uint32_t)slot * WK * kTileBytes;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks)
            kf[ks] = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(kaddr[ks] + kSlotBytes);
    };
    auto scores = [&](const bf16x8_t (&kf)[kKSteps], f32x16_t (&sacc)[R]) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (ks == 0) {
                    f32x16_t zero;
#pragma unroll
                    for (int x = 0; x < 16; ++x) zero[x] = 0.f;
                    sacc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[r][ks], zero, 0, 0, 0);
                } else {
                    sacc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[r][ks], sacc[r], 0, 0, 0);
                }
            }
        }
    };
    // Visibility of the keys of tile t (ring slot `slot`) for the queries of this lane.
    auto tile_is_full = [&](int t) __attribute__((always_inline)) { return t < prefix_tiles && (t + 1) * kKeyTile <= P; };
    auto visibility = [&](int t, int slot, int r) __attribute__((always_inline)) -> uint32_t {   // selects only, no branches
        const int left = P - t * kKeyTile;
        const uint32_t in_prefix = left >= 32 ? 0xFFFFFFFFu : (left <= 0 ? 0u : ((1u << left) - 1u));
        const int word = t - prefix_tiles;
        const uint32_t in_tree = maddr[r][slot * WK * kCells * 64];
        return t < prefix_tiles ? in_prefix : ((qvalid[r] && word < p.words_per_row) ? in_tree : 0u);
    };
    // O^T += V^T P^T.  Matrix step m contracts keys (2m+a)*8 + half*4 + 0..3, a = 0,1 -- the
    // keys whose probabilities sit in accumulator elements 8m..8m+7.
    auto weighted_values = [&](int slot, const uint32_t (&pw)[R][2][4]) __attribute__((always_inline)) {
        const uint32_t kSlotBytes = (uint32_t)slot * WK * kTileBytes;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            bf16x8_t pf[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint4 pq;
                pq.x = pw[r][m][0]; pq.y = pw[r][m][1]; pq.z = pw[r][m][2]; pq.w = pw[r][m][3];
                pf[r] = __builtin_bit_cast(bf16x8_t, pq);
            }
#pragma unroll
            for (int b = 0; b < kDBlocks; ++b) {
                v4i16 part[2];
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    part[a] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (v4i16 __attribute__((address_space(3)))*)(vaddr[b] + kSlotBytes + ((2 * m + a) * 8) * kRowBytes));
                uint4 vw;
                vw.x = __builtin_bit_cast(uint2, part[0]).x;
                vw.y = __builtin_bit_cast(uint2, part[0]).y;
                vw.z = __builtin_bit_cast(uint2, part[1]).x;
                vw.w = __builtin_bit_cast(uint2, part[1]).y;
#pragma unroll
                for (int r = 0; r < R; ++r)
                    oacc[r][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vw), pf[r], oacc[r][b], 0, 0, 0);
            }
        }
    };
    auto rescale = [&](int r, float alpha) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) oacc[r][b][x] *= alpha;
    };

    // The K fragments of a wavefront's next tile are requested while its current tile is still
    // being worked on: right after a barrier all eight wavefronts would otherwise ask LDS for
    // their fragments at once and sit out the queue.  That tile therefore has to be in LDS one
    // barrier earlier, which takes a ring of more than two rounds: one or two key groups (with
    // two the gain is small, 1 % at the Vicuna shape; with one it is what the long loops need).
    constexpr bool kPrefetchK = WK <= 2;
    bf16x8_t kf[kKSteps];
    if (kPrefetchK) {
        wait_vmcnt<(kAheadRounds - 1) * kLoadsPerRound>();
        __syncthreads();   // tile 0 is in LDS
        load_k(0, kf);
    }
    auto round = [&](int rho, int slot) __attribute__((always_inline)) {
        // my copies of the round needed next have landed once at most the copies of the rounds
        // issued after it are in flight (copies complete in order)
        wait_vmcnt<(kAheadRounds - 1 - (kPrefetchK ? 1 : 0)) * kLoadsPerRound>();
        ATTN_STAMP(10);
        __syncthreads();   // everybody's copies are in LDS; the previous round's buffers are free
        ATTN_STAMP(11);
        issue_round(rho + kAheadRounds, (slot + kAheadRounds) % kSlots);
        const int t = t_begin + rho * WK + wk;
        if (!blk_valid || t >= t_end) return;
        f32x16_t sacc[1];
        if (!kPrefetchK) {
            load_k(slot, kf);   // all K fragments before the first matrix instruction: one LDS latency per tile
            __builtin_amdgcn_sched_barrier(0);
        }
        scores(kf, sacc);
        if (kPrefetchK) load_k((slot + 1) % kSlots, kf);   // (past the last tile: a tile nobody needs)
        ATTN_STAMP(12);
        if (!tile_is_full(t)) {   // tiles inside the prefix need no mask
            // A tree tile that holds no ancestor of any of my 32 queries adds nothing for them: a
            // node has at most depth-many ancestors, so most (row block, tree tile) pairs are like
            // that.  The wavefront leaves the tile out once it has the visibility words, after the
            // score product (leaving before it as well made the compiler run out of registers and
            // wait for every V fragment on the spot); the copies and the barrier are the workgroup's
            // and stay.
            const uint32_t vis = visibility(t, slot, 0);
            if (t >= prefix_tiles && !__any(vis != 0u)) return;
            mask_scores(sacc[0], vis, half);
        }
        uint32_t pw[1][2][4];
        bool moved;
        const SoftmaxCarry c = softmax_first(sacc[0], p.scale_log2, m_run[0], pw[0], moved);
        if (__any(moved)) rescale(0, c.alpha);   // the reference of some column moved
        softmax_second(sacc[0], p.scale_log2, c, l_run[0], pw[0]);
        ATTN_STAMP(13);
        weighted_values(slot, pw);
    };
    if constexpr (WK == 1) {
        // long key ranges, many rounds: unrolled over the ring, slots are literals
        for (int rho0 = 0; rho0 < n_rounds; rho0 += kSlots) one_turn(rho0, n_rounds, round);
    } else {
        // few rounds per workgroup: one copy of the body, fetched once; the slot costs a few
        // additions per tile
#pragma unroll 1
        for (int rho = 0; rho < n_rounds; ++rho) round(rho, rho % kSlots);
    }
    // A long range of a two-size schedule ends long after its unit's short range: if every other
    // range of the unit has been counted as arrived by now, this workgroup is the one that merges,
    // and its own partial result need not travel through memory.  (One lane asks, beside the
    // last copies; the answer is shared through the barrier that follows.  Only where the merge
    // below takes a single batch, so that the kept items are register arrays with literal indices.
    // Long ranges are what workgroups of eight row blocks get: the kernels for short ranges,
    // whose epilogue is most of their time, do not carry the code.)
    constexpr int kKeepUpTo = WK == 1 ? 2 : 0;
    const bool may_keep = kKeepUpTo > 0 && p.keep_own && p.short_ranges > 0 && split >= p.short_ranges && S <= kKeepUpTo;
    uint32_t seen_arrived = 0;
    if (may_keep && tid == 0) seen_arrived = __hip_atomic_load(&p.counters[unit], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    wait_vmcnt<0>();   // nothing of mine may still be landing in LDS when the ring is reused below
    ATTN_STAMP(20);
    if (tid == 0) s_last = may_keep && seen_arrived == (uint32_t)(S - 1);

    // ---- epilogue ---------------------------------------------------------------------------
    // Code that runs once per workgroup is fetched cold, at a small fraction of the speed of a
    // loop that sits in the instruction cache, and for short key ranges the epilogue is most of
    // the kernel: it is kept short, and every pass over LDS or the workspace that can be left
    // out is left out.
    //
    // Wavefronts of the same row block hold their cells in the same register layout, so the key
    // groups of a workgroup are merged lane by lane, through LDS (the tile rings, free by now),
    // and the merged row block goes to `out` (single range) or the workspace.
    //   o[cell][k4][lane][4]   unnormalised output; k4 = b*4 + rq holds features
    //                          b*32 + rq*8 + half*4 .. +3 of query (lane % 32), half = lane / 32
    //   ml[cell][2][64]        running maximum and (per-lane part of the) normaliser
    // A range's partial result in the workspace has the same shape, but its output is normalised
    // and kept in fp16 (half the bytes to write, and to pull through one CU at the merge): a convex
    // combination of V rows is as large as V's entries at most, round-toward-zero conversion
    // saturates instead of overflowing, and 11 bits of a value that is then weighted and rounded
    // to bf16's 8 leave the result where fp32 partial results put it (bf16 ones do not).
    //   part[k4][lane]         4 x fp16;   then [2][64] fp32: reference and the query's normaliser
    constexpr int kK4 = kDBlocks * 4;
    const size_t block_words = (size_t)kK4 * 128 + 128;            // one (unit, range, query block)
    float* const my_part = p.partials + ((size_t)unit * S + split) * WQ * block_words;
    // 8-byte store of four consecutive output features of my query (the row block of my wavefront)
    uint16_t* const out_row = p.out + ((size_t)qi[0] * p.H + qh[0]) * D + half * 4;
    auto store_out = [&](int k4, float4 acc, float inv) __attribute__((always_inline)) {
        if (!qvalid[0]) return;
        f32x2_t lo = {acc.x * inv, acc.y * inv}, hi = {acc.z * inv, acc.w * inv};
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2_t));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2_t));
        *reinterpret_cast<uint2*>(out_row + (k4 >> 2) * 32 + (k4 & 3) * 8) = w;
    };
    __syncthreads();
    const bool keep_mine = may_keep && s_last;   // (the same in every wavefront)
    constexpr int kKept = kDBlocks * 4 / WK;
    uint2 kept[kKept];
    float kept_m = 0.f, kept_l = 0.f;
    float* const lds_f = reinterpret_cast<float*>(&sm_union);
    float* const o_s = lds_f;                                        // [kCells][kK4][64][4]
    float* const ml_s = o_s + (size_t)kCells * kK4 * 256;            // [kCells][2][64]
    auto item_of = [&](int k4) __attribute__((always_inline)) {
        return make_float4(oacc[0][k4 >> 2][(k4 & 3) * 4], oacc[0][k4 >> 2][(k4 & 3) * 4 + 1],
                           oacc[0][k4 >> 2][(k4 & 3) * 4 + 2], oacc[0][k4 >> 2][(k4 & 3) * 4 + 3]);
    };
    float* const part_ml = my_part + (size_t)wqw * block_words + (size_t)kK4 * 128;
    uint2* const part_o = reinterpret_cast<uint2*>(my_part + (size_t)wqw * block_words) + lane;
    // (`mine`: the item's number among those of this wavefront, a literal)
    auto store_part = [&](int k4, int mine, float4 acc, float inv) __attribute__((always_inline)) {
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(acc.x * inv, acc.y * inv));
        w.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(acc.z * inv, acc.w * inv));
        kept[mine] = w;
        if (!keep_mine) part_o[k4 * 64] = w;
    };
    // (a query whose keys in this range are all masked has normaliser and output 0)
    auto whole_normaliser = [&](float mine) __attribute__((always_inline)) {
        const auto r2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(mine), __float_as_uint(mine), false, false);
        return __uint_as_float(r2[0]) + __uint_as_float(r2[1]);
    };
    if constexpr (WK == 1) {
        // my row block is in my registers
        const float l_all = whole_normaliser(l_run[0]);
        if (S == 1) {
            const float inv = __builtin_amdgcn_rcpf(l_all);
#pragma unroll
            for (int k4 = 0; k4 < kK4; ++k4) store_out(k4, item_of(k4), inv);
        } else {
            const float inv = l_all > 0.f ? __builtin_amdgcn_rcpf(l_all) : 0.f;
#pragma unroll
            for (int k4 = 0; k4 < kK4; ++k4) store_part(k4, k4, item_of(k4), inv);
            kept_m = m_run[0];
            kept_l = l_all;
            if (!keep_mine) {
                part_ml[lane] = m_run[0];
                part_ml[64 + lane] = l_all;
            }
        }
    } else {
        // Every wavefront drops its cell; wavefront (row block q, key group j) then merges items
        // j * kK4 / WK .. of row block q over the WK cells (a lone wavefront issues a vector
        // instruction every 6 to 10 clocks: the merge is shared by all, not left to one per row
        // block).  Its own items it takes from registers, which is why the fold is written once
        // per key group: register arrays want literal indices.
        {
            const int cell = wk * WQ + wqw;
            float4* dst = reinterpret_cast<float4*>(o_s) + (size_t)cell * kK4 * 64 + lane;
#pragma unroll
            for (int k4 = 0; k4 < kK4; ++k4) dst[k4 * 64] = item_of(k4);
            ml_s[cell * 128 + lane] = m_run[0];
            ml_s[cell * 128 + 64 + lane] = l_run[0];
        }
        __syncthreads();
        float f[WK];
        float big = -INFINITY, lsum = 0.f;
#pragma unroll
        for (int o = 0; o < WK; ++o) {
            f[o] = ml_s[(o * WQ + wqw) * 128 + lane];
            big = fmaxf(big, f[o]);
        }
        const float ref = (big == -INFINITY) ? 0.f : big;
#pragma unroll
        for (int o = 0; o < WK; ++o) {
            f[o] = __builtin_amdgcn_exp2f(f[o] - ref);
            lsum = fmaf(ml_s[(o * WQ + wqw) * 128 + 64 + lane], f[o], lsum);
        }
        constexpr int kMine = kK4 / WK;
        float4 acc[kMine];
        auto fold = [&](auto j_c) __attribute__((always_inline)) {
            constexpr int J = decltype(j_c)::value;
#pragma unroll
            for (int i = 0; i < kMine; ++i) {
                const float4 mine = item_of(J * kMine + i);
                acc[i] = make_float4(mine.x * f[J], mine.y * f[J], mine.z * f[J], mine.w * f[J]);
            }
#pragma unroll
            for (int o = 0; o < WK; ++o) {
                if (o == J) continue;
                const float4* src = reinterpret_cast<const float4*>(o_s) + ((size_t)(o * WQ + wqw) * kK4 + J * kMine) * 64 + lane;
#pragma unroll
                for (int i = 0; i < kMine; ++i) {
                    const float4 v = src[i * 64];
                    acc[i].x = fmaf(v.x, f[o], acc[i].x); acc[i].y = fmaf(v.y, f[o], acc[i].y);
                    acc[i].z = fmaf(v.z, f[o], acc[i].z); acc[i].w = fmaf(v.w, f[o], acc[i].w);
                }
            }
        };
        if (wk == 0) fold(std::integral_constant<int, 0>{});
        else if (wk == 1) fold(std::integral_constant<int, 1>{});
        else if constexpr (WK > 2) {
            if (wk == 2) fold(std::integral_constant<int, 2>{});
            else fold(std::integral_constant<int, 3>{});
        }
        static_assert(WK == 2 || WK == 4, "one fold per key group");
        const float l_all = whole_normaliser(lsum);
        if (S == 1) {
            const float inv = __builtin_amdgcn_rcpf(l_all);
#pragma unroll
            for (int i = 0; i < kMine; ++i) store_out(wk * kMine + i, acc[i], inv);
        } else {
            const float inv = l_all > 0.f ? __builtin_amdgcn_rcpf(l_all) : 0.f;
#pragma unroll
            for (int i = 0; i < kMine; ++i) store_part(wk * kMine + i, i, acc[i], inv);
            kept_m = big;
            kept_l = l_all;
            if (wk == 0 && !keep_mine) {
                part_ml[lane] = big;
                part_ml[64 + lane] = l_all;
            }
        }
    }
    if (S == 1) { ATTN_STAMP_FLUSH(); return; }
    ATTN_STAMP(21);

    // See whether we are the last range of this unit to finish.  The partial results must be
    // visible to that workgroup, which runs on another CU.  When all ranges of a unit run on one
    // XCD they meet in its L2: every wavefront waits until the L2 has acknowledged its own stores
    // (the vector memory counter counts stores too; a workgroup-scope fence would not wait, since
    // within a workgroup the CU's own cache is the meeting point), and only then does the barrier
    // let thread 0 count the workgroup as arrived.  Otherwise the L2 has to be written back.
    // (Sharing the merge among the S workgroups of a unit -- count arrivals, poll a bounded
    // number of times, claim a slice -- was tried: the polling costs more than the one CU's
    // memory pipeline it saves, and workgroups that wait hold CUs that a later batch needs.)
    if (!keep_mine) {
        if (p.share_l2) wait_vmcnt<0>();
        else __threadfence();
        __syncthreads();
        if (tid == 0) {
            const uint32_t arrived = atomicAdd(&p.counters[unit], 1u);
            s_last = (arrived == (uint32_t)(S - 1));
        }
        __syncthreads();
        ATTN_STAMP(22);
        if (!s_last) { ATTN_STAMP_FLUSH(); return; }
    }
    // The partial results are read from the L2, not from whatever this CU's own cache holds for
    // those addresses: every load of the merge is a device-scope atomic load, which goes past the
    // CU's cache.  (A device-scope acquire fence would do as well, but its invalidate also sweeps
    // the XCD's L2 for lines of memory that is not kept coherent there: the first load behind it
    // came back after 5 us, where the same load before it took 0.4, and the K/V tiles of every
    // workgroup still running on the XCD went with it.)
    if (!p.share_l2) __threadfence();
    ATTN_STAMP(23);

    // Merge the ranges of the unit.  One workgroup pulls S partial results through one CU's memory
    // pipeline, so what matters is how many loads are in flight, how few round trips there are,
    // and that the arithmetic around them stays small.  Wavefront (row block q, key group j) merges
    // features j * kK4 / WK .. of row block q: a lane keeps one query for the whole merge (its row
    // of `out` and its weights are worked out once, in registers), requests all S values of a
    // batch of items before it touches the first (NS = S, rounded up beyond 8; the surplus
    // requests repeat the last range), and requests the first batch before the statistics, which
    // are a round trip of their own.
    const float* const row_part = p.partials + (size_t)unit * S * WQ * block_words + (size_t)wqw * block_words;
    const size_t range_words = (size_t)WQ * block_words;
    auto merge_ranges = [&](auto ns_c) __attribute__((always_inline)) {
        constexpr int NS = decltype(ns_c)::value;
        constexpr int kItems = kK4 / WK;                                 // per lane
        const bool keeping = NS <= kKeepUpTo && keep_mine;               // (never, for most numbers of ranges: their copies carry no code for it)
        // items requested together: the largest power of two with at most 32 requests (of 8 bytes)
        // per lane; the partial results were written a long time ago and come from memory, so a
        // batch is a full round trip
        constexpr int kFit = NS <= 2 ? 16 : (NS <= 4 ? 8 : (NS <= 8 ? 4 : 2));
        constexpr int kBatch = kFit < kItems ? kFit : kItems;
        static_assert(kItems % kBatch == 0, "batches");
        // (addresses: a uniform base per range and item, plus the lane)
        const uint2* const src = reinterpret_cast<const uint2*>(row_part) + (wk * kItems) * 64;
        uint2 v[2][kBatch][NS];   // two batches: one being summed, one in flight
        auto request = [&](int k0, uint2 (&dst)[kBatch][NS]) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < NS; ++r) {
                if (keeping && r == split) {   // (mine are in `kept`)
#pragma unroll
                    for (int j = 0; j < kBatch; ++j) dst[j][r] = make_uint2(0u, 0u);
                    continue;
                }
                // (a base in scalar registers plus the lane: an address pair per range in vector
                // registers, which is what the compiler makes of an atomic load otherwise, does not fit)
                const uint2* const src_r = static_cast<const uint2*>(scalar_pointer(src + (size_t)min(r, S - 1) * (range_words / 2) + k0 * 64));
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const unsigned long long two = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(src_r + j * 64 + lane),
                                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    dst[j][r] = make_uint2((uint32_t)two, (uint32_t)(two >> 32));
                }
            }
        };
        request(0, v[0]);
        ATTN_STAMP(25);
        float f[NS];
        float lsum = 0.f;
        {
            const float* ml = row_part + (size_t)kK4 * 128;
            float mv[NS], lv[NS];
#pragma unroll
            for (int r = 0; r < NS; ++r) {
                const float* m = static_cast<const float*>(scalar_pointer(ml + (size_t)min(r, S - 1) * range_words));
                const bool mine = keeping && r == split;
                // (asked for whether mine or not: under a condition every one of these loads
                // would be a block of its own with a wait at its end)
                const float m_r = __hip_atomic_load(m + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float l_r = __hip_atomic_load(m + 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                mv[r] = mine ? kept_m : m_r;
                lv[r] = mine ? kept_l : l_r;
            }
            float big = -INFINITY;
#pragma unroll
            for (int r = 0; r < NS; ++r) big = fmaxf(big, mv[r]);
            const float ref = (big == -INFINITY) ? 0.f : big;
#pragma unroll
            // a range's weight: its normaliser brought to the common reference (its output is
            // normalised already)
            for (int r = 0; r < NS; ++r) {
                f[r] = r < S ? __builtin_amdgcn_exp2f(mv[r] - ref) * lv[r] : 0.f;
                lsum += f[r];
            }
        }
        const float inv = __builtin_amdgcn_rcpf(lsum);
        ATTN_STAMP(26);
        // The merged rows leave through LDS (the rings, free by now).  A lane holds four features
        // of its query per item: stored from there, an instruction writes 16 bytes to each of 32
        // rows of `out`, and a row is put together from eight such instructions -- one CU's
        // memory pipeline took 8 us over the 64 KB of a unit that way.  Each wavefront drops its
        // items into a tile of its own, [32 queries][its 16 * kItems bytes of a row] (rows 16
        // bytes apart from a multiple of 256: two-way bank conflicts at worst), and writes the
        // tile out with 16 bytes per lane, whole runs of a row per instruction.
        constexpr int kSpanBytes = 16 * kItems;
        constexpr int kStageRow = kSpanBytes + 16;
        static_assert(8 * 32 * kStageRow <= (int)sizeof(Rings<D, kCells>), "the rows of eight wavefronts fit the rings");
        char* const stage = reinterpret_cast<char*>(lds_f) + (size_t)wave * 32 * kStageRow;
        auto stage_out = [&](int item, float4 acc) __attribute__((always_inline)) {
            f32x2_t lo = {acc.x * inv, acc.y * inv}, hi = {acc.z * inv, acc.w * inv};
            uint2 w;
            w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2_t));
            w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2_t));
            *reinterpret_cast<uint2*>(stage + col * kStageRow + item * 16 + half * 8) = w;
        };
        auto sum_up = [&](int k0, const uint2 (&src_v)[kBatch][NS]) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int r = 0; r < NS; ++r) {
                    uint2 item = src_v[j][r];
                    if constexpr (kItems == kBatch) {
                        if (keeping && r == split) item = kept[j];
                    }
                    const half2_t lo = __builtin_bit_cast(half2_t, item.x), hi = __builtin_bit_cast(half2_t, item.y);
                    acc.x = fmaf((float)lo[0], f[r], acc.x); acc.y = fmaf((float)lo[1], f[r], acc.y);
                    acc.z = fmaf((float)hi[0], f[r], acc.z); acc.w = fmaf((float)hi[1], f[r], acc.w);
                }
                stage_out(k0 + j, acc);
            }
        };
        if constexpr (kItems == kBatch) {
            sum_up(0, v[0]);
        } else {
            static_assert(kItems % (2 * kBatch) == 0, "pairs of batches");
#pragma unroll 1
            for (int k0 = 0; k0 < kItems; k0 += 2 * kBatch) {
                request(k0 + kBatch, v[1]);
                sum_up(k0, v[0]);
                if (k0 + 2 * kBatch < kItems) request(k0 + 2 * kBatch, v[0]);
                sum_up(k0 + kBatch, v[1]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // my lanes' items are in the tile (nobody else's are)
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int kLanesPerRow = kSpanBytes / 16, kRowsPerPass = 64 / kLanesPerRow, kPasses = 32 / kRowsPerPass;
        const int chunk = lane % kLanesPerRow;
#pragma unroll
        for (int pass = 0; pass < kPasses; ++pass) {
            const int row = pass * kRowsPerPass + lane / kLanesPerRow;
            const int qrow = qb * kUnitRows + wqw * 32 + row;
            if (qrow < rows) {
                const int node = (int)fast_div((uint32_t)qrow, p.by_G);
                const uint4 v16 = *reinterpret_cast<const uint4*>(stage + row * kStageRow + chunk * 16);
                uint16_t* const dst = p.out + ((size_t)node * p.H + (g * p.G + (qrow - node * p.G))) * D;
                *reinterpret_cast<uint4*>(reinterpret_cast<char*>(dst) + wk * kSpanBytes + chunk * 16) = v16;
            }
        }
    };
    // (one copy of the merge per number of ranges up to 8: a surplus request costs as much of the
    // CU's memory pipeline as a real one)
    switch (S) {
        case 2: merge_ranges(std::integral_constant<int, 2>{}); break;
        case 3: merge_ranges(std::integral_constant<int, 3>{}); break;
        case 4: merge_ranges(std::integral_constant<int, 4>{}); break;
        case 5: merge_ranges(std::integral_constant<int, 5>{}); break;
        case 6: merge_ranges(std::integral_constant<int, 6>{}); break;
        case 7: merge_ranges(std::integral_constant<int, 7>{}); break;
        case 8: merge_ranges(std::integral_constant<int, 8>{}); break;
        case 9: case 10: merge_ranges(std::integral_constant<int, 10>{}); break;
        case 11: case 12: merge_ranges(std::integral_constant<int, 12>{}); break;
        default: merge_ranges(std::integral_constant<int, kMaxSplits>{}); break;
    }
    if (tid == 0) atomicExch(&p.counters[unit], 0u);   // every range has been counted: ready for the next call
    ATTN_STAMP(24);
    ATTN_STAMP_FLUSH();
}

}  // namespace

int g_splits_override = 0;  // tuning hooks, 0 = automatic
int g_wq_override = 0;
int g_keep_own = 1;   // test hook: 0 = every partial result goes through memory
int g_uneven_override = -1, g_short_weight_override = 1, g_long_weight_override = 1;   // -1 = automatic, 0 = equal ranges only, m > 0 = m short ranges
int g_long_tiles_override = -1;   // -1 = automatic, 0 = long ranges in proportion to their unit's tiles, L > 0 = long ranges of L tiles

static AttnSchedule work_out_attn_schedule(int P, int n, int H, int Hk, int D);

// The schedule depends on the prefix only through its number of tiles, and a caller that decodes
// asks for the same few shapes over and over (the prefix grows by a handful of tokens per step):
// the last sixteen answers are kept.  Working one out takes 0.5 us, or 12 to 17 us where a launch
// is played through, which is what an eager caller would otherwise pay per layer.
AttnSchedule plan_attn_schedule(int P, int n, int H, int Hk, int D) {
    struct Kept {
        int key[12];
        AttnSchedule schedule;
        bool valid = false;
    };
    static std::mutex guard;
    static Kept kept[16];
    static unsigned next = 0;
    const int key[12] = {(P + kKeyTile - 1) / kKeyTile, n, H, Hk, D, g_splits_override, g_wq_override, g_uneven_override,
                         g_short_weight_override, g_long_weight_override, g_long_tiles_override, 0};
    {
        std::lock_guard<std::mutex> lock(guard);
        for (const Kept& k : kept)
            if (k.valid && std::equal(key, key + 12, k.key)) return k.schedule;
    }
    const AttnSchedule s = work_out_attn_schedule(P, n, H, Hk, D);
    std::lock_guard<std::mutex> lock(guard);
    Kept& slot = kept[next++ % 16];
    std::copy(key, key + 12, slot.key);
    slot.schedule = s;
    slot.valid = true;
    return s;
}

static AttnSchedule work_out_attn_schedule(int P, int n, int H, int Hk, int D) {
    AttnSchedule s;
    const int G = H / Hk;
    const int rows = G * n;
    const int prefix_tiles = (P + kKeyTile - 1) / kKeyTile;
    const int tiles = prefix_tiles + (n + kKeyTile - 1) / kKeyTile;
    // Two choices: row blocks per workgroup (wq; the 8 / wq wavefronts left over share the key
    // tiles of a round) and key ranges per unit.  One workgroup fits on a CU at a time, so a
    // launch runs in batches of 256 workgroups (the compute units of an MI355X, eight XCDs of 32;
    // the workspace query has no device to ask, and the cost figures below were measured on that
    // part and no other); a workgroup costs its rounds -- dearer the more
    // tiles a round copies -- plus a fixed prologue/epilogue plus, with more than one range, the
    // hand-over of the partial results and their merge (figures in tenths of a microsecond,
    // chosen against the measured times of every (wq, ranges) pair at the head shapes of the
    // paper's models: trees of 16 to 768 nodes under prefixes of 512 to 20000 keys, and trees of
    // 128 to 768 nodes under prefixes of 128 to 1024; the pair chosen is on average 0.7 % slower
    // than the best pair measured, 16 % at worst and 11 % next).  A wq beyond what the rows of a
    // KV head fill is never considered; a smaller one is, because it multiplies the units when
    // there are few KV heads.
    const int wq_cover = rows <= 64 ? 2 : (rows <= 128 ? 4 : 8);
    constexpr long kFixed = 70, kHandOver = 20;   // prologue and epilogue of a workgroup; partial results handed over and merged at all
    constexpr long kFixedShort = 120;             // the same of a short range that runs behind another (measured at the lengths below)
    double long_share = 0.;                       // of the ranges of two sizes chosen, before rounding to 64ths
    long best = -1;
    s.wq = wq_cover;
    s.splits = 1;
    s.short_ranges = 0;
    s.short_weight = s.long_weight = 1;
    for (int wq = 2; wq <= wq_cover; wq *= 2) {
        if (g_wq_override > 0 && wq != std::min(g_wq_override, wq_cover)) continue;
        const int wk = kMaxCells / wq;
        const int units = Hk * ((rows + 32 * wq - 1) / (32 * wq));
        const long round_cost = wk == 1 ? 9 : (wk == 2 ? 10 : 14);
        const int max_splits = std::min(kMaxSplits, std::max(1, tiles / wk));
        for (int cand = 1; cand <= max_splits; ++cand) {
            if (g_splits_override > 0 && cand != std::min(g_splits_override, max_splits)) continue;
            const long batches = ((long)units * cand + 255) / 256;
            const long rounds = (tiles + cand * wk - 1) / (cand * wk);
            const long apiece = kFixed + (cand > 1 ? kHandOver + 2 * cand * wq : 0);
            long cost = batches * (rounds * round_cost + apiece);
            // Where the units of a KV head differ in their tree tiles (short prefixes under large
            // trees: 5 to 28 tiles) and there are more workgroups than compute units, whole batches
            // of the longest workgroup are far from what happens: the dispatcher hands the next
            // workgroup to whichever CU is free.  Then the launch is played through for one XCD
            // -- its units, in the order the kernel takes them (range-major, last row block
            // first), on its 32 CUs.
            const int per_head = (rows + 32 * wq - 1) / (32 * wq), units_per_xcd = (units + 7) / 8;
            const long jobs = (long)units_per_xcd * cand;
            if (per_head > 1 && jobs > 32 && jobs <= 160) {
                long free_at[32] = {};   // a min-heap of the times at which the CUs fall free
                long end = 0;
                for (int turn = 0; turn < cand; ++turn) {
                    const int range = cand - 1 - turn;
                    for (int local = units_per_xcd - 1; local >= 0; --local) {
                        if (local >= units) continue;
                        const int qb = local % per_head;
                        const int last_row = std::min(rows - 1, qb * 32 * wq + 32 * wq - 1);
                        const long unit_tiles = prefix_tiles + last_row / G / kKeyTile + 1;
                        const long length = unit_tiles * (range + 1) / cand - unit_tiles * range / cand;
                        std::pop_heap(free_at, free_at + 32, std::greater<long>());
                        free_at[31] += (length + wk - 1) / wk * round_cost + apiece;
                        end = std::max(end, free_at[31]);
                        std::push_heap(free_at, free_at + 32, std::greater<long>());
                    }
                }
                cost = end;
            }
            if (best < 0 || cost < best) { best = cost; s.wq = wq; s.splits = cand; s.short_ranges = 0; s.short_weight = s.long_weight = 1; }
        }
        // Ranges of two sizes.  When the units leave CUs over but too few for another range each
        // (192 units: 64), equal ranges either leave those CUs idle or come in several batches,
        // each workgroup of which pays the fixed part again.  Instead every unit gets `longs`
        // long ranges, whose workgroups are dispatched first and take a CU each, and one short
        // range; the short ones run k in a row on the CUs left over, and the weights are chosen so
        // that both kinds end together.  One prologue, epilogue and partial result per long range instead
        // of one per batch.
        if (g_splits_override > 0 || g_uneven_override >= 0) continue;
        for (int longs = 1; longs * units < 256 && longs + 1 <= kMaxSplits; ++longs) {
            const int left_over = 256 - longs * units;
            const long k = (units + left_over - 1) / left_over;
            if (k < 2) continue;   // (k = 1 is longs + 1 equal ranges in one batch)
            if (k > 3) break;      // (measured: with more short ranges in a row their fixed parts eat the gain)
            // the long ranges' share f of a unit's tiles for which a long workgroup takes as long
            // as k short ones in a row, in 64ths
            const long all_rounds = (tiles + wk - 1) / wk, merge = kHandOver + 2 * (longs + 1) * wq;
            const long num = k * all_rounds * round_cost + k * kFixedShort - kFixed - merge, den = all_rounds * round_cost * (1 + k * longs);
            const int long_w = (int)((64 * num + den / 2) / den), short_w = 64 - longs * long_w;
            if (long_w < 1 || short_w < 1) continue;
            const long rounds_long = ((long)tiles * long_w / 64 + wk) / wk, rounds_short = ((long)tiles * short_w / 64 + wk) / wk;
            if (rounds_short < 16) continue;   // (measured: short ranges of a few rounds are all fixed part, which the model overrates evenly but not here)
            const long cost = std::max(rounds_long * round_cost + kFixed + merge, k * (rounds_short * round_cost + kFixedShort));
            if (cost < best) {
                best = cost; s.wq = wq; s.splits = longs + 1; s.short_ranges = 1; s.short_weight = short_w; s.long_weight = long_w;
                long_share = (double)num / (double)den;
            }
        }
    }
    if (s.short_ranges == 0) long_share = 0.;   // (an equal candidate of another wq won in the end)
    if (g_uneven_override > 0 && g_uneven_override < s.splits) {
        s.short_ranges = g_uneven_override;
        s.short_weight = g_short_weight_override;
        s.long_weight = g_long_weight_override;
        long_share = 0.;
    }
    s.query_blocks = (rows + 32 * s.wq - 1) / (32 * s.wq);
    // Long ranges of one length: the long share of the tiles of the average unit (the units of a
    // KV head differ in their tree tiles; with one unit per head nothing changes).  Taken by
    // itself from eight units per head on: the short ranges then differ in length from unit to
    // unit, workgroups are dispatched in the order of the units, and with few units per head the
    // same compute unit gets several of the longest short ranges in a row (two units per head,
    // three short ranges in a row: 12 % slower than shares in proportion).
    s.long_tiles = 0;
    if (s.short_ranges > 0 && g_long_tiles_override != 0 && (g_long_tiles_override > 0 || s.query_blocks >= 8)) {
        long tree_tiles = 0;
        for (int qb = 0; qb < s.query_blocks; ++qb) {
            const int last_row = std::min(rows - 1, qb * 32 * s.wq + 32 * s.wq - 1);
            tree_tiles += last_row / G / kKeyTile + 1;
        }
        const double mean_tiles = (double)prefix_tiles + (double)tree_tiles / s.query_blocks;
        if (long_share <= 0.)
            long_share = (double)s.long_weight / (double)(s.short_ranges * s.short_weight + (s.splits - s.short_ranges) * s.long_weight);
        s.long_tiles = g_long_tiles_override > 0 ? g_long_tiles_override : (int)(mean_tiles * long_share + 0.5);
        if (s.long_tiles < 1) s.long_tiles = 0;
    }
    const int units = Hk * s.query_blocks;
    const size_t block_words = (size_t)(D / 32) * 4 * 128 + 128;   // one (unit, range, query block): fp16 output, fp32 statistics
    s.workspace_bytes = s.splits > 1 ? (size_t)units * s.splits * s.wq * block_words * sizeof(float) : 0;
    if (s.workspace_bytes < 256) s.workspace_bytes = 256;
    return s;
}

int launch_tree_attn_mfma_bf16(const void* q, const void* k_cache, const void* v_cache,
                               const void* k_tree, const void* v_tree, const TreePlan& plan,
                               int P, int cap, int n, int H, int Hk, int D, void* out,
                               const AttnSchedule& sched, float* workspace, uint32_t* counters,
                               bool units_share_l2, hipStream_t stream, const int32_t* prefix_lens,
                               int seq_kv_heads) {
    MfmaParams p;
    p.q = static_cast<const uint16_t*>(q);
    p.k_cache = static_cast<const uint16_t*>(k_cache);
    p.v_cache = static_cast<const uint16_t*>(v_cache);
    p.k_tree = static_cast<const uint16_t*>(k_tree);
    p.v_tree = static_cast<const uint16_t*>(v_tree);
    p.out = static_cast<uint16_t*>(out);
    p.anc = plan.anc_words;
    p.words_per_row = plan.words_per_row;
    p.P_bound = P; p.cap = cap; p.n = n; p.H = H; p.Hk = Hk; p.G = H / Hk;
    p.prefix_lens = prefix_lens;
    p.by_seq_kv_heads = make_fast_div((uint32_t)(seq_kv_heads > 0 ? seq_kv_heads : Hk));
    p.query_blocks = sched.query_blocks;
    p.prefix_tiles_bound = (P + kKeyTile - 1) / kKeyTile;
    p.splits = sched.splits;
    p.partials = workspace;
    p.counters = counters;
    p.scale_log2 = 1.4426950408889634f / sqrtf((float)D);
    p.share_l2 = units_share_l2 ? 1 : 0;
    const int units = Hk * sched.query_blocks;
    p.by_units_per_xcd = make_fast_div((uint32_t)((units + 7) >> 3));
    p.by_query_blocks = make_fast_div((uint32_t)sched.query_blocks);
    p.by_G = make_fast_div((uint32_t)(H / Hk));
    p.short_ranges = sched.short_ranges;
    p.short_weight = sched.short_weight;
    p.long_weight = sched.long_weight;
    p.long_tiles = prefix_lens ? 0 : sched.long_tiles;   // (lengths that differ by sequence: each unit's own proportion)
    p.by_short_ranges = make_fast_div((uint32_t)std::max(sched.short_ranges, 1));
    p.keep_own = g_keep_own;
    p.by_weights = make_fast_div((uint32_t)(sched.short_ranges * sched.short_weight + (sched.splits - sched.short_ranges) * sched.long_weight));
    if (units > kAttnMaxCounters) return SEQ_ERR_SHAPE;
    const int unit_groups = (units + 7) / 8;
    const dim3 grid((unsigned)(unit_groups * 8 * sched.splits)), block(512);
#define SEQ_ATTN_LAUNCH(DD, WQ_, WK_)                                                             \
    hipLaunchKernelGGL((tree_attn_mfma_kernel<DD, WQ_, WK_>), grid, block, 0, stream, p)
    if (D == 64) {
        if (sched.wq == 2) SEQ_ATTN_LAUNCH(64, 2, 4);
        else if (sched.wq == 4) SEQ_ATTN_LAUNCH(64, 4, 2);
        else SEQ_ATTN_LAUNCH(64, 8, 1);
    } else {
        if (sched.wq == 2) SEQ_ATTN_LAUNCH(128, 2, 4);
        else if (sched.wq == 4) SEQ_ATTN_LAUNCH(128, 4, 2);
        else SEQ_ATTN_LAUNCH(128, 8, 1);
    }
#undef SEQ_ATTN_LAUNCH
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}

}  // namespace seqtree

// Tuning hooks (not part of the public header): force the number of key-axis ranges and the
// number of query blocks per workgroup (2, 4 or 8).
#ifdef SEQTREE_STAMPS
extern "C" void seqtree_internal_read_attn_wg_times(long long* out, int count) {
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(seqtree::g_attn_wg_times), sizeof(long long) * 2 * count);
}
extern "C" int seqtree_internal_read_attn_stamps(long long* out) {
    int count = 0;
    (void)hipMemcpyFromSymbol(&count, HIP_SYMBOL(seqtree::g_attn_stamp_count), sizeof(int));
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(seqtree::g_attn_stamps), sizeof(long long) * 128);
    return count;
}
#endif
extern "C" void seqtree_internal_set_attn_splits(int splits) { seqtree::g_splits_override = splits; }
extern "C" void seqtree_internal_set_attn_wq(int wq) { seqtree::g_wq_override = wq; }
// The schedule the library would take: {wq, ranges, short ranges, short weight, long weight}.
extern "C" void seqtree_internal_attn_schedule(int P, int n, int H, int Hk, int D, int* five) {
    const seqtree::AttnSchedule s = seqtree::plan_attn_schedule(P, n, H, Hk, D);
    five[0] = s.wq; five[1] = s.splits; five[2] = s.short_ranges; five[3] = s.short_weight; five[4] = s.long_weight;
}
extern "C" int seqtree_internal_attn_range_start(int tiles, int range, int ranges, int short_ranges, int short_weight, int long_weight,
                                                 int long_tiles) {
    const seqtree::FastDiv by = seqtree::make_fast_div((uint32_t)(short_ranges * short_weight + (ranges - short_ranges) * long_weight));
    const seqtree::FastDiv by_short = seqtree::make_fast_div((uint32_t)(short_ranges > 0 ? short_ranges : 1));
    return seqtree::range_start(tiles, range, ranges, short_ranges, short_weight, long_weight, long_tiles, by, by_short);
}
// the length the library would give the long ranges (0: in proportion to each unit's tiles)
extern "C" int seqtree_internal_attn_long_tiles(int P, int n, int H, int Hk, int D) {
    return seqtree::plan_attn_schedule(P, n, H, Hk, D).long_tiles;
}
extern "C" void seqtree_internal_set_attn_long_tiles(int mode) { seqtree::g_long_tiles_override = mode; }
extern "C" void seqtree_internal_set_attn_keep_own(int on) { seqtree::g_keep_own = on; }
extern "C" void seqtree_internal_set_attn_uneven(int short_ranges, int short_weight, int long_weight) {
    seqtree::g_uneven_override = short_ranges;
    seqtree::g_short_weight_override = short_weight > 0 ? short_weight : 1;
    seqtree::g_long_weight_override = long_weight > 0 ? long_weight : 1;
}
// the prologue's division by multiplication, evaluated on the host (for the tests)
extern "C" uint32_t seqtree_internal_fast_div(uint32_t n, uint32_t d) { return seqtree::fast_div(n, seqtree::make_fast_div(d)); }
