// bf16 tree attention on the gfx950 matrix cores.
//
// Work split.  A "unit" is a block of 128*R query rows of one KV head -- a query row is a
// (tree token i, head hh of the group) pair, numbered rho = i * G + hh -- and one workgroup of
// four wavefronts owns a unit together with a contiguous range of 64-key tiles of the key axis
// [cache rows 0..P) ++ [tree rows 0..n).  Each wavefront keeps R blocks of 32 query rows
// (R = 2 when a KV head has many query rows, which halves the LDS traffic per matrix
// instruction; R = 1 otherwise).
//
// Data path.  K and V tiles go from global memory straight into LDS (global_load_lds_dwordx4,
// 16 bytes per lane, no register staging) into a ring of kStages tile buffers, several tiles
// ahead of the one being consumed, so that the HBM/L2 latency of a tile is covered by the work
// on the tiles before it.  Both tiles are stored row-major; 16-byte chunks are XOR-swizzled
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
// unnormalised output) in the workspace and the last one to arrive for a unit merges them by
// log-sum-exp; no workgroup ever waits for another.
#include <type_traits>

#include "seq_internal.h"
#include "tree_attn_kernels.h"

namespace seqtree {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kStages = 4;          // tile buffers in the LDS ring
constexpr int kAhead = kStages - 1; // tiles in flight beyond the one being consumed
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
    int P, cap, n, H, Hk, G;
    int query_blocks;     // units per KV head
    int prefix_tiles;     // ceil(P / 64)
    int splits;
    float* partials;
    uint32_t* counters;
    float scale_log2;     // log2(e) / sqrt(D)
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// 16 bytes per lane from global memory into LDS at lds_base + lane * 16 (lds_base uniform).
__device__ __forceinline__ void async_copy16(const void* gptr, uint32_t lds_base) {
    uint32_t saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved)
        : "v"(gptr), "s"(lds_base)
        : "memory");
}

// 4 bytes per lane into LDS at lds_base + lane * 4.
__device__ __forceinline__ void async_copy4(const void* gptr, uint32_t lds_base) {
    uint32_t saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\t"
        "s_mov_b32 m0, %2\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dword %1, off\n\t"
        "s_mov_b32 m0, %0"
        : "=&s"(saved)
        : "v"(gptr), "s"(lds_base)
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

template <int D>
struct Smem {
    static constexpr int kTileElems = kKeyTile * D;   // bf16 elements per K (or V) tile
    uint16_t k[kStages][kTileElems];
    uint16_t v[kStages][kTileElems];
};

// Visibility words of a tree tile travel through the same ring as K and V: lane l of a
// wavefront fetches word (l / 32) of the tile for query (l % 32) of each of its R blocks.
template <int R>
struct MaskRing {
    uint32_t w[kStages][kWaves][R][64];
};

// Phase timestamps of workgroup 0 (100 MHz wall clock), compiled in with -DSEQTREE_STAMPS only.
#ifdef SEQTREE_STAMPS
__device__ long long g_attn_stamps[128];
__device__ int g_attn_stamp_count;
#define ATTN_STAMP_RESET() do { if (blockIdx.x == 0 && threadIdx.x == 0) g_attn_stamp_count = 0; } while (0)
#define ATTN_STAMP(id) do { if (blockIdx.x == 0 && threadIdx.x == 0 && g_attn_stamp_count < 63) { \
    g_attn_stamps[2 * g_attn_stamp_count] = (id); g_attn_stamps[2 * g_attn_stamp_count + 1] = wall_clock64(); ++g_attn_stamp_count; } } while (0)
#else
#define ATTN_STAMP_RESET() do {} while (0)
#define ATTN_STAMP(id) do {} while (0)
#endif

template <int D, int R>
__global__ __launch_bounds__(kThreads, 1) void tree_attn_mfma_kernel(const MfmaParams p) {
    constexpr int kKSteps = D / 16;        // contraction steps of Q K^T
    constexpr int kDBlocks = D / 32;       // 32-row blocks of O^T
    constexpr int kChunks = D / 8;         // 16-byte chunks per K/V row
    constexpr int kRowBytes = D * 2;
    constexpr int kRowsPerCopy = 64 / kChunks;               // rows one wave-wide copy covers
    constexpr int kCopies = kKeyTile / kRowsPerCopy / kWaves; // copies per wavefront per tile
    constexpr int kLoadsPerTile = 2 * kCopies + R;           // K, V and visibility words, per lane
    constexpr int kPartialWords = kDBlocks * 16 + 2;
    constexpr int kUnitRows = 128 * R;
    using SM = Smem<D>;
    __shared__ __attribute__((aligned(1024))) SM sm;
    __shared__ __attribute__((aligned(256))) MaskRing<R> mr;
    __shared__ int s_last;

    ATTN_STAMP_RESET();
    ATTN_STAMP(0);
    const int S = p.splits;
    const int bid = blockIdx.x;
    // Consecutive workgroup ids go to consecutive XCDs, each with its own L2.  Give every XCD a
    // contiguous run of units: all key ranges of a unit, and all units of a KV head, then share
    // one L2, which holds that head's K and V for all of them.
    const int xcd = bid & 7, idx = bid >> 3;
    const int total_units = p.Hk * p.query_blocks;
    const int units_per_xcd = (total_units + 7) >> 3;
    const int local = idx / S, split = idx % S;
    const int unit = xcd * units_per_xcd + local;
    if (local >= units_per_xcd || unit >= total_units) return;
    const int g = unit / p.query_blocks, qb = unit % p.query_blocks;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int rows = p.G * p.n;
    int qi[R], qh[R];
    bool qvalid[R], blk_valid[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row0 = qb * kUnitRows + (wave * R + r) * 32;
        blk_valid[r] = row0 < rows;
        const int qrow = row0 + col;
        qvalid[r] = qrow < rows;
        qi[r] = qvalid[r] ? qrow / p.G : 0;
        qh[r] = qvalid[r] ? g * p.G + qrow % p.G : 0;
    }
    const bool wave_valid = blk_valid[0];

    // key tiles of this workgroup
    const int last_row = min(rows - 1, qb * kUnitRows + kUnitRows - 1);
    const int i_max = last_row / p.G;                 // tree rows beyond i_max are masked for all
    const int tree_tiles = i_max / kKeyTile + 1;
    const int total_tiles = p.prefix_tiles + tree_tiles;
    const int t_begin = (int)((long long)total_tiles * split / S);
    const int t_end = (int)((long long)total_tiles * (split + 1) / S);

    const uint32_t k_lds = lds_address(&sm.k[0][0]);
    const uint32_t v_lds = lds_address(&sm.v[0][0]);
    const uint32_t m_lds = lds_address(&mr.w[0][0][0][0]);
    constexpr uint32_t kTileBytes = SM::kTileElems * 2;

    // one tile: every lane moves kCopies 16-byte chunks of K and of V (and R visibility words)
    auto issue_tile = [&](int t) {
        const int buf = (t - t_begin) % kStages;
        const bool is_prefix = t < p.prefix_tiles;
        const int key0 = is_prefix ? t * kKeyTile : (t - p.prefix_tiles) * kKeyTile;
        const int limit = is_prefix ? p.P : p.n;
        const uint16_t* kbase = is_prefix ? p.k_cache + (size_t)g * p.cap * D : p.k_tree + (size_t)g * D;
        const uint16_t* vbase = is_prefix ? p.v_cache + (size_t)g * p.cap * D : p.v_tree + (size_t)g * D;
        const size_t row_stride = is_prefix ? (size_t)D : (size_t)p.Hk * D;
#pragma unroll
        for (int j = 0; j < kCopies; ++j) {
            const int copy = wave * kCopies + j;                 // 1 KB block of the tile
            const int row = copy * kRowsPerCopy + lane / kChunks;
            const int slot = lane % kChunks;
            // Rows past the valid keys fetch the last valid row instead: the copy count per tile
            // stays the same for every wavefront (the waits below count copies), memory past the
            // valid range is never touched, and those keys are masked anyway.
            const int key = min(key0 + row, limit - 1);
            const uint32_t block_off = (uint32_t)buf * kTileBytes + (uint32_t)copy * 1024u;
            async_copy16(kbase + (size_t)key * row_stride + ((slot ^ k_swizzle<D>(row)) * 8),
                         __builtin_amdgcn_readfirstlane(k_lds + block_off));
            async_copy16(vbase + (size_t)key * row_stride + ((slot ^ v_swizzle<D>(row)) * 8),
                         __builtin_amdgcn_readfirstlane(v_lds + block_off));
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int word = is_prefix ? 0 : (t - p.prefix_tiles) * 2 + half;
            const bool real = !is_prefix && qvalid[r] && word < p.words_per_row;
            const uint32_t* src = p.anc + (real ? (size_t)qi[r] * p.words_per_row + word : 0);
            async_copy4(src, __builtin_amdgcn_readfirstlane(m_lds + (uint32_t)(((buf * kWaves + wave) * R + r) * 256)));
        }
    };

    // start the pipeline before anything else touches memory
#pragma unroll
    for (int a = 0; a < kAhead; ++a)
        if (t_begin + a < t_end) issue_tile(t_begin + a);

    ATTN_STAMP(1);
    // Q fragments (B operand): lane holds query `col`, features ks*16 + half*8 .. +7
    bf16x8_t qf[R][kKSteps];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint16_t* qp = p.q + ((size_t)qi[r] * p.H + qh[r]) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (qvalid[r]) v = *reinterpret_cast<const uint4*>(qp + ks * 16);
            qf[r][ks] = __builtin_bit_cast(bf16x8_t, v);
        }
    }
    // Make the compiler settle these loads here.  It cannot see the copies issued in assembly,
    // and a wait for the Q fragments placed at their first use inside the tile loop would also
    // wait, on every iteration, for every copy in flight.
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qf[r][ks]));

    ATTN_STAMP(2);
    // Per-lane LDS byte offsets inside a tile, fixed for the whole kernel.  Everything else in
    // an address is a compile-time constant that goes into the instruction's offset field.
    //   K (ds_read_b128): key row `col` (+32 for the second half), chunk (2*ks + half) ^ swizzle
    //   V (transpose read): 16-lane group, lanes 4r..4r+3 address 16 features of key row r
    const int grp = lane >> 4, li = lane & 15;
    uint32_t koff[kKSteps], voff[kDBlocks];
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks)
        koff[ks] = (uint32_t)(col * kRowBytes + (((ks * 2 + half) ^ k_swizzle<D>(col)) * 16));
#pragma unroll
    for (int b = 0; b < kDBlocks; ++b) {
        const int vrow = half * 4 + (li >> 2);                 // + kb*32 + (2m+a)*8, multiples of 8
        const int feat = b * 32 + (grp & 1) * 16 + (li & 3) * 4;  // 4 features = 8 bytes
        voff[b] = (uint32_t)(vrow * kRowBytes + (((feat >> 3) ^ v_swizzle<D>(vrow)) * 16) + (feat & 7) * 2);
    }
    typedef __attribute__((address_space(3))) const char* lds_cptr;
    const lds_cptr k_base = (lds_cptr)(lds_ptr_t)&sm.k[0][0];
    const lds_cptr v_base = (lds_cptr)(lds_ptr_t)&sm.v[0][0];

    f32x16_t oacc[R][kDBlocks];
    float m_run[R], l_run[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m_run[r] = -INFINITY;
        l_run[r] = 0.f;
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) oacc[r][b][x] = 0.f;
    }

    for (int t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) % kStages;
        // my copies of tile t have landed once at most the copies of the tiles after it are
        // still in flight (copies complete in order); near the end of the range wait for all
        if (t + kAhead - 1 < t_end) wait_vmcnt<(kAhead - 1) * kLoadsPerTile>();
        else wait_vmcnt<0>();
        ATTN_STAMP(10);
        __syncthreads();   // everybody's copies of tile t are in LDS; tile t-1's buffer is free
        ATTN_STAMP(11);
        if (t + kAhead < t_end) issue_tile(t + kAhead);
        if (!wave_valid) continue;

        const lds_cptr kt = k_base + buf * kTileBytes;
        const lds_cptr vt = v_base + buf * kTileBytes;

        // S^T = K Q^T for the two 32-key halves of the tile
        f32x16_t sacc[R][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                const bf16x8_t kf = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(
                    kt + koff[ks] + kb * 32 * kRowBytes);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if (ks == 0) {
                        f32x16_t zero;
#pragma unroll
                        for (int x = 0; x < 16; ++x) zero[x] = 0.f;
                        sacc[r][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[r][ks], zero, 0, 0, 0);
                    } else {
                        sacc[r][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[r][ks], sacc[r][kb], 0, 0, 0);
                    }
                }
            }
        }

        ATTN_STAMP(12);
        // Tiles that lie wholly inside the prefix need no masking at all.
        const bool full = t < p.prefix_tiles && (t + 1) * kKeyTile <= p.P;
        if (!full) {
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    uint32_t m;   // bit x <=> key kb*32+x of this tile is visible to my query
                    if (t < p.prefix_tiles) {
                        const int left = p.P - (t * kKeyTile + kb * 32);
                        m = left >= 32 ? 0xFFFFFFFFu : (left <= 0 ? 0u : ((1u << left) - 1u));
                    } else {
                        const int word = (t - p.prefix_tiles) * 2 + kb;
                        m = (qvalid[r] && word < p.words_per_row) ? mr.w[buf][wave][r][kb * 32 + col] : 0u;
                    }
                    m >>= half * 4;
#pragma unroll
                    for (int x = 0; x < 16; ++x)   // accumulator element x holds key (x/4)*8 + half*4 + x%4
                        sacc[r][kb][x] = ((m >> ((x >> 2) * 8 + (x & 3))) & 1u) ? sacc[r][kb][x] : -INFINITY;
                }
        }

        // online softmax per query column (scores are scaled inside the exponential), and the
        // probabilities packed as the B operand of the second product
        uint32_t pw[R][2][2][4];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int x = 0; x < 16; ++x) mx = fmaxf(mx, sacc[r][kb][x]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[r], mx * p.scale_log2);
            const float ref = (m_new == -INFINITY) ? 0.f : m_new;
            const bool moved = m_new != m_run[r];
            const float alpha = __builtin_amdgcn_exp2f(m_run[r] - ref);
            m_run[r] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int x = 0; x < 16; x += 2) {
                    f32x2_t e;
                    e[0] = __builtin_amdgcn_exp2f(fmaf(sacc[r][kb][x], p.scale_log2, -ref));
                    e[1] = __builtin_amdgcn_exp2f(fmaf(sacc[r][kb][x + 1], p.scale_log2, -ref));
                    psum += e[0] + e[1];
                    pw[r][kb][x >> 3][(x & 7) >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(e, bf16x2_t));
                }
            l_run[r] = l_run[r] * alpha + psum;
            if (__any(moved)) {   // the running maximum of some column changed: rescale the output
#pragma unroll
                for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
                    for (int x = 0; x < 16; ++x) oacc[r][b][x] *= alpha;
            }
        }

        ATTN_STAMP(13);
        // O^T += V^T P^T.  Matrix step (kb, m) contracts keys kb*32 + (2m+a)*8 + half*4 + 0..3,
        // a = 0,1 -- the keys whose probabilities sit in accumulator elements 8m..8m+7.
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int b = 0; b < kDBlocks; ++b) {
                    v4i16 part[2];
#pragma unroll
                    for (int a = 0; a < 2; ++a)
                        part[a] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (v4i16 __attribute__((address_space(3)))*)(vt + voff[b] +
                                                                       (kb * 32 + (2 * m + a) * 8) * kRowBytes));
                    uint4 vw;
                    vw.x = __builtin_bit_cast(uint2, part[0]).x;
                    vw.y = __builtin_bit_cast(uint2, part[0]).y;
                    vw.z = __builtin_bit_cast(uint2, part[1]).x;
                    vw.w = __builtin_bit_cast(uint2, part[1]).y;
                    const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, vw);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        uint4 pq;
                        pq.x = pw[r][kb][m][0]; pq.y = pw[r][kb][m][1]; pq.z = pw[r][kb][m][2]; pq.w = pw[r][kb][m][3];
                        oacc[r][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            vf, __builtin_bit_cast(bf16x8_t, pq), oacc[r][b], 0, 0, 0);
                    }
                }
    }

    ATTN_STAMP(20);
    auto write_out = [&](auto rc, float l_lane) {
        constexpr int r = decltype(rc)::value;
        const float l_tot = l_lane + __shfl_xor(l_lane, 32);
        if (!qvalid[r]) return;
        const float inv = 1.0f / l_tot;
        uint16_t* op = p.out + ((size_t)qi[r] * p.H + qh[r]) * D;
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int d0 = b * 32 + rq * 8 + half * 4;
                f32x2_t lo = {oacc[r][b][rq * 4 + 0] * inv, oacc[r][b][rq * 4 + 1] * inv};
                f32x2_t hi = {oacc[r][b][rq * 4 + 2] * inv, oacc[r][b][rq * 4 + 3] * inv};
                uint2 w;
                w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2_t));
                w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2_t));
                *reinterpret_cast<uint2*>(op + d0) = w;
            }
    };

    // one query block: either the final result, or a partial result left for the merge
    const size_t block_words = (size_t)kPartialWords * 64;
    const size_t split_stride = (size_t)kWaves * R * block_words;
    auto leave = [&](auto rc) {
        constexpr int r = decltype(rc)::value;
        if (!blk_valid[r]) return;
        if (S == 1) { write_out(rc, l_run[r]); return; }
        float* dst = p.partials + ((size_t)unit * S + split) * split_stride + (size_t)(wave * R + r) * block_words + lane;
        dst[0] = m_run[r];
        dst[64] = l_run[r];
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) dst[(2 + b * 16 + x) * 64] = oacc[r][b][x];
    };
    leave(std::integral_constant<int, 0>{});
    if constexpr (R == 2) leave(std::integral_constant<int, 1>{});
    ATTN_STAMP(21);
    if (S == 1) return;

    // see whether we are the last range of this unit to finish
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t arrived = atomicAdd(&p.counters[unit], 1u);
        s_last = (arrived == (uint32_t)(S - 1));
        if (s_last) atomicExch(&p.counters[unit], 0u);  // ready for the next call
    }
    __syncthreads();
    ATTN_STAMP(22);
    if (!s_last) return;
    __threadfence();
    ATTN_STAMP(23);

    auto merge = [&](auto rc) {
        constexpr int r = decltype(rc)::value;
        if (!blk_valid[r]) return;
        const float* src0 = p.partials + (size_t)unit * S * split_stride + (size_t)(wave * R + r) * block_words + lane;
        // weights of the ranges first, then the weighted sums; every load is unconditional (ranges
        // past S re-read the last one with weight zero) so that they are all in flight together
        float w[kMaxSplits], ls[kMaxSplits];
        float m_all = -INFINITY;
#pragma unroll
        for (int s = 0; s < kMaxSplits; ++s) {
            const float* src = src0 + (size_t)min(s, S - 1) * split_stride;
            w[s] = src[0];
            ls[s] = src[64];
        }
#pragma unroll
        for (int s = 0; s < kMaxSplits; ++s) {
            if (s >= S) w[s] = -INFINITY;
            m_all = fmaxf(m_all, w[s]);
        }
        const float ref = (m_all == -INFINITY) ? 0.f : m_all;
        float l_all = 0.f;
#pragma unroll
        for (int s = 0; s < kMaxSplits; ++s) {
            w[s] = __builtin_amdgcn_exp2f(w[s] - ref);
            l_all += ls[s] * w[s];
        }
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int x = 0; x < 16; ++x) {
                float acc = 0.f;
#pragma unroll
                for (int s = 0; s < kMaxSplits; ++s)
                    acc = fmaf(src0[(size_t)min(s, S - 1) * split_stride + (2 + b * 16 + x) * 64], w[s], acc);
                oacc[r][b][x] = acc;
            }
        write_out(rc, l_all);
    };
    merge(std::integral_constant<int, 0>{});
    if constexpr (R == 2) merge(std::integral_constant<int, 1>{});
    ATTN_STAMP(24);
}

}  // namespace

int g_splits_override = 0;  // tuning hooks, 0 = automatic
int g_rblocks_override = 0;

AttnSchedule plan_attn_schedule(int P, int n, int H, int Hk, int D) {
    AttnSchedule s;
    const int G = H / Hk;
    const int rows = G * n;
    s.r_blocks = rows > 128 ? 2 : 1;
    if (g_rblocks_override > 0) s.r_blocks = g_rblocks_override;
    const int unit_rows = 128 * s.r_blocks;
    s.query_blocks = (rows + unit_rows - 1) / unit_rows;
    const int units = Hk * s.query_blocks;
    const int prefix_tiles = (P + kKeyTile - 1) / kKeyTile;
    int splits = 256 / (units > 0 ? units : 1);
    if (g_splits_override > 0) splits = g_splits_override;
    if (splits > prefix_tiles + 1) splits = prefix_tiles + 1;
    if (splits > kMaxSplits) splits = kMaxSplits;
    if (splits < 1) splits = 1;
    s.splits = splits;
    const size_t words = (size_t)(D / 32) * 16 + 2;
    s.workspace_bytes = splits > 1 ? (size_t)units * splits * kWaves * s.r_blocks * words * 64 * sizeof(float) : 0;
    if (s.workspace_bytes < 256) s.workspace_bytes = 256;
    return s;
}

int launch_tree_attn_mfma_bf16(const void* q, const void* k_cache, const void* v_cache,
                               const void* k_tree, const void* v_tree, const TreePlan& plan,
                               int P, int cap, int n, int H, int Hk, int D, void* out,
                               const AttnSchedule& sched, float* workspace, uint32_t* counters,
                               hipStream_t stream) {
    MfmaParams p;
    p.q = static_cast<const uint16_t*>(q);
    p.k_cache = static_cast<const uint16_t*>(k_cache);
    p.v_cache = static_cast<const uint16_t*>(v_cache);
    p.k_tree = static_cast<const uint16_t*>(k_tree);
    p.v_tree = static_cast<const uint16_t*>(v_tree);
    p.out = static_cast<uint16_t*>(out);
    p.anc = plan.anc_words;
    p.words_per_row = plan.words_per_row;
    p.P = P; p.cap = cap; p.n = n; p.H = H; p.Hk = Hk; p.G = H / Hk;
    p.query_blocks = sched.query_blocks;
    p.prefix_tiles = (P + kKeyTile - 1) / kKeyTile;
    p.splits = sched.splits;
    p.partials = workspace;
    p.counters = counters;
    p.scale_log2 = 1.4426950408889634f / sqrtf((float)D);
    const int units = Hk * sched.query_blocks;
    if (units > kAttnMaxCounters) return SEQ_ERR_SHAPE;
    const int unit_groups = (units + 7) / 8;
    const dim3 grid((unsigned)(unit_groups * 8 * sched.splits)), block(kThreads);
    if (D == 64) {
        if (sched.r_blocks == 2) hipLaunchKernelGGL((tree_attn_mfma_kernel<64, 2>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((tree_attn_mfma_kernel<64, 1>), grid, block, 0, stream, p);
    } else {
        if (sched.r_blocks == 2) hipLaunchKernelGGL((tree_attn_mfma_kernel<128, 2>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((tree_attn_mfma_kernel<128, 1>), grid, block, 0, stream, p);
    }
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}

}  // namespace seqtree

// Tuning hooks (not part of the public header): force the number of key-axis ranges and the
// number of 32-row query blocks per wavefront.
#ifdef SEQTREE_STAMPS
extern "C" int seqtree_internal_read_attn_stamps(long long* out) {
    int count = 0;
    (void)hipMemcpyFromSymbol(&count, HIP_SYMBOL(seqtree::g_attn_stamp_count), sizeof(int));
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(seqtree::g_attn_stamps), sizeof(long long) * 128);
    return count;
}
#endif
extern "C" void seqtree_internal_set_attn_splits(int splits) { seqtree::g_splits_override = splits; }
extern "C" void seqtree_internal_set_attn_rblocks(int r) { seqtree::g_rblocks_override = r; }
