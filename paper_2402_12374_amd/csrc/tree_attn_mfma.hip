// bf16 tree attention on the gfx950 matrix cores.
//
// One workgroup (4 wavefronts) owns a block of 128 query rows of one KV head -- a query row is
// a (tree token i, head h of the group) pair, numbered rho = i * G + hh -- and a contiguous
// range of 64-key tiles of the key axis [cache rows 0..P) ++ [tree rows 0..n).  Each wavefront
// keeps 32 query rows.  Per tile the workgroup stages K (row-major) and V (transposed, keys in
// the order the matrix instruction consumes them) in LDS, shared by all its queries; each
// wavefront then forms the TRANSPOSED score tile S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so
// that a lane owns one query column: the running maximum, the normaliser and the rescaling of
// the output are per-lane scalars and the only cross-lane step is one exchange with lane^32.
// The accumulator layout of S^T is, value for value, the B-operand layout of O^T += V^T P^T, so
// probabilities go from registers straight back into the matrix unit.
//
// Masking (which keys a tree token may see: cache rows below prefix_len, itself and its
// ancestors) is a bit test on one 32-bit word of the ancestor-or-self bitset per 32 keys; a
// masked score is replaced by -inf, so its weight is exactly zero.
//
// When the key axis is cut into several ranges, every workgroup leaves (max, normaliser,
// unnormalised output) in the workspace and the last one to arrive for a query block merges
// them by log-sum-exp; no workgroup ever waits for another.
#include "seq_internal.h"
#include "tree_attn_kernels.h"

namespace seqtree {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int kThreads = 256;
constexpr int kWaves = 4;

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
    int query_blocks;     // per KV head
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

template <int D>
struct Smem {
    static constexpr int kKStride = D + 8;          // bf16 elements per K row (16 B pad)
    static constexpr int kVStride = kKeyTile + 8;   // bf16 elements per V^T row
    uint16_t k[2][kKeyTile * kKStride];
    uint16_t vt[2][D * kVStride];
};

// Position, inside its 32-key block, at which key (4 * quad) is stored in a V^T row so that the
// 8 keys one lane feeds to one matrix instruction are contiguous: key = (2m+a)*8 + half*4 + b
// goes to m*16 + half*8 + a*4 + b.
__device__ __forceinline__ int vt_pos_of_quad(int quad) {
    const int kb = quad >> 3, rem = quad & 7;
    const int m = rem >> 2, a = (rem >> 1) & 1, half = rem & 1;
    return kb * 32 + m * 16 + half * 8 + a * 4;
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void tree_attn_mfma_kernel(const MfmaParams p) {
    constexpr int kKSteps = D / 16;        // contraction steps of Q K^T
    constexpr int kDBlocks = D / 32;       // 32-row blocks of O^T
    constexpr int kChunks = D / 8;         // 16-byte chunks per K/V row
    constexpr int kKLoads = kKeyTile * kChunks / kThreads;
    constexpr int kVItems = 16 * kChunks;  // (key quad, chunk) pairs per tile
    constexpr int kPartialWords = kDBlocks * 16 + 2;
    using SM = Smem<D>;
    __shared__ __attribute__((aligned(16))) SM sm;
    __shared__ int s_last;

    const int S = p.splits;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, idx = bid >> 3;
    const int unit = (idx / S) * 8 + xcd;   // consecutive workgroup ids go to different XCDs:
    const int split = idx % S;              // keep every split of a unit on one XCD (one L2)
    if (unit >= p.Hk * p.query_blocks) return;
    const int g = unit / p.query_blocks, qb = unit % p.query_blocks;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int rows = p.G * p.n;
    const int wave_row0 = qb * kQueryBlock + wave * 32;
    const bool wave_valid = wave_row0 < rows;
    const int qrow = wave_row0 + col;
    const bool qvalid = qrow < rows;
    const int qi = qvalid ? qrow / p.G : 0;
    const int qh = qvalid ? g * p.G + qrow % p.G : 0;

    // key tiles of this workgroup
    const int last_row = min(rows - 1, qb * kQueryBlock + kQueryBlock - 1);
    const int i_max = last_row / p.G;                 // tree rows beyond i_max are masked for all
    const int tree_tiles = i_max / kKeyTile + 1;
    const int total_tiles = p.prefix_tiles + tree_tiles;
    const int t_begin = (int)((long long)total_tiles * split / S);
    const int t_end = (int)((long long)total_tiles * (split + 1) / S);

    // Q fragments (B operand): lane holds query `col`, features ks*16 + half*8 .. +7
    bf16x8_t qf[kKSteps];
    {
        const uint16_t* qp = p.q + ((size_t)qi * p.H + qh) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < kKSteps; ++ks) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (qvalid) v = *reinterpret_cast<const uint4*>(qp + ks * 16);
            qf[ks] = __builtin_bit_cast(bf16x8_t, v);
        }
    }

    f32x16_t oacc[kDBlocks];
#pragma unroll
    for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[b][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    uint4 kreg[kKLoads];
    uint4 vreg[4];
    const int v_item = tid;                       // at most one (quad, chunk) item per thread
    const bool v_active = v_item < kVItems;
    const int v_quad = v_item & 15, v_chunk = v_item >> 4;

    auto load_tile = [&](int t) {
        const bool is_prefix = t < p.prefix_tiles;
        const int key0 = is_prefix ? t * kKeyTile : (t - p.prefix_tiles) * kKeyTile;
        const int limit = is_prefix ? p.P : p.n;
        const uint16_t* kbase = is_prefix ? p.k_cache + (size_t)g * p.cap * D : p.k_tree + (size_t)g * D;
        const uint16_t* vbase = is_prefix ? p.v_cache + (size_t)g * p.cap * D : p.v_tree + (size_t)g * D;
        const size_t row_stride = is_prefix ? (size_t)D : (size_t)p.Hk * D;
#pragma unroll
        for (int k = 0; k < kKLoads; ++k) {
            const int item = tid + k * kThreads;
            const int row = item / kChunks, chunk = item % kChunks;
            const int key = key0 + row;
            kreg[k] = make_uint4(0, 0, 0, 0);
            if (key < limit)
                kreg[k] = *reinterpret_cast<const uint4*>(kbase + (size_t)key * row_stride + chunk * 8);
        }
        if (v_active) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int key = key0 + v_quad * 4 + b;
                vreg[b] = make_uint4(0, 0, 0, 0);  // rows past the valid range must read as zero
                if (key < limit)
                    vreg[b] = *reinterpret_cast<const uint4*>(vbase + (size_t)key * row_stride + v_chunk * 8);
            }
        }
    };

    auto store_tile = [&](int buf) {
#pragma unroll
        for (int k = 0; k < kKLoads; ++k) {
            const int item = tid + k * kThreads;
            const int row = item / kChunks, chunk = item % kChunks;
            *reinterpret_cast<uint4*>(&sm.k[buf][row * SM::kKStride + chunk * 8]) = kreg[k];
        }
        if (v_active) {
            const int pos = vt_pos_of_quad(v_quad);
            const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&vreg[0]);
            const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&vreg[1]);
            const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&vreg[2]);
            const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&vreg[3]);
#pragma unroll
            for (int dd = 0; dd < 8; ++dd) {
                const int w = dd >> 1;
                uint32_t lo, hi;
                if (dd & 1) {
                    lo = (w0[w] >> 16) | (w1[w] & 0xFFFF0000u);
                    hi = (w2[w] >> 16) | (w3[w] & 0xFFFF0000u);
                } else {
                    lo = (w0[w] & 0xFFFFu) | (w1[w] << 16);
                    hi = (w2[w] & 0xFFFFu) | (w3[w] << 16);
                }
                *reinterpret_cast<uint2*>(&sm.vt[buf][(v_chunk * 8 + dd) * SM::kVStride + pos]) =
                    make_uint2(lo, hi);
            }
        }
    };

    if (t_begin < t_end) load_tile(t_begin);
    for (int t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        store_tile(buf);
        __syncthreads();
        if (t + 1 < t_end) load_tile(t + 1);
        if (!wave_valid) continue;

        // S^T = K Q^T for the two 32-key halves of the tile
        f32x16_t sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
            const uint16_t* krow = &sm.k[buf][(kb * 32 + col) * SM::kKStride + half * 8];
#pragma unroll
            for (int ks = 0; ks < kKSteps; ++ks) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(krow + ks * 16);
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[kb], 0, 0, 0);
            }
        }

        // visibility words: bit x of mask[kb] <=> key kb*32+x of this tile is visible to my query
        uint32_t mask[2];
        if (t < p.prefix_tiles) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int left = p.P - (t * kKeyTile + kb * 32);
                mask[kb] = left >= 32 ? 0xFFFFFFFFu : (left <= 0 ? 0u : ((1u << left) - 1u));
            }
        } else {
            const int tt = t - p.prefix_tiles;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int word = tt * 2 + kb;
                mask[kb] = (qvalid && word < p.words_per_row)
                               ? p.anc[(size_t)qi * p.words_per_row + word] : 0u;
            }
        }

        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int x = (r >> 2) * 8 + half * 4 + (r & 3);
                const float s = ((mask[kb] >> x) & 1u) ? sacc[kb][r] * p.scale_log2 : -INFINITY;
                sacc[kb][r] = s;
                mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - ref);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = __builtin_amdgcn_exp2f(sacc[kb][r] - ref);
                sacc[kb][r] = e;
                psum += e;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[b][r] *= alpha;

        // O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                uint4 pw;
                pw.x = pack_bf16(sacc[kb][m * 8 + 0], sacc[kb][m * 8 + 1]);
                pw.y = pack_bf16(sacc[kb][m * 8 + 2], sacc[kb][m * 8 + 3]);
                pw.z = pack_bf16(sacc[kb][m * 8 + 4], sacc[kb][m * 8 + 5]);
                pw.w = pack_bf16(sacc[kb][m * 8 + 6], sacc[kb][m * 8 + 7]);
                const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, pw);
#pragma unroll
                for (int b = 0; b < kDBlocks; ++b) {
                    const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(
                        &sm.vt[buf][(b * 32 + col) * SM::kVStride + kb * 32 + m * 16 + half * 8]);
                    oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[b], 0, 0, 0);
                }
            }
    }

    auto write_out = [&](const f32x16_t* o, float l_lane) {
        const float l_tot = l_lane + __shfl_xor(l_lane, 32);
        if (!qvalid) return;
        const float inv = 1.0f / l_tot;
        uint16_t* op = p.out + ((size_t)qi * p.H + qh) * D;
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int d0 = b * 32 + rq * 8 + half * 4;
                uint2 w;
                w.x = pack_bf16(o[b][rq * 4 + 0] * inv, o[b][rq * 4 + 1] * inv);
                w.y = pack_bf16(o[b][rq * 4 + 2] * inv, o[b][rq * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(op + d0) = w;
            }
    };

    if (S == 1) {
        if (wave_valid) write_out(oacc, l_run);
        return;
    }

    // leave this range's partial result, then see whether we are the last range to finish
    if (wave_valid) {
        float* dst = p.partials + (((size_t)unit * S + split) * kWaves + wave) * kPartialWords * 64 + lane;
        dst[0] = m_run;
        dst[64] = l_run;
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[(2 + b * 16 + r) * 64] = oacc[b][r];
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t arrived = atomicAdd(&p.counters[unit], 1u);
        s_last = (arrived == (uint32_t)(S - 1));
        if (s_last) atomicExch(&p.counters[unit], 0u);  // ready for the next call
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (!wave_valid) return;

    const float* src0 = p.partials + (((size_t)unit * S) * kWaves + wave) * kPartialWords * 64 + lane;
    const size_t split_stride = (size_t)kWaves * kPartialWords * 64;
    float m_all = -INFINITY;
    for (int s = 0; s < S; ++s) m_all = fmaxf(m_all, src0[s * split_stride]);
    const float ref = (m_all == -INFINITY) ? 0.f : m_all;
    float l_all = 0.f;
#pragma unroll
    for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[b][r] = 0.f;
    for (int s = 0; s < S; ++s) {
        const float* src = src0 + s * split_stride;
        const float w = __builtin_amdgcn_exp2f(src[0] - ref);
        l_all += src[64] * w;
#pragma unroll
        for (int b = 0; b < kDBlocks; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[b][r] += src[(2 + b * 16 + r) * 64] * w;
    }
    write_out(oacc, l_all);
}

}  // namespace

int g_splits_override = 0;  // tuning hook, 0 = automatic

AttnSchedule plan_attn_schedule(int P, int n, int H, int Hk, int D) {
    AttnSchedule s;
    const int G = H / Hk;
    const int rows = G * n;
    s.query_blocks = (rows + kQueryBlock - 1) / kQueryBlock;
    const int units = Hk * s.query_blocks;
    const int prefix_tiles = (P + kKeyTile - 1) / kKeyTile;
    int splits = 256 / (units > 0 ? units : 1);
    if (g_splits_override > 0) splits = g_splits_override;
    if (splits > prefix_tiles + 1) splits = prefix_tiles + 1;
    if (splits > 32) splits = 32;
    if (splits < 1) splits = 1;
    s.splits = splits;
    const size_t words = (size_t)(D / 32) * 16 + 2;
    s.workspace_bytes = splits > 1 ? (size_t)units * splits * kWaves * words * 64 * sizeof(float) : 0;
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
    if (D == 64)
        hipLaunchKernelGGL(tree_attn_mfma_kernel<64>, grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL(tree_attn_mfma_kernel<128>, grid, block, 0, stream, p);
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}

}  // namespace seqtree

// Tuning hook (not part of the public header): force the number of key-axis ranges.
extern "C" void seqtree_internal_set_attn_splits(int splits) { seqtree::g_splits_override = splits; }
