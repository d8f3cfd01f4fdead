// Row-wise tree attention: one workgroup per (tree token, query head), fp32 arithmetic.
// This is the fp32 path of seq_tree_attn (the toy configuration, where the work is tiny and
// accuracy to 1e-5 is what matters).  The bf16 path lives in tree_attn_mfma.hip.
//
// For output row (i, h) the workgroup walks the key axis [cache rows 0..P) ++ [tree rows 0..n)
// in chunks, keeps a running maximum and normaliser (online softmax) and a running weighted sum
// of value rows.  A tree row j contributes only if bit j of row i of the ancestor-or-self
// bitset is set; every other key is skipped, so its weight is exactly zero and its memory is
// never read.
#include "seq_internal.h"
#include "tree_attn_kernels.h"

namespace seqtree {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 1024;  // keys per online-softmax step

__device__ __forceinline__ float block_reduce_max(float v, float* red) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, red[w]);
    return r;
}

__device__ __forceinline__ float block_reduce_sum(float v, float* red) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float r = red[0];
    for (int w = 1; w < kThreads / 64; ++w) r += red[w];
    return r;
}

template <int D>
__global__ __launch_bounds__(kThreads) void tree_attn_rowwise_f32(
    const float* __restrict__ q, const float* __restrict__ k_cache, const float* __restrict__ v_cache,
    const float* __restrict__ k_tree, const float* __restrict__ v_tree,
    const uint32_t* __restrict__ anc, int words_per_row, int P_bound, int cap, int n, int H, int Hk,
    float* __restrict__ out, const int32_t* __restrict__ prefix_lens, int seq_kv_heads) {
    __shared__ float qs[D];
    __shared__ float sc[kChunk];
    __shared__ float red[kThreads / 64];
    __shared__ float acc_s[kThreads];

    const int i = blockIdx.x / H;
    const int h = blockIdx.x % H;
    const int g = h / (H / Hk);
    // (a batch whose sequences differ in prefix length: that of this KV head's sequence)
    const int P = prefix_lens ? min(max(prefix_lens[g / seq_kv_heads], 0), P_bound) : P_bound;
    const int tid = threadIdx.x;
    const float scale = 1.0f / sqrtf((float)D);
    const uint32_t* anc_row = anc + (size_t)i * words_per_row;

    if (tid < D) qs[tid] = q[((size_t)i * H + h) * D + tid];
    __syncthreads();

    constexpr int kSlices = kThreads / D;  // value columns are spread over D threads per slice
    const int col = tid % D;
    const int slice = tid / D;

    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
    const int total = P + n;
    for (int base = 0; base < total; base += kChunk) {
        const int len = min(kChunk, total - base);
        // scores of this chunk
        float cmax = -INFINITY;
        for (int x = tid; x < len; x += kThreads) {
            const int key = base + x;
            const float* kr = nullptr;
            if (key < P) {
                kr = k_cache + ((size_t)g * cap + key) * D;
            } else {
                const int j = key - P;
                if ((anc_row[j >> 5] >> (j & 31)) & 1u) kr = k_tree + ((size_t)j * Hk + g) * D;
            }
            float s = -INFINITY;
            if (kr) {
                float dot = 0.f;
#pragma unroll 8
                for (int c = 0; c < D; c += 4) {
                    const float4 kv = *reinterpret_cast<const float4*>(kr + c);
                    dot = fmaf(qs[c], kv.x, dot);
                    dot = fmaf(qs[c + 1], kv.y, dot);
                    dot = fmaf(qs[c + 2], kv.z, dot);
                    dot = fmaf(qs[c + 3], kv.w, dot);
                }
                s = dot * scale;
            }
            sc[x] = s;
            cmax = fmaxf(cmax, s);
        }
        cmax = block_reduce_max(cmax, red);
        if (cmax == -INFINITY) { __syncthreads(); continue; }  // nothing visible in this chunk
        const float m_new = fmaxf(m_run, cmax);
        const float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
        float csum = 0.f;
        for (int x = tid; x < len; x += kThreads) {
            const float s = sc[x];
            const float p = (s == -INFINITY) ? 0.f : expf(s - m_new);
            sc[x] = p;
            csum += p;
        }
        csum = block_reduce_sum(csum, red);  // also orders the sc[] writes before the reads below
        l_run = l_run * alpha + csum;
        m_run = m_new;
        acc *= alpha;
        for (int x = slice; x < len; x += kSlices) {
            const float p = sc[x];
            if (p == 0.f) continue;  // masked (or underflowed) keys: never read their value row
            const int key = base + x;
            const float* vr = (key < P) ? v_cache + ((size_t)g * cap + key) * D
                                        : v_tree + ((size_t)(key - P) * Hk + g) * D;
            acc = fmaf(p, vr[col], acc);
        }
        __syncthreads();
    }
    acc_s[tid] = acc;
    __syncthreads();
    if (tid < D) {
        float o = 0.f;
        for (int s = 0; s < kSlices; ++s) o += acc_s[s * D + tid];
        out[((size_t)i * H + h) * D + tid] = o / l_run;
    }
}

}  // namespace

int launch_tree_attn_rowwise_f32(const float* q, const float* k_cache, const float* v_cache,
                                 const float* k_tree, const float* v_tree, const TreePlan& plan,
                                 int P, int cap, int n, int H, int Hk, int D, float* out,
                                 hipStream_t stream, const int32_t* prefix_lens, int seq_kv_heads) {
    if (seq_kv_heads <= 0) seq_kv_heads = Hk;
    const dim3 grid((unsigned)(n * H)), block(kThreads);
    if (D == 64)
        hipLaunchKernelGGL(tree_attn_rowwise_f32<64>, grid, block, 0, stream, q, k_cache, v_cache,
                           k_tree, v_tree, plan.anc_words, plan.words_per_row, P, cap, n, H, Hk, out, prefix_lens, seq_kv_heads);
    else
        hipLaunchKernelGGL(tree_attn_rowwise_f32<128>, grid, block, 0, stream, q, k_cache, v_cache,
                           k_tree, v_tree, plan.anc_words, plan.words_per_row, P, cap, n, H, Hk, out, prefix_lens, seq_kv_heads);
    return hipGetLastError() == hipSuccess ? SEQ_OK : SEQ_ERR_HIP;
}

}  // namespace seqtree
