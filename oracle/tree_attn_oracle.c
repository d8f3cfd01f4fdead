/*
 * CPU checker for tree-masked attention.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may call this; it exists so the tests, the smoke check and the benchmark's CPU
 * baseline can compare the HIP kernels with a plain definition.
 *
 * What is computed.  The paper only says that the target model scores all tokens of the
 * speculated tree together, in one forward pass (Sec. 1), and that the tree root stands for
 * the current prefix (Sec. 2.1).  For the attention layer of that forward
 * pass this means: tree token i sees the whole prefix KV cache, its ancestors in the tree,
 * and itself -- nothing else.  Written out, for query head h with KV head g = h / (H/Hk):
 *
 *     keys(i) = { cache row t : 0 <= t < P }  u  { tree row j : j is i or an ancestor of i }
 *     s_x     = <q[i,h,:], k_x[g,:]> / sqrt(d)                          x in keys(i)
 *     w_x     = exp(s_x - max s) / sum_x exp(s_x - max s)
 *     out[i,h,:] = sum_x w_x * v_x[g,:]
 *
 * Keys outside keys(i) are never touched, so their weight is exactly zero.
 *
 * Arithmetic is fp64 throughout.  Inputs arrive as float, which holds every bf16 and fp32
 * value exactly, and are widened element by element.  One thread, no tiling, no reordering:
 * the loops below are the definition.
 *
 * Layouts (row-major): q, out [n][H][d]; k_cache, v_cache [Hk][cap][d] with the first P rows
 * of each head valid; k_tree, v_tree [n][Hk][d]; parent [n] with parent[0] = -1 and
 * 0 <= parent[i] < i.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* One output row.  w_prefix (P entries) and w_tree (n entries) may be NULL; when given they
 * receive the softmax weights (w_tree[j] = 0.0 for every tree row not in keys(i)). */
int oracle_tree_attn_row(const float* q, const float* k_cache, const float* v_cache,
                         const float* k_tree, const float* v_tree, const int32_t* parent,
                         int32_t P, int32_t cap, int32_t n, int32_t H, int32_t Hk, int32_t d,
                         int32_t i, int32_t h, double* out_row, double* w_prefix, double* w_tree)
{
    if (n < 1 || H < 1 || Hk < 1 || H % Hk != 0 || d < 1 || P < 0 || P > cap) return -1;
    if (i < 0 || i >= n || h < 0 || h >= H) return -1;
    const int32_t G = H / Hk;
    const int32_t g = h / G;
    const double scale = 1.0 / sqrt((double)d);
    const float* qv = q + ((size_t)i * H + h) * d;

    /* membership of tree rows: walk from i up to the root */
    unsigned char* member = (unsigned char*)calloc((size_t)n, 1);
    double* s_pre = (double*)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
    double* s_tree = (double*)malloc(sizeof(double) * (size_t)n);
    if (!member || !s_pre || !s_tree) { free(member); free(s_pre); free(s_tree); return -2; }
    for (int32_t j = i; j >= 0; j = parent[j]) member[j] = 1;

    double smax = -INFINITY;
    for (int32_t t = 0; t < P; ++t) {
        const float* kv = k_cache + ((size_t)g * cap + t) * d;
        double acc = 0.0;
        for (int32_t c = 0; c < d; ++c) acc += (double)qv[c] * (double)kv[c];
        s_pre[t] = acc * scale;
        if (s_pre[t] > smax) smax = s_pre[t];
    }
    for (int32_t j = 0; j < n; ++j) {
        if (!member[j]) continue;
        const float* kv = k_tree + ((size_t)j * Hk + g) * d;
        double acc = 0.0;
        for (int32_t c = 0; c < d; ++c) acc += (double)qv[c] * (double)kv[c];
        s_tree[j] = acc * scale;
        if (s_tree[j] > smax) smax = s_tree[j];
    }

    double denom = 0.0;
    for (int32_t t = 0; t < P; ++t) { s_pre[t] = exp(s_pre[t] - smax); denom += s_pre[t]; }
    for (int32_t j = 0; j < n; ++j)
        if (member[j]) { s_tree[j] = exp(s_tree[j] - smax); denom += s_tree[j]; }

    for (int32_t c = 0; c < d; ++c) out_row[c] = 0.0;
    for (int32_t t = 0; t < P; ++t) {
        const double w = s_pre[t] / denom;
        const float* vv = v_cache + ((size_t)g * cap + t) * d;
        for (int32_t c = 0; c < d; ++c) out_row[c] += w * (double)vv[c];
        if (w_prefix) w_prefix[t] = w;
    }
    for (int32_t j = 0; j < n; ++j) {
        if (!member[j]) { if (w_tree) w_tree[j] = 0.0; continue; }
        const double w = s_tree[j] / denom;
        const float* vv = v_tree + ((size_t)j * Hk + g) * d;
        for (int32_t c = 0; c < d; ++c) out_row[c] += w * (double)vv[c];
        if (w_tree) w_tree[j] = w;
    }
    free(member); free(s_pre); free(s_tree);
    return 0;
}

/* Every row: out [n][H][d] in fp64. */
int oracle_tree_attn(const float* q, const float* k_cache, const float* v_cache,
                     const float* k_tree, const float* v_tree, const int32_t* parent,
                     int32_t P, int32_t cap, int32_t n, int32_t H, int32_t Hk, int32_t d,
                     double* out)
{
    if (n < 1 || parent[0] != -1) return -1;
    for (int32_t i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i) return -1;
    for (int32_t i = 0; i < n; ++i)
        for (int32_t h = 0; h < H; ++h) {
            int rc = oracle_tree_attn_row(q, k_cache, v_cache, k_tree, v_tree, parent, P, cap, n,
                                          H, Hk, d, i, h, out + ((size_t)i * H + h) * d, NULL, NULL);
            if (rc) return rc;
        }
    return 0;
}
