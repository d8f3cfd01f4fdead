/*
 * Runs every entry point of the CPU checker on small inputs, edge cases included, so that the
 * test suite can execute them under AddressSanitizer and UndefinedBehaviorSanitizer (the checker
 * is what every parity claim rests on; an out-of-bounds read in it would be silent otherwise).
 * Built and run by tests/test_oracle_sanitizers.py.  Prints "ok" and exits 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_tree_attn_row(const float*, const float*, const float*, const float*, const float*, const int32_t*,
                         int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, double*, double*, double*);
int oracle_tree_attn(const float*, const float*, const float*, const float*, const float*, const int32_t*,
                     int32_t, int32_t, int32_t, int32_t, int32_t, int32_t, double*);
int oracle_verify(const float*, const float*, const int32_t*, const int32_t*, double, const float*, int32_t, int32_t,
                  int32_t*, int32_t*, double*, int32_t*, double*, double*, double*, int32_t*);
int oracle_verify_trials(int64_t, int32_t, const float*, const float*, const int32_t*, const int32_t*, double,
                         const float*, int32_t, int32_t, int32_t*, int32_t*, int32_t*);
int oracle_verify_baseline(int32_t, const float*, const float*, const int32_t*, const int32_t*, double, const float*,
                           int32_t, int32_t, int32_t*, int32_t*, double*, int32_t*, double*);
int oracle_draft_sample(const float*, const int32_t*, int32_t, int32_t, const int32_t*, double, uint64_t, uint64_t,
                        int32_t, int32_t*, double*, int32_t*);
void oracle_philox4x32_10(const uint32_t*, const uint32_t*, uint32_t*);

static uint64_t state = 88172645463325252ull;
static double unit(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (double)(state >> 11) / 9007199254740992.0; }
static float* floats(size_t n, double scale) { float* p = malloc(sizeof(float) * (n ? n : 1)); for (size_t i = 0; i < n; ++i) p[i] = (float)((unit() - 0.5) * scale); return p; }
#define CHECK(x) do { if (!(x)) { printf("failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

int main(void) {
    /* attention: GQA, a prefix shorter than the cache, a one-node tree, an empty prefix */
    {
        const int32_t n = 7, H = 4, Hk = 2, d = 16, P = 9, cap = 12;
        const int32_t parent[7] = {-1, 0, 0, 1, 1, 3, 2};
        float *q = floats((size_t)n * H * d, 2), *kc = floats((size_t)Hk * cap * d, 2), *vc = floats((size_t)Hk * cap * d, 2);
        float *kt = floats((size_t)n * Hk * d, 2), *vt = floats((size_t)n * Hk * d, 2);
        double* out = malloc(sizeof(double) * n * H * d);
        double row[16], wp[12], wt[7];
        CHECK(oracle_tree_attn(q, kc, vc, kt, vt, parent, P, cap, n, H, Hk, d, out) == 0);
        CHECK(oracle_tree_attn(q, kc, vc, kt, vt, parent, 0, cap, n, H, Hk, d, out) == 0);
        CHECK(oracle_tree_attn(q, kc, vc, kt, vt, parent, P, cap, 1, H, Hk, d, out) == 0);
        CHECK(oracle_tree_attn_row(q, kc, vc, kt, vt, parent, P, cap, n, H, Hk, d, 6, 3, row, wp, wt) == 0);
        CHECK(oracle_tree_attn_row(q, kc, vc, kt, vt, parent, P, cap, n, H, Hk, d, 7, 0, row, wp, wt) != 0);
        free(q); free(kc); free(vc); free(kt); free(vt); free(out);
    }
    /* verification: Algorithm 2 and the baselines, T > 0 and T = 0, a one-node tree, -inf logits */
    {
        const int32_t n = 6, V = 11;
        const int32_t parent[6] = {-1, 0, 0, 0, 1, 1};
        int32_t tokens[6] = {0, 3, 3, 10, 0, 7};
        float *tl = floats((size_t)n * V, 6), *dl = floats((size_t)n * V, 6), *un = floats(n, 1);
        for (int i = 0; i < n; ++i) un[i] = (float)unit();
        dl[2] = -INFINITY; tl[V + 4] = -INFINITY;
        int32_t path[6], bonus, n_dec, counters[2];
        double dec[6 * 8], binfo[8], fr[11], fd[11];
        for (int t = 0; t < 2; ++t) {
            const double T = t ? 0.0 : 0.7;
            CHECK(oracle_verify(tl, dl, tokens, parent, T, un, n, V, path, &bonus, dec, &n_dec, binfo, fr, fd, counters) == 0);
            CHECK(bonus >= 0 && bonus < V);
            CHECK(oracle_verify(tl, dl, tokens, parent, T, un, 1, V, path, &bonus, NULL, NULL, NULL, NULL, NULL, NULL) == 0);
            for (int alg = 1; alg <= 2; ++alg) {
                CHECK(oracle_verify_baseline(alg, tl, dl, tokens, parent, T, un, n, V, path, &bonus, dec, &n_dec, binfo) == 0);
                CHECK(bonus >= 0 && bonus < V && n_dec <= n);
            }
        }
        CHECK(oracle_verify_baseline(3, tl, dl, tokens, parent, 1.0, un, n, V, path, &bonus, NULL, NULL, NULL) != 0);
        int32_t plen[4], first[4], bon[4], tok4[4 * 6];
        float* un4 = floats(4 * n, 1);
        for (int i = 0; i < 4 * n; ++i) { un4[i] = (float)unit(); tok4[i] = (int32_t)(unit() * V); }
        CHECK(oracle_verify_trials(4, 1, tl, dl, tok4, parent, 0.9, un4, n, V, plen, first, bon) == 0);
        free(tl); free(dl); free(un); free(un4);
    }
    /* the drafter's draw: every token drawn, no children, -inf and NaN logits, row ids, T = 0 */
    {
        const int32_t rows = 4, V = 9, ks = 9;
        float* l = floats((size_t)rows * V, 4);
        l[1] = -INFINITY; l[V + 2] = NAN;
        const int32_t nc[4] = {9, 0, 3, 1}, ids[4] = {5, 0, 1023, 7};
        int32_t tok[4 * 9], cls[4 * 10];
        double keys[4 * 10];
        CHECK(oracle_draft_sample(l, NULL, rows, V, nc, 0.6, 1ull << 63, 12345, ks, tok, keys, cls) == 0);
        CHECK(oracle_draft_sample(l, ids, rows, V, nc, 0.0, 7, 8, ks, tok, NULL, NULL) == 0);
        const int32_t too_many[4] = {10, 0, 0, 0};
        CHECK(oracle_draft_sample(l, NULL, rows, V, too_many, 1.0, 0, 0, 10, tok, NULL, NULL) != 0);
        uint32_t c[4] = {0, 0, 0, 0}, k[2] = {0, 0}, o[4];
        oracle_philox4x32_10(c, k, o);
        CHECK(o[0] == 0x6627e8d5u);
        free(l);
    }
    printf("ok\n");
    return 0;
}
